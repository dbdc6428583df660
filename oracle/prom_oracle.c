/*
 * CPU oracle for the ternary pointwise-convolution path.  TEST INFRASTRUCTURE ONLY:
 * this file is the slow, plain definition that the HIP kernels are checked against.
 * It shares no code, header, table or helper with the HIP path, and nothing in the
 * product path may call it.
 *
 * What it follows:
 *  - Pointwise conv with ternary weights = for every pixel and output channel, the sum
 *    of the input channels whose weight is +1 minus the sum of those whose weight is -1
 *    (paper, Section 2 "Impact on Quantization Efficiency"; Section 3.1 "Pointwise
 *    Convolutions": the input is convolved directly with the ternary weights and the
 *    result is scaled per output channel afterwards; Figure 12, inference branch:
 *    convolve in low bit-width, then rescale).
 *  - Depthwise 3x3 conv with 8-bit weights between the two pointwise convs
 *    (Section 2, first paragraph; Section 3.1 "Depthwise Convolutions", Eq. 4-5).
 *    All quantisers of the paper are symmetric (Eq. 1-7 have no zero-point), so the
 *    padding value is the literal 0.
 *  - Block order expand -> depthwise -> project (Section 2; Figure 4 caption).
 *
 * The paper rescales in floating point and never states an integer form.  The integer
 * epilogue here is this build's contract (parity unpinned by the paper; pinned against
 * exact rational arithmetic in the tests):
 *     s = acc + bias[c]                              (int64)
 *     q = floor( (s*mult[c] + 2^(30+shift[c])) / 2^(31+shift[c]) )
 *       = floor( s * mult[c] * 2^-(31+shift[c]) + 1/2 )      one rounding, ties toward +inf
 *     y = min(max(q, act_min), act_max)
 *     if residual:  y = min(max(y + residual, -128), 127)
 * Preconditions: |bias| <= 2^30, 0 <= shift <= 31, 0 < mult < 2^31, so every
 * intermediate fits in int64.
 *
 * PReLU variant (the *_prelu functions; the paper's MobileNetV2 and RegNetX models replace
 * ReLU6 / ReLU by PReLU, Section 3.2, last paragraph; PReLU itself is
 * f(z) = z for z >= 0 and a_c * z for z < 0 with one learned slope a_c per channel).  The
 * real pre-activation is z = sigma_c * s with sigma_c > 0, so its sign is the sign of s, and
 * the slope folds into a second multiplier mult_neg[c] ~ a_c * mult[c] (same shift, any
 * int32 value, a slope may be negative):
 *     s = acc + bias[c]
 *     m = mult[c] if s >= 0 else mult_neg[c]
 *     q = floor( (s*m + 2^(30+shift[c])) / 2^(31+shift[c]) )
 *     y = clamp as above (+ residual as above)
 * Integer form again this build's contract (parity unpinned by the paper; pinned in the tests
 * against the plain requantisation where the two must agree, and against a float PReLU).
 *
 * Loops are plain and in definition order.  The only parallelism is an OpenMP
 * "parallel for" over pixels (each pixel's outputs are independent).
 */
#include <stdint.h>
#include <stddef.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* floor(a / b) for b > 0, written out (C's / truncates toward zero). */
static int64_t floor_div_pos(int64_t a, int64_t b)
{
    int64_t q = a / b;
    int64_t r = a % b;
    if (r != 0 && r < 0) q -= 1;
    return q;
}

/* Requantise one accumulator+bias value s. */
int64_t oracle_requant(int64_t s, int32_t mult, int32_t shift)
{
    int64_t num = s * (int64_t)mult + ((int64_t)1 << (30 + shift));
    int64_t den = (int64_t)1 << (31 + shift);
    return floor_div_pos(num, den);
}

static int8_t finish(int64_t acc, int32_t bias, int32_t mult, int32_t shift,
                     int32_t act_min, int32_t act_max, int has_res, int8_t res)
{
    int64_t s = acc + (int64_t)bias;
    int64_t q = oracle_requant(s, mult, shift);
    if (q < act_min) q = act_min;
    if (q > act_max) q = act_max;
    if (has_res) {
        q += (int64_t)res;
        if (q < -128) q = -128;
        if (q > 127) q = 127;
    }
    return (int8_t)q;
}

/* Requantise s with the multiplier chosen by its sign (PReLU). */
int64_t oracle_requant_prelu(int64_t s, int32_t mult, int32_t mult_neg, int32_t shift)
{
    int64_t m = (s >= 0) ? (int64_t)mult : (int64_t)mult_neg;
    int64_t num = s * m + ((int64_t)1 << (30 + shift));
    int64_t den = (int64_t)1 << (31 + shift);
    return floor_div_pos(num, den);
}

static int8_t finish_prelu(int64_t acc, int32_t bias, int32_t mult, int32_t mult_neg, int32_t shift,
                           int32_t act_min, int32_t act_max, int has_res, int8_t res)
{
    int64_t s = acc + (int64_t)bias;
    int64_t q = oracle_requant_prelu(s, mult, mult_neg, shift);
    if (q < act_min) q = act_min;
    if (q > act_max) q = act_max;
    if (has_res) {
        q += (int64_t)res;
        if (q < -128) q = -128;
        if (q > 127) q = 127;
    }
    return (int8_t)q;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Raw accumulators of the pointwise conv: acc[m][co] = sum_k x[m][k] * W[co][k]. */
int oracle_pw_accum(const int8_t *x, int64_t m_pixels, int cin,
                    const int8_t *w /* [cout][cin], values in {-1,0,1} */, int cout,
                    int32_t *acc /* [m][cout] */)
{
    if (!x || !w || !acc || m_pixels < 0 || cin <= 0 || cout <= 0) return -1;
    int64_t m;
#pragma omp parallel for schedule(static)
    for (m = 0; m < m_pixels; ++m) {
        for (int co = 0; co < cout; ++co) {
            int64_t a = 0;
            for (int k = 0; k < cin; ++k)
                a += (int64_t)x[m * cin + k] * (int64_t)w[(int64_t)co * cin + k];
            acc[m * cout + co] = (int32_t)a;
        }
    }
    return 0;
}

/* Pointwise 1x1 conv, NHWC int8 in and out. */
int oracle_pw_conv(const int8_t *x, int n, int h, int wd, int cin,
                   const int8_t *w /* [cout][cin], values in {-1,0,1} */, int cout,
                   const int32_t *bias, const int32_t *mult, const int32_t *shift,
                   int32_t act_min, int32_t act_max,
                   const int8_t *residual /* [n][h][w][cout] or NULL */,
                   int8_t *y /* [n][h][w][cout] */)
{
    if (!x || !w || !bias || !mult || !shift || !y) return -1;
    if (n <= 0 || h <= 0 || wd <= 0 || cin <= 0 || cout <= 0) return -1;
    for (int64_t i = 0; i < (int64_t)cout * cin; ++i)
        if (w[i] < -1 || w[i] > 1) return -2;
    int64_t m_pixels = (int64_t)n * h * wd;
    int64_t m;
#pragma omp parallel for schedule(static)
    for (m = 0; m < m_pixels; ++m) {
        for (int co = 0; co < cout; ++co) {
            int64_t acc = 0;
            for (int k = 0; k < cin; ++k) {
                int8_t wk = w[(int64_t)co * cin + k];
                if (wk == 1) acc += (int64_t)x[m * cin + k];
                else if (wk == -1) acc -= (int64_t)x[m * cin + k];
            }
            y[m * cout + co] = finish(acc, bias[co], mult[co], shift[co], act_min, act_max,
                                      residual != NULL,
                                      residual ? residual[m * cout + co] : 0);
        }
    }
    return 0;
}

/* Pointwise 1x1 conv with the PReLU requantisation. */
int oracle_pw_conv_prelu(const int8_t *x, int n, int h, int wd, int cin,
                         const int8_t *w /* [cout][cin], values in {-1,0,1} */, int cout,
                         const int32_t *bias, const int32_t *mult, const int32_t *mult_neg,
                         const int32_t *shift, int32_t act_min, int32_t act_max,
                         const int8_t *residual /* [n][h][w][cout] or NULL */,
                         int8_t *y /* [n][h][w][cout] */)
{
    if (!x || !w || !bias || !mult || !mult_neg || !shift || !y) return -1;
    if (n <= 0 || h <= 0 || wd <= 0 || cin <= 0 || cout <= 0) return -1;
    for (int64_t i = 0; i < (int64_t)cout * cin; ++i)
        if (w[i] < -1 || w[i] > 1) return -2;
    int64_t m_pixels = (int64_t)n * h * wd;
    int64_t m;
#pragma omp parallel for schedule(static)
    for (m = 0; m < m_pixels; ++m) {
        for (int co = 0; co < cout; ++co) {
            int64_t acc = 0;
            for (int k = 0; k < cin; ++k) {
                int8_t wk = w[(int64_t)co * cin + k];
                if (wk == 1) acc += (int64_t)x[m * cin + k];
                else if (wk == -1) acc -= (int64_t)x[m * cin + k];
            }
            y[m * cout + co] = finish_prelu(acc, bias[co], mult[co], mult_neg[co], shift[co],
                                            act_min, act_max, residual != NULL,
                                            residual ? residual[m * cout + co] : 0);
        }
    }
    return 0;
}

/* Depthwise 3x3 conv, pad 1, stride 1 or 2, NHWC, weights [3][3][c]. */
int oracle_dw_conv(const int8_t *x, int n, int h, int wd, int c,
                   const int8_t *w /* [3][3][c] */, int stride,
                   const int32_t *bias, const int32_t *mult, const int32_t *shift,
                   int32_t act_min, int32_t act_max,
                   int8_t *y /* [n][ho][wo][c] */)
{
    if (!x || !w || !bias || !mult || !shift || !y) return -1;
    if (n <= 0 || h <= 0 || wd <= 0 || c <= 0 || (stride != 1 && stride != 2)) return -1;
    int ho = (h + 2 - 3) / stride + 1;
    int wo = (wd + 2 - 3) / stride + 1;
    int64_t rows = (int64_t)n * ho;
    int64_t row;
#pragma omp parallel for schedule(static)
    for (row = 0; row < rows; ++row) {
        int in_ = (int)(row / ho);
        int oy = (int)(row % ho);
        for (int ox = 0; ox < wo; ++ox) {
            for (int ch = 0; ch < c; ++ch) {
                int64_t acc = 0;
                for (int i = 0; i < 3; ++i) {
                    for (int j = 0; j < 3; ++j) {
                        int iy = oy * stride + i - 1;
                        int ix = ox * stride + j - 1;
                        if (iy < 0 || iy >= h || ix < 0 || ix >= wd) continue; /* zero pad */
                        int64_t xv = x[(((int64_t)in_ * h + iy) * wd + ix) * c + ch];
                        int64_t wv = w[(i * 3 + j) * c + ch];
                        acc += xv * wv;
                    }
                }
                y[(((int64_t)in_ * ho + oy) * wo + ox) * c + ch] =
                    finish(acc, bias[ch], mult[ch], shift[ch], act_min, act_max, 0, 0);
            }
        }
    }
    return 0;
}

/* Depthwise 3x3 conv with the PReLU requantisation. */
int oracle_dw_conv_prelu(const int8_t *x, int n, int h, int wd, int c,
                         const int8_t *w /* [3][3][c] */, int stride,
                         const int32_t *bias, const int32_t *mult, const int32_t *mult_neg,
                         const int32_t *shift, int32_t act_min, int32_t act_max,
                         int8_t *y /* [n][ho][wo][c] */)
{
    if (!x || !w || !bias || !mult || !mult_neg || !shift || !y) return -1;
    if (n <= 0 || h <= 0 || wd <= 0 || c <= 0 || (stride != 1 && stride != 2)) return -1;
    int ho = (h + 2 - 3) / stride + 1;
    int wo = (wd + 2 - 3) / stride + 1;
    int64_t rows = (int64_t)n * ho;
    int64_t row;
#pragma omp parallel for schedule(static)
    for (row = 0; row < rows; ++row) {
        int in_ = (int)(row / ho);
        int oy = (int)(row % ho);
        for (int ox = 0; ox < wo; ++ox) {
            for (int ch = 0; ch < c; ++ch) {
                int64_t acc = 0;
                for (int i = 0; i < 3; ++i) {
                    for (int j = 0; j < 3; ++j) {
                        int iy = oy * stride + i - 1;
                        int ix = ox * stride + j - 1;
                        if (iy < 0 || iy >= h || ix < 0 || ix >= wd) continue; /* zero pad */
                        int64_t xv = x[(((int64_t)in_ * h + iy) * wd + ix) * c + ch];
                        int64_t wv = w[(i * 3 + j) * c + ch];
                        acc += xv * wv;
                    }
                }
                y[(((int64_t)in_ * ho + oy) * wo + ox) * c + ch] =
                    finish_prelu(acc, bias[ch], mult[ch], mult_neg[ch], shift[ch],
                                 act_min, act_max, 0, 0);
            }
        }
    }
    return 0;
}

/* Grouped 3x3 conv, pad 1, stride 1 or 2, NHWC, as many output as input channels, groups of
 * `gs` channels (RegNet / ResNeXt use group sizes above one where MobileNetV2 has the depthwise
 * conv: paper, Section 2; its weights W[cout][cin per group][K][K] are 8-bit with one scale per
 * output channel, Section 3.1 "Depthwise Convolutions", Eq. 4-5).  Output channel ch belongs to
 * group ch / gs and sees input channels (ch / gs) * gs + 0 .. gs-1.  Weights [3][3][c][gs]:
 * w[(i*3 + j)*c + ch][k] multiplies input channel (ch / gs) * gs + k at tap (i, j).
 * acc_out (optional) receives the raw sums; y (optional) the requantised bytes, with the PReLU
 * form when mult_neg is given. */
int oracle_gconv3x3(const int8_t *x, int n, int h, int wd, int c,
                    const int8_t *w /* [3][3][c][gs] */, int gs, int stride,
                    const int32_t *bias, const int32_t *mult, const int32_t *mult_neg /* or NULL */,
                    const int32_t *shift, int32_t act_min, int32_t act_max,
                    int32_t *acc_out /* [n][ho][wo][c] or NULL */, int8_t *y /* [n][ho][wo][c] or NULL */)
{
    if (!x || !w || (!y && !acc_out)) return -1;
    if (y && (!bias || !mult || !shift)) return -1;
    if (n <= 0 || h <= 0 || wd <= 0 || c <= 0 || gs <= 0 || c % gs != 0) return -1;
    if (stride != 1 && stride != 2) return -1;
    int ho = (h + 2 - 3) / stride + 1;
    int wo = (wd + 2 - 3) / stride + 1;
    int64_t rows = (int64_t)n * ho;
    int64_t row;
#pragma omp parallel for schedule(static)
    for (row = 0; row < rows; ++row) {
        int in_ = (int)(row / ho);
        int oy = (int)(row % ho);
        for (int ox = 0; ox < wo; ++ox) {
            for (int ch = 0; ch < c; ++ch) {
                int first = (ch / gs) * gs; /* first input channel of the group */
                int64_t acc = 0;
                for (int i = 0; i < 3; ++i) {
                    for (int j = 0; j < 3; ++j) {
                        int iy = oy * stride + i - 1;
                        int ix = ox * stride + j - 1;
                        if (iy < 0 || iy >= h || ix < 0 || ix >= wd) continue; /* zero pad */
                        for (int k = 0; k < gs; ++k) {
                            int64_t xv = x[(((int64_t)in_ * h + iy) * wd + ix) * c + first + k];
                            int64_t wv = w[((int64_t)(i * 3 + j) * c + ch) * gs + k];
                            acc += xv * wv;
                        }
                    }
                }
                int64_t o = (((int64_t)in_ * ho + oy) * wo + ox) * c + ch;
                if (acc_out) acc_out[o] = (int32_t)acc;
                if (y)
                    y[o] = mult_neg ? finish_prelu(acc, bias[ch], mult[ch], mult_neg[ch], shift[ch],
                                                   act_min, act_max, 0, 0)
                                    : finish(acc, bias[ch], mult[ch], shift[ch], act_min, act_max, 0, 0);
            }
        }
    }
    return 0;
}

/* Inverted-residual block: pointwise expand -> depthwise 3x3 -> pointwise project
 * (+ saturating add of the block input when add_residual).  It is the three functions
 * above chained through caller-provided intermediates t1 [n][h][w][chid] and
 * t2 [n][ho][wo][chid]. */
int oracle_block(const int8_t *x, int n, int h, int wd, int cin, int chid, int cout, int stride,
                 const int8_t *w_exp, const int32_t *b_exp, const int32_t *m_exp,
                 const int32_t *s_exp, int32_t lo_exp, int32_t hi_exp,
                 const int8_t *w_dw, const int32_t *b_dw, const int32_t *m_dw,
                 const int32_t *s_dw, int32_t lo_dw, int32_t hi_dw,
                 const int8_t *w_prj, const int32_t *b_prj, const int32_t *m_prj,
                 const int32_t *s_prj, int32_t lo_prj, int32_t hi_prj,
                 int add_residual, int8_t *t1, int8_t *t2, int8_t *y)
{
    if (add_residual && !(stride == 1 && cin == cout)) return -1;
    int ho = (h + 2 - 3) / stride + 1;
    int wo = (wd + 2 - 3) / stride + 1;
    int rc = oracle_pw_conv(x, n, h, wd, cin, w_exp, chid, b_exp, m_exp, s_exp,
                            lo_exp, hi_exp, NULL, t1);
    if (rc) return rc;
    rc = oracle_dw_conv(t1, n, h, wd, chid, w_dw, stride, b_dw, m_dw, s_dw, lo_dw, hi_dw, t2);
    if (rc) return rc;
    return oracle_pw_conv(t2, n, ho, wo, chid, w_prj, cout, b_prj, m_prj, s_prj,
                          lo_prj, hi_prj, add_residual ? x : NULL, y);
}
