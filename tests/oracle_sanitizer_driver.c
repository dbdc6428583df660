/* Driver for the sanitizer run of the CPU oracle (tests/test_oracle_sanitized.py): every layer
 * function of oracle/prom_oracle.c on heap buffers of exactly the documented sizes, with odd image
 * sizes, both strides and ragged channel counts, so that AddressSanitizer sees any read or write
 * outside a tensor and UndefinedBehaviorSanitizer any overflow or bad shift.  Values come from a
 * small linear congruential generator; the results are not checked here (the pins do that). */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int64_t oracle_requant(int64_t s, int32_t mult, int32_t shift);
int64_t oracle_requant_prelu(int64_t s, int32_t mult, int32_t mult_neg, int32_t shift);
int oracle_pw_accum(const int8_t *x, int64_t m_pixels, int cin, const int8_t *w, int cout, int32_t *acc);
int oracle_pw_conv(const int8_t *x, int n, int h, int wd, int cin, const int8_t *w, int cout,
                   const int32_t *bias, const int32_t *mult, const int32_t *shift, int32_t act_min,
                   int32_t act_max, const int8_t *residual, int8_t *y);
int oracle_pw_conv_prelu(const int8_t *x, int n, int h, int wd, int cin, const int8_t *w, int cout,
                         const int32_t *bias, const int32_t *mult, const int32_t *mult_neg, const int32_t *shift,
                         int32_t act_min, int32_t act_max, const int8_t *residual, int8_t *y);
int oracle_dw_conv(const int8_t *x, int n, int h, int wd, int c, const int8_t *w, int stride,
                   const int32_t *bias, const int32_t *mult, const int32_t *shift, int32_t act_min,
                   int32_t act_max, int8_t *y);
int oracle_dw_conv_prelu(const int8_t *x, int n, int h, int wd, int c, const int8_t *w, int stride,
                         const int32_t *bias, const int32_t *mult, const int32_t *mult_neg, const int32_t *shift,
                         int32_t act_min, int32_t act_max, int8_t *y);
int oracle_gconv3x3(const int8_t *x, int n, int h, int wd, int c, const int8_t *w, int gs, int stride,
                    const int32_t *bias, const int32_t *mult, const int32_t *mult_neg, const int32_t *shift,
                    int32_t act_min, int32_t act_max, int32_t *acc_out, int8_t *y);
int oracle_block(const int8_t *x, int n, int h, int wd, int cin, int chid, int cout, int stride,
                 const int8_t *w_exp, const int32_t *b_exp, const int32_t *m_exp, const int32_t *s_exp,
                 int32_t lo_exp, int32_t hi_exp, const int8_t *w_dw, const int32_t *b_dw, const int32_t *m_dw,
                 const int32_t *s_dw, int32_t lo_dw, int32_t hi_dw, const int8_t *w_prj, const int32_t *b_prj,
                 const int32_t *m_prj, const int32_t *s_prj, int32_t lo_prj, int32_t hi_prj, int add_residual,
                 int8_t *t1, int8_t *t2, int8_t *y);

static uint32_t state = 12345u;
static uint32_t rnd(void) { state = state * 1664525u + 1013904223u; return state >> 8; }

static int8_t *i8(size_t n, int ternary)
{
    int8_t *p = malloc(n ? n : 1);
    for (size_t i = 0; i < n; ++i) p[i] = ternary ? (int8_t)((int)(rnd() % 3) - 1) : (int8_t)(rnd() & 0xFF);
    return p;
}
static int32_t *i32(size_t n, int kind) /* 0 bias, 1 mult, 2 shift, 3 mult_neg */
{
    int32_t *p = malloc(4 * (n ? n : 1));
    for (size_t i = 0; i < n; ++i)
        p[i] = kind == 0 ? (int32_t)(rnd() % 8193) - 4096
             : kind == 1 ? (int32_t)(0x40000000u + (rnd() % 0x3FFFFFFFu))
             : kind == 2 ? (int32_t)(rnd() % 32)
                         : (int32_t)(rnd() % 0x7FFFFFFFu) - 0x20000000;
    return p;
}
#define CHECK(call) do { int rc_ = (call); if (rc_ != 0) { printf("FAILED %s -> %d\n", #call, rc_); return 1; } } while (0)

int main(void)
{
    /* requantisation at the ends of its documented range */
    (void)oracle_requant(((int64_t)1 << 30) - 1, 0x7FFFFFFF, 0);
    (void)oracle_requant(-(((int64_t)1 << 30) - 1), 0x7FFFFFFF, 31);
    (void)oracle_requant_prelu(-(((int64_t)1 << 30) - 1), 0x7FFFFFFF, -0x7FFFFFFF - 1, 31);
    for (int stride = 1; stride <= 2; ++stride) {
        const int n = 2, h = 5, w = 7, cin = 13, chid = 22, cout = cin, c = 12, gs = 4;
        const int ho = (h - 1) / stride + 1, wo = (w - 1) / stride + 1;
        const size_t m = (size_t)n * h * w, mo = (size_t)n * ho * wo;
        int8_t *x = i8(m * cin, 0), *wp = i8((size_t)cout * cin, 1), *res = i8(m * cout, 0), *y = i8(m * cout, 0);
        int32_t *b = i32(cout, 0), *mu = i32(cout, 1), *sh = i32(cout, 2), *mn = i32(cout, 3);
        int32_t *acc = malloc(4 * m * cout);
        CHECK(oracle_pw_accum(x, (int64_t)m, cin, wp, cout, acc));
        CHECK(oracle_pw_conv(x, n, h, w, cin, wp, cout, b, mu, sh, -128, 127, res, y));
        CHECK(oracle_pw_conv(x, n, h, w, cin, wp, cout, b, mu, sh, 0, 127, NULL, y));
        CHECK(oracle_pw_conv_prelu(x, n, h, w, cin, wp, cout, b, mu, mn, sh, -128, 127, res, y));
        int8_t *xd = i8(m * c, 0), *wd = i8((size_t)9 * c, 0), *yd = i8(mo * c, 0);
        int32_t *bd = i32(c, 0), *md = i32(c, 1), *sd = i32(c, 2), *nd = i32(c, 3);
        CHECK(oracle_dw_conv(xd, n, h, w, c, wd, stride, bd, md, sd, 0, 127, yd));
        CHECK(oracle_dw_conv_prelu(xd, n, h, w, c, wd, stride, bd, md, nd, sd, -128, 127, yd));
        int8_t *wg = i8((size_t)9 * c * gs, 0);
        int32_t *accg = malloc(4 * mo * c);
        CHECK(oracle_gconv3x3(xd, n, h, w, c, wg, gs, stride, bd, md, NULL, sd, 0, 127, accg, yd));
        CHECK(oracle_gconv3x3(xd, n, h, w, c, wg, gs, stride, bd, md, nd, sd, -128, 127, NULL, yd));
        CHECK(oracle_gconv3x3(xd, n, h, w, c, wg, 1, stride, bd, md, NULL, sd, -128, 127, accg, NULL));
        /* block: cin -> chid -> cout with the skip at stride 1 */
        int8_t *we = i8((size_t)chid * cin, 1), *wdd = i8((size_t)9 * chid, 0), *wpr = i8((size_t)cout * chid, 1);
        int32_t *be = i32(chid, 0), *me = i32(chid, 1), *se = i32(chid, 2);
        int32_t *bdd = i32(chid, 0), *mdd = i32(chid, 1), *sdd = i32(chid, 2);
        int8_t *t1 = i8(m * chid, 0), *t2 = i8(mo * chid, 0), *yb = i8(mo * cout, 0);
        CHECK(oracle_block(x, n, h, w, cin, chid, cout, stride, we, be, me, se, 0, 127, wdd, bdd, mdd, sdd, 0, 127,
                           wpr, b, mu, sh, -128, 127, stride == 1, t1, t2, yb));
        free(x); free(wp); free(res); free(y); free(b); free(mu); free(sh); free(mn); free(acc);
        free(xd); free(wd); free(yd); free(bd); free(md); free(sd); free(nd); free(wg); free(accg);
        free(we); free(wdd); free(wpr); free(be); free(me); free(se); free(bdd); free(mdd); free(sdd);
        free(t1); free(t2); free(yb);
    }
    printf("ok\n");
    return 0;
}
