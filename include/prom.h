/*
 * prom.h -- C ABI of the MI355X (gfx950) ternary pointwise-convolution library.
 *
 * The operations are the inference hot path of PROM (arXiv 2505.03254):
 *   - a pointwise 1x1 convolution whose weights are ternary {-1,0,+1}, so that every
 *     output is a signed sum of int8 input channels (paper Section 2, last paragraph;
 *     Section 3.1 "Pointwise Convolutions"; Figure 12, inference branch), followed by a
 *     per-output-channel rescale after the convolution (Section 3.1, "Pointwise
 *     Convolutions"; Figure 12), here in integer form;
 *   - the int8 depthwise 3x3 convolution that sits between two pointwise convolutions
 *     (Section 2, first paragraph; Section 3.1 "Depthwise Convolutions", Eq. 4-5);
 *   - the block expand -> depthwise -> project with optional skip (Section 2; Figure 4).
 *
 * Conventions shared by every entry point
 *   Layout      activations are int8 NHWC, dense (no strides); a pointwise layer sees them
 *               as a row-major [M = n*h*w][C] matrix.
 *   Memory      "dev" pointers are device (HBM) addresses, "host" pointers are host
 *               addresses.  The caller owns every buffer.  The library allocates nothing,
 *               frees nothing and never synchronises: kernels are enqueued on `stream`
 *               (a hipStream_t passed as void*, NULL = the default stream) and the call
 *               returns immediately.
 *   Requant     with acc the int32 accumulator of output channel c,
 *                   s = acc + bias[c]
 *                   q = floor( s * mult[c] / 2^(31 + shift[c]) + 1/2 )   (one rounding,
 *                                                                  ties toward +infinity)
 *                   y = min(max(q, act_min), act_max)
 *                   if a residual is given:  y = min(max(y + residual, -128), 127)
 *               The paper rescales in floating point (Figure 12); this integer form with
 *               bias (folded BatchNorm shift), Q31 multiplier and shift is the contract of
 *               this library.  Preconditions (not checked, the arrays live on the device):
 *               0 < mult[c] < 2^31, 0 <= shift[c] <= 31, |bias[c]| < 2^29 and |acc + bias[c]| < 2^30;
 *               prom_requant_check copies the arrays back and checks them, for tests and bring-up.
 *   Errors      every int-returning function returns PROM_OK (0) or a negative code; on an
 *               argument error nothing has been enqueued.  PROM_EHIP (the runtime refused a
 *               launch) from an entry point that makes several launches -- prom_block in its
 *               multi-launch forms, prom_pw_conv_sequence -- can leave the earlier launches
 *               enqueued.
 */
#ifndef PROM_H
#define PROM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    PROM_OK = 0,
    PROM_EINVAL = -1,        /* null pointer, non-positive dimension, bad window or stride    */
    PROM_EUNSUPPORTED = -2,  /* shape beyond a compiled limit (see each function)             */
    PROM_EALIAS = -3,        /* output overlaps an input it must not overlap                  */
    PROM_EWORKSPACE = -4,    /* workspace missing or too small                                */
    PROM_EHIP = -5,          /* the HIP runtime reported an error at launch                   */
    PROM_EVALUE = -6,        /* prom_pack_ternary: a weight outside {-1,0,+1}                 */
    PROM_ESCRATCH = -7       /* a no-allocation entry point: the problem needs more scratch
                                memory than the library's fixed array holds                  */
};

/* Per-output-channel requantisation and activation window.  The struct itself is read on
 * the host at call time; its arrays are device memory of C int32 values each.
 *
 * PReLU (the paper's MobileNetV2 and RegNetX models replace ReLU6 / ReLU by PReLU, Section 3.2,
 * last paragraph): with mult_neg != NULL the multiplier of an output follows the sign of
 * s = acc + bias[c] (which is the sign of the real pre-activation, the scales being positive):
 *     m = s >= 0 ? mult[c] : mult_neg[c]
 *     q = floor((s*m + 2^(30+shift[c])) / 2^(31+shift[c])),  then the window and the residual
 * mult_neg[c] is the slope a_c folded into the multiplier (a_c * mult[c], same shift); any int32
 * value is computed exactly (a slope may be negative or, with a smaller mult, above 1).  The
 * window is then usually the full [-128, 127].  mult_neg == NULL gives the plain form above. */
typedef struct {
    const int32_t *bias;     /* dev [C]                                                       */
    const int32_t *mult;     /* dev [C]  Q31 multiplier, 2^30 <= mult < 2^31 for a normalised
                                          scale (any 0 < mult < 2^31 is computed exactly)     */
    const int32_t *shift;    /* dev [C]  extra right shift, 0..31                             */
    int32_t act_min;         /* -128 <= act_min <= act_max <= 127; [0,127] is ReLU6 when the  */
    int32_t act_max;         /*  output scale maps 6.0 to 127                                 */
    const int32_t *mult_neg; /* dev [C] or NULL: PReLU multiplier for acc + bias < 0          */
} prom_requant_t;

/* Opt-in check of the preconditions above, for tests and bring-up (the layer entry points cannot
 * afford it: the arrays live on the device).  Copies bias, mult and shift of `channels` channels
 * back to the host -- which waits for the work already enqueued on the device -- and returns
 * PROM_EINVAL, with the first offending channel in *bad_channel (if not NULL), when a multiplier
 * is not in (0, 2^31), a shift not in [0, 31], |bias| >= 2^29, or 128 * cin + |bias| >= 2^30
 * (the accumulator of a pointwise layer with cin input channels is at most 128 * cin in
 * magnitude; for a depthwise or grouped 3x3 layer, whose weights reach 127, pass
 * cin = 9 * 127 * group_size).  mult_neg may be
 * any int32 and is not looked at.  PROM_EHIP if the copies fail. */
int prom_requant_check(const prom_requant_t *rq, int channels, int cin, int *bad_channel);

/* Optional launch plan of prom_pw_conv_ex; zero in a field means "library default".
 * With tiles_per_wave or pixel_tiles given and row_waves == 0 the plain streaming kernel runs
 * (every wavefront on its own pixel groups, one chunk of 16*tiles_per_wave channels per
 * workgroup).  row_waves = 2, 3 or 4 asks for the row-cooperative kernel: that many wavefronts
 * of a workgroup share a pixel group and write whole rows of 16*tiles_per_wave*row_waves
 * channels together; it needs tiles_per_wave in 1..6, pixel_tiles 0 or 1 and
 * cout % (16*tiles_per_wave*row_waves) == 0 (and, like the fast path in general, cin % 8 == 0).
 * k_outer = 1 asks for the kernel of wide layers (the k loop outermost over a workgroup tile of 128
 * output channels x 256 pixels, weights decoded per k step): it needs cin % 64 == 0,
 * cout % 16 == 0, 16-byte aligned x, y, residual, 8-byte aligned packed weights and every other
 * field zero; k_outer = -1 keeps it off; 0 leaves the choice to the library (it takes this kernel
 * from 1024 input and 256 output channels on). */
typedef struct {
    int32_t tiles_per_wave;  /* NT: 16-channel output tiles each wavefront owns (1..10)       */
    int32_t pixel_tiles;     /* PT: 16-pixel tiles a wavefront processes per iteration (1,2,4)*/
    int32_t workgroups;      /* workgroups launched per output-channel chunk (per row piece)  */
    int32_t row_waves;       /* 0, 2, 3 or 4: wavefronts per pixel group, see above           */
    int32_t k_outer;         /* 1: the kernel of wide layers, -1: never, 0: library default   */
} prom_pw_plan_t;

/* ---- ternary weight packing (host side, once per layer: the paper notes that weights are
 * quantised and fixed in advance, Figure 12) ------------------------------------------- */

/* Bytes of the packed form of a [cout][cin] ternary matrix: 2 bits per weight, each row
 * padded to a multiple of 16 weights (one 32-bit word per 16 weights). 0 if a dimension is
 * not positive. */
size_t prom_packed_size(int cout, int cin);

/* Pack w_host[cout][cin] (row-major int8, every value in {-1,0,+1}) into packed_host.
 * Codes: 0 -> 00, +1 -> 01, -1 -> 11 (two-bit two's complement); 10 never occurs and padding
 * weights are 00.  Word j of row c holds weights k = 16j..16j+15 of that row; weight
 * k = 16j + 4d + b (d, b in 0..3) sits at bits [8b+2d, 8b+2d+1] of the word, so that
 * (word >> 2d) & 0x03030303 yields the four codes of 32-bit lane d of the decoded 16-byte
 * group.  Returns PROM_EVALUE for a weight outside {-1,0,+1} (nothing useful is written),
 * PROM_EWORKSPACE if packed_bytes < prom_packed_size(cout, cin).  Host to host; the caller
 * copies the result to the device. */
int prom_pack_ternary(const int8_t *w_host, int cout, int cin, void *packed_host,
                      size_t packed_bytes);

/* Inverse of prom_pack_ternary (host to host), for round-trip checks and tooling. */
int prom_unpack_ternary(const void *packed_host, size_t packed_bytes, int cout, int cin,
                        int8_t *w_host);

/* ---- weight preparation (the step before the path; paper Section 3.1 and its pseudocode of the
 * weight quantisation) ------------------------------------------------------------------
 * Channel-wise absmean ternary quantisation of a pointwise layer, on the device:
 *   scale[i] = 1 / max(mean_j |w[i][j]|, eps),  code = clamp(round(w[i][j] * scale[i]), -1, 1),
 * round half to even; the mean is the float64 sum of the row divided by cin and rounded to
 * float32, the scale one float32 division, the product one float32 multiplication (the paper's
 * code is float32).  The per-channel dequantisation factor of the layer is 1 / scale[i].
 *   w       dev float32 [cout][cin]
 *   packed  dev, receives the prom_pack_ternary layout (prom_packed_size(cout, cin) bytes,
 *           4-byte aligned): ready to be passed as w_packed
 *   codes   dev int8 [cout][cin] or NULL: the codes unpacked, for inspection
 *   scale   dev float32 [cout]
 * PROM_EINVAL for null / misaligned pointers, non-positive sizes or eps <= 0; PROM_EWORKSPACE
 * if packed_bytes is too small. */
int prom_quantize_pw_absmean(const float *w, int cout, int cin, float eps, void *packed,
                             size_t packed_bytes, int8_t *codes, float *scale, void *stream);

/* Channel-wise absmax 8-bit quantisation of a depthwise 3x3 layer, on the device:
 *   scale[c] = 127 / max(max_t |w[c][t]|, eps),  q = clamp(round(w[c][t] * scale[c]), -128, 127).
 *   w   dev float32 [c][3][3] (the paper's [c_out][1][k][k])
 *   wq  dev int8 [3][3][c], the layout prom_dw_conv takes;  scale dev float32 [c] */
int prom_quantize_dw_absmax(const float *w, int c, float eps, int8_t *wq, float *scale, void *stream);

/* The same for a grouped 3x3 layer (Section 3.1: W[c_out][c_in per group][K][K], Eq. 4-5): one
 * scale per output channel over its group's input channels and the 9 taps.
 *   w   dev float32 [c][group_size][3][3]
 *   wq  dev int8 [3][3][c][group_size], the layout prom_gconv3x3 takes;  scale dev float32 [c]
 * PROM_EINVAL if c % group_size != 0. */
int prom_quantize_gconv_absmax(const float *w, int c, int group_size, float eps, int8_t *wq,
                               float *scale, void *stream);

/* Activation quantisation with one dynamic scale per batch element (paper Section 3.1, Eq. 6-7;
 * factor 127 and eps clamp as in its pseudocode), on the device:
 *   scale[i] = 127 / max(max over the image |x[i][...]|, eps),
 *   q[i][...] = clamp(round(x[i][...] * scale[i]), -128, 127), round half to even, float32.
 *   x      dev float32 [n][per_image] (any layout inside an image: the scale is over all of it)
 *   q      dev int8 [n][per_image];  scale dev float32 [n] (also used as scratch during the call)
 * Two passes over x (maximum, then quantise) plus two tiny kernels; n <= 65535.  PROM_EINVAL
 * for null or misaligned pointers, non-positive sizes, eps <= 0. */
int prom_quantize_activation_absmax(const float *x, int n, long long per_image, float eps, int8_t *q,
                                    float *scale, void *stream);

/* Ternary pointwise layer whose int8 output takes the dynamic per-image activation scale of the
 * paper (Section 3.1: the layer's real-valued output is the integer accumulator times the weight
 * scale of Eq. 1 and the input's activation step; Eq. 6-7 with the factor 127 and the eps clamp of
 * the pseudocode quantise it with one absmax scale per batch element), fused: the real-valued
 * tensor is never written.  With i the image of pixel m:
 *   z[m][co]  = (float(acc[m][co]) * w_scale[co]) * x_step[i] + bias[co]   three float32 operations,
 *               each rounded once, in this order;  z = max(z, 0) if relu != 0
 *   amax[i]   = max |z| over the image;  scale[i] = 127 / max(amax[i], eps)
 *   q[m][co]  = clamp(round_half_even(z * scale[i]), -128, 127)
 *   x        dev int8 [n][h][w][cin], 16-byte aligned; real value x * x_step[i]
 *   w_packed dev, prom_pack_ternary output for [cout][cin]; real value code * w_scale[co]
 *   x_step   dev float32 [n];  w_scale dev float32 [cout];  bias dev float32 [cout] or NULL
 *   q        dev int8 [n][h][w][cout], 16-byte aligned;  amax, scale dev float32 [n] (outputs)
 * Three launches on `stream`: clear amax, the layer with a maximum-only epilogue (one atomic
 * maximum per wavefront and image), the layer again with the quantising epilogue.
 * PROM_EINVAL for null or misaligned pointers, non-positive sizes or eps; PROM_EUNSUPPORTED unless
 * cin % 4 == 0, cout % 16 == 0 and cin <= 1024, or if a tensor reaches 2 GiB. */
int prom_pw_conv_dynq(const int8_t *x, int n, int h, int w, int cin, const void *w_packed, int cout,
                      const float *x_step, const float *w_scale, const float *bias, int relu, float eps,
                      int8_t *q, float *amax, float *scale, void *stream);

/* ---- pointwise 1x1 convolution with ternary weights ------------------------------------
 * y[m][co] = requant_co( sum_k x[m][k] * W[co][k] ),  m over n*h*w pixels.
 *   x         dev int8 [n][h][w][cin]
 *   w_packed  dev, prom_pack_ternary output for [cout][cin], 4-byte aligned
 *   rq        host struct; arrays dev [cout]
 *   residual  dev int8 [n][h][w][cout] or NULL; may be the same buffer as y (each element
 *             is read before it is written)
 *   y         dev int8 [n][h][w][cout]; must not overlap x or w_packed
 * Limits: cin <= 4096 (PROM_EUNSUPPORTED above).  n*h*w*max(cin,cout) must be < 2^40.
 * Fast path needs cin % 8 == 0, cout % 4 == 0 and 4-byte aligned x, y, residual; other
 * shapes run a slower kernel with identical results. */
int prom_pw_conv(const int8_t *x, int n, int h, int w, int cin,
                 const void *w_packed, int cout, const prom_requant_t *rq,
                 const int8_t *residual, int8_t *y, void *stream);

/* Same operation with an explicit launch plan (testing and tuning); plan == NULL is
 * prom_pw_conv.  PROM_EINVAL if the plan is not realisable for this shape. */
int prom_pw_conv_ex(const int8_t *x, int n, int h, int w, int cin,
                    const void *w_packed, int cout, const prom_requant_t *rq,
                    const int8_t *residual, int8_t *y, const prom_pw_plan_t *plan,
                    void *stream);

/* The launch plan prom_pw_conv would use for this shape (all pointers assumed 4-byte aligned):
 * fills every field of plan_out (row_waves = 0 for the plain streaming kernel) and, if
 * load_bytes_out is not NULL, the activation load width in bytes (16, 8, or 1 for the slow
 * generic kernel).  Host only, launches nothing. */
int prom_pw_plan_query(int n, int h, int w, int cin, int cout, prom_pw_plan_t *plan_out,
                       int *load_bytes_out);

/* One layer of a sequence for prom_pw_conv_sequence: the arguments of prom_pw_conv. */
typedef struct {
    const int8_t *x;
    int32_t n, h, w, cin;
    const void *w_packed;
    int32_t cout;
    prom_requant_t rq;
    const int8_t *residual;
    int8_t *y;
} prom_pw_layer_t;

/* Enqueue `count` pointwise layers on `stream` with one host call.  The results are those of
 * running the layers one after the other in the given order.  Consecutive small layers that do
 * not touch each other's data (no layer's output overlaps another's input, residual, weights
 * or output) are put into one kernel launch and run concurrently, which hides their launch,
 * first-load and write-back latencies; anything else is launched layer by layer.  All layers
 * are validated first; on an argument error nothing is enqueued and the index of the offending
 * layer is stored in *bad_layer when bad_layer is not NULL. */
int prom_pw_conv_sequence(const prom_pw_layer_t *layers, int count, int *bad_layer, void *stream);

/* 1 if a layer of this shape (4-byte aligned pointers assumed) is small enough and regular
 * enough to join a batched launch of prom_pw_conv_sequence, 0 if not, negative on bad shapes. */
int prom_pw_batchable(int n, int h, int w, int cin, int cout);

/* Which shared launch prom_pw_conv_sequence would put a layer of this shape into (pointers assumed
 * 4-byte aligned): 1 = the launch of small layers, 2 = the launch of large layers, 0 = none (the
 * layer is launched alone); negative = error code.  Host only, launches nothing. */
int prom_pw_batch_class(int n, int h, int w, int cin, int cout);

/* The same layer computed by the other design that was evaluated: multiplication-free
 * accumulation on the vector ALU (sums of the input bytes whose weight is +1 / -1, paper
 * Section 2), one lane per pixel.  Bit-identical results; kept for the A/B measurement against
 * the MFMA kernel, not for production use.  Limits: cin <= 256, cin % 4 == 0, cout % 4 == 0,
 * 4-byte aligned pointers, tensors below 2 GiB, no PReLU multipliers (PROM_EUNSUPPORTED
 * otherwise). */
int prom_pw_conv_addsub(const int8_t *x, int n, int h, int w, int cin,
                        const void *w_packed, int cout, const prom_requant_t *rq,
                        const int8_t *residual, int8_t *y, void *stream);

/* Raw int32 accumulators acc[m][co] = sum_k x[m][k] * W[co][k] (no bias, no requant), for
 * staged checking of the accumulation alone.  acc: dev int32 [n*h*w][cout]. */
int prom_pw_accum_i32(const int8_t *x, int n, int h, int w, int cin,
                      const void *w_packed, int cout, int32_t *acc, void *stream);

/* ---- depthwise 3x3 convolution, pad 1, stride 1 or 2 -----------------------------------
 * acc[n][oy][ox][c] = sum_{i,j in 0..2} x[n][oy*stride+i-1][ox*stride+j-1][c] * w_dw[i][j][c]
 * with x = 0 outside the image (the paper's quantisers are symmetric: no zero-point), then
 * the requantisation above.  ho = (h-1)/stride + 1, wo = (w-1)/stride + 1.
 *   x dev int8 [n][h][w][c];  w_dw dev int8 [3][3][c];  y dev int8 [n][ho][wo][c];
 *   y must not overlap x. */
int prom_dw_conv(const int8_t *x, int n, int h, int w, int c,
                 const int8_t *w_dw, int stride, const prom_requant_t *rq,
                 int8_t *y, void *stream);

/* One layer of a sequence for prom_dw_conv_sequence: the arguments of prom_dw_conv. */
typedef struct {
    const int8_t *x;
    int32_t n, h, w, c;
    const int8_t *w_dw;
    int32_t stride;
    prom_requant_t rq;
    int8_t *y;
} prom_dw_layer_t;

/* Enqueue `count` depthwise layers (the operation of prom_dw_conv, paper Section 3.1 "Depthwise
 * Convolutions") on `stream` with one host call.  The results are those of running the layers one
 * after the other in the given order.  Consecutive layers that do not touch each other's data (no
 * layer's output overlaps another's input, weights, parameters or output) share one kernel launch
 * and run concurrently, which hides the launch, first-load and write-back latencies of the small
 * layers; anything else is launched layer by layer.  All layers are validated first; on an
 * argument error nothing is enqueued and the index of the offending layer is stored in *bad_layer
 * when bad_layer is not NULL.  PROM_EHIP if a launch fails (earlier launches stay enqueued). */
int prom_dw_conv_sequence(const prom_dw_layer_t *layers, int count, int *bad_layer, void *stream);

/* ---- grouped 3x3 convolution, pad 1, stride 1 or 2 --------------------------------------
 * RegNet and ResNeXt have group sizes above one where MobileNetV2 has the depthwise convolution
 * (paper Section 2); the weights are 8-bit with one scale per output channel like the depthwise
 * ones (Section 3.1, Eq. 4-5).  As many output as input channels; output channel ch belongs to
 * group ch / group_size and sees that group's input channels:
 *   acc[n][oy][ox][ch] = sum_{i,j in 0..2} sum_{k < group_size}
 *         x[n][oy*stride+i-1][ox*stride+j-1][(ch / group_size) * group_size + k] * w_g[i][j][ch][k]
 * with x = 0 outside the image, then the requantisation above (plain or PReLU).
 *   x dev int8 [n][h][w][c];  w_g dev int8 [3][3][c][group_size];  y dev int8 [n][ho][wo][c];
 *   c % group_size == 0 (PROM_EINVAL otherwise); group_size <= 4096; y must not overlap x or w_g.
 * group_size 4, 8, 16, 32 or 64 (c % 4 == 0, 4-byte aligned tensors below 2 GiB, 16-byte aligned
 * parameter arrays, w <= 190) runs on the matrix cores; any other multiple of 4 on a tiled
 * vector-ALU kernel, group_size 1 is prom_dw_conv, anything else a slow one-thread-per-output
 * kernel.
 *   w_frag (optional, may be NULL): the same weights in the operand order of the matrix-core
 *   kernel, prepared once per layer with prom_gconv_pack (weights are fixed at inference, paper
 *   Figure 12) and copied to the device, 16-byte aligned; with it a workgroup starts with a plain
 *   copy instead of decoding w_g.  It must describe the same weights as w_g (not checked); it is
 *   ignored by the kernels that do not use it, and PROM_EINVAL if prom_gconv_frag_size(c,
 *   group_size) is 0. */
int prom_gconv3x3(const int8_t *x, int n, int h, int w, int c,
                  const int8_t *w_g, const void *w_frag, int group_size, int stride,
                  const prom_requant_t *rq, int8_t *y, void *stream);

/* One layer of a sequence for prom_gconv3x3_sequence: the arguments of prom_gconv3x3. */
typedef struct {
    const int8_t *x;
    int32_t n, h, w, c;
    const int8_t *w_g;
    const void *w_frag; /* or NULL */
    int32_t group_size, stride;
    prom_requant_t rq;
    int8_t *y;
} prom_gconv_layer_t;

/* Enqueue `count` grouped 3x3 layers (the operation of prom_gconv3x3; paper Section 2 for the
 * layer, Section 3.1 and Eq. 4-5 for its quantisation) on `stream` with one host call.  The
 * results are those of running the layers one after the other in the given order.  Consecutive
 * layers that run on the same matrix-core kernel (group sizes 4, 8, 16; group sizes 32, 64) and do
 * not touch each other's data (no layer's output overlaps another's input, weights, parameters or
 * output) share one kernel launch, up to 24 of them, and run concurrently; anything else is
 * launched layer by layer.  All layers are validated first; on an argument error nothing is
 * enqueued and the index of the offending layer is stored in *bad_layer when bad_layer is not
 * NULL (a layer with group size 1 is handed to prom_dw_conv when its turn comes, and what that
 * call checks beyond pointers, sizes and the window is checked then).  PROM_EHIP if a launch fails
 * (earlier launches stay enqueued). */
int prom_gconv3x3_sequence(const prom_gconv_layer_t *layers, int count, int *bad_layer, void *stream);

/* Bytes of the prepared form of prom_gconv_pack; 0 if the matrix-core kernel does not take this
 * layer (group_size not 4, 8, 16, 32 or 64, c % 4 != 0 or c % group_size != 0). */
size_t prom_gconv_frag_size(int c, int group_size);

/* Host to host: w_host[3][3][c][group_size] -> frag_host, laid out
 * [block of 64 channels][tile t: 4][tap: 9][lane: 64][16 bytes]: lane (i = lane & 15, kg = lane >> 4)
 * of tile t holds, for output channel oc = 64*block + 16*(i >> 2) + 4*t + (i & 3), the weights on
 * input channels 64*block + 16*kg + 0..15 (those of oc's group, zero elsewhere).
 * PROM_EUNSUPPORTED if prom_gconv_frag_size is 0, PROM_EWORKSPACE if frag_bytes is too small. */
int prom_gconv_pack(const int8_t *w_host, int c, int group_size, void *frag_host, size_t frag_bytes);

/* ---- inverted-residual block ------------------------------------------------------------
 * pointwise expand (cin -> chid, rq_expand) -> depthwise 3x3 (stride, rq_dw) ->
 * pointwise project (chid -> cout, rq_project); if add_residual (requires stride == 1 and
 * cin == cout) the block input x is added with saturation after the projection's clamp.
 *   workspace  dev, at least prom_block_workspace_size(...) bytes, 256-byte aligned; holds
 *              intermediates, contents undefined afterwards
 *   y          dev int8 [n][ho][wo][cout]; must not overlap x or the workspace */
int prom_block(const int8_t *x, int n, int h, int w, int cin, int chid, int cout, int stride,
               const void *w_expand_packed, const prom_requant_t *rq_expand,
               const int8_t *w_dw, const prom_requant_t *rq_dw,
               const void *w_project_packed, const prom_requant_t *rq_project,
               int add_residual, void *workspace, size_t workspace_bytes,
               int8_t *y, void *stream);

size_t prom_block_workspace_size(int n, int h, int w, int cin, int chid, int cout, int stride);

/* The same with the choice between the forms of the block made by the caller: as one kernel whose
 * expanded band stays in LDS as 16-channel planes (PROM_BLOCK_PLANES: any number of hidden
 * channels that is a multiple of 16), as one chunk-interleaved kernel with every weight decoded in
 * LDS (PROM_BLOCK_FUSED: up to 192 hidden channels), as three launches through the workspace, or as
 * two launches (expand, then depthwise and projection fused: prom_dw_pw_conv; only the expanded
 * tensor goes through the workspace).  prom_block is prom_block_ex with PROM_BLOCK_AUTO, which takes
 * the form measured faster for the shape.  A form returns PROM_EUNSUPPORTED where it does not apply
 * (prom_block_planes_applies with 16-byte aligned parameter arrays of the first two layers,
 * prom_block_can_fuse, prom_dw_pw_can_fuse; x, y, w_dw 8-byte aligned). */
enum { PROM_BLOCK_AUTO = 0, PROM_BLOCK_FUSED = 1, PROM_BLOCK_UNFUSED = 2, PROM_BLOCK_DWPROJ = 3, PROM_BLOCK_PLANES = 4 };
int prom_block_ex(const int8_t *x, int n, int h, int w, int cin, int chid, int cout, int stride,
                  const void *w_expand_packed, const prom_requant_t *rq_expand,
                  const int8_t *w_dw, const prom_requant_t *rq_dw,
                  const void *w_project_packed, const prom_requant_t *rq_project,
                  int add_residual, void *workspace, size_t workspace_bytes,
                  int8_t *y, int path, void *stream);

/* 1 if prom_block (PROM_BLOCK_AUTO) runs this shape as one kernel of either kind (pointers
 * assumed aligned), 0 if as three launches through the workspace, PROM_EINVAL for bad dimensions.
 * Host only, launches nothing. */
int prom_block_is_fused(int n, int h, int w, int cin, int chid, int cout, int stride);

/* 1 if the chunk-interleaved fused kernel (PROM_BLOCK_FUSED) applies to the shape at all (cin % 8 == 0, chid % 4 == 0, cout % 4 == 0,
 * cout <= 160, chid <= 192, a band of rows fits in LDS), 0 if not. */
int prom_block_can_fuse(int n, int h, int w, int cin, int chid, int cout, int stride);

/* 1 if PROM_BLOCK_PLANES applies to the shape (one kernel; a band of the expanded tensor stays in
 * LDS as 16-channel planes and no weight matrix passes through LDS: cin % 8 == 0, cin <= 192,
 * chid % 16 == 0, cout % 4 == 0, tensors below 2 GiB, a band of one output row fits 160 KB of LDS;
 * pointers assumed 8-byte aligned), 0 if not, PROM_EINVAL for bad dimensions.  Host only. */
int prom_block_planes_applies(int n, int h, int w, int cin, int chid, int cout, int stride);

/* ---- depthwise 3x3 and the pointwise projection behind it, in one kernel ---------------------
 * The second half of the block (Section 2; Figure 4: depthwise, then the projecting pointwise
 * layer, then the skip): y = pw(dw(x)) (+ residual), the depthwise output never leaves the chip.
 * It is also the whole first bottleneck of MobileNetV2 (t = 1: no expansion layer).
 *   x                 dev int8 [n][h][w][c]; w_dw dev int8 [3][3][c]; rq_dw [c]
 *   w_project_packed  dev, prom_pack_ternary output for [cout][c]; rq_project [cout]
 *   residual          dev int8 [n][ho][wo][cout] or NULL (may be y itself); y dev int8 [n][ho][wo][cout]
 * The result is bit for bit that of prom_dw_conv followed by prom_pw_conv.  Limits
 * (PROM_EUNSUPPORTED otherwise; prom_dw_pw_can_fuse tells): c % 16 == 0, cout % 4 == 0,
 * cout <= 320, 4-byte aligned tensors below 2 GiB, and a band of at least one output row whose
 * input rows are at most 256 pixels (w <= 85 at stride 1) and fit LDS with the layer's weights. */
int prom_dw_pw_conv(const int8_t *x, int n, int h, int w, int c, const int8_t *w_dw, int stride,
                    const prom_requant_t *rq_dw, const void *w_project_packed, int cout,
                    const prom_requant_t *rq_project, const int8_t *residual, int8_t *y, void *stream);

/* 1 if prom_dw_pw_conv takes the shape (pointers assumed aligned), 0 if not, PROM_EINVAL for bad
 * dimensions.  Host only. */
int prom_dw_pw_can_fuse(int n, int h, int w, int c, int cout, int stride);

/* ---- the block for callers that cannot allocate --------------------------------------------
 * For callers that cannot call hipMalloc or bring a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation.  prom_block with PROM_BLOCK_AUTO, but
 * the two intermediates of the three-launch form live in a fixed array inside the library's
 * device image instead of a caller workspace: the call allocates nothing (no hipMalloc, no
 * hipFree, no allocating library routine) and takes inputs and outputs only.
 *   Limit    prom_block_workspace_size(...) of the shape must not exceed
 *            prom_block_noalloc_max_workspace() (32 MiB), else PROM_ESCRATCH and nothing is
 *            enqueued.  All other arguments, limits and errors are prom_block's.
 *   Memory   the array exists once per GPU that the library runs on, from the first call there
 *            until the process ends.  Its device address is looked up on the first call on each
 *            device (with that device current).
 *   Sharing  every call on a GPU uses that GPU's one array and finds the previous call's bytes
 *            in it; nothing in it has to start at zero (each intermediate element is written
 *            before it is read).  Two calls that overlap in time on one GPU (different streams
 *            without an ordering between them) race on it: order them. */
int prom_block_noalloc(const int8_t *x, int n, int h, int w, int cin, int chid, int cout, int stride,
                       const void *w_expand_packed, const prom_requant_t *rq_expand,
                       const int8_t *w_dw, const prom_requant_t *rq_dw,
                       const void *w_project_packed, const prom_requant_t *rq_project,
                       int add_residual, int8_t *y, void *stream);

/* Bytes of the fixed array behind prom_block_noalloc. */
size_t prom_block_noalloc_max_workspace(void);

/* ---- measurement utility ------------------------------------------------------------------
 * Plain streaming copy of nbytes (multiple of 16, both pointers 16-byte aligned) from src to
 * dst, dev to dev, as a kernel of this library: the HBM-bandwidth yardstick the pointwise
 * kernel is compared with, and the known-size reference for scaling hardware byte counters. */
int prom_copy_bytes(const void *src, void *dst, size_t nbytes, void *stream);

/* Read-only and write-only streaming kernels over nbytes (multiple of 16, 16-byte aligned) of
 * device memory: the measured HBM ceilings that go beside the data-sheet bandwidth.  sink is a
 * device int that is never written for ordinary data (it keeps the reads alive). */
int prom_stream_read(const void *src, size_t nbytes, int *sink, void *stream);
int prom_stream_write(void *dst, size_t nbytes, int value, void *stream);

/* Register-resident int8 matrix-core loop (v_mfma_i32_16x16x64_i8, no memory traffic): the measured
 * MFMA ceiling.  Every wavefront of a grid that fills the chip issues 8 * iters instructions.
 * Returns the number of integer operations the launch performs (2 per multiply-accumulate), or a
 * negative error code. */
long long prom_mfma_i8_loop(int iters, int *sink, void *stream);

/* Static, human-readable text for a return code. */
const char *prom_strerror(int code);

/* Text of the HIP runtime error behind the most recent PROM_EHIP on the calling thread. */
const char *prom_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PROM_H */
