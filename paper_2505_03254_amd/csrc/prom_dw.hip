// int8 depthwise 3x3 convolution (pad 1, stride 1 or 2), NHWC, with the exact integer
// requantisation epilogue.  This is the 8-bit convolution that sits between the two ternary
// pointwise convolutions of a block (paper Section 2; Section 3.1 "Depthwise Convolutions").
// It is not a dense contraction (9 taps per output, channels independent), so it runs on
// the vector ALU: a thread owns 4 consecutive channels (one dword of the NHWC row) of one
// output column and walks down a strip of output rows.
#include "prom.h"
#include "prom_device.h"
#include "prom_launch.h"

namespace prom {

struct DwArgs {
    const int8_t *x;
    const int8_t *w;  // [3][3][C]
    const int32_t *bias;
    const int32_t *mult;
    const int32_t *shift;
    int8_t *y;
    int N, H, W, C, Ho, Wo, stride;
    int strips;      // row strips per image
    int strip_rows;  // output rows per strip
    int lo_b, hi_b;
    long long total;  // threads with work
};

// C % 4 == 0, 4-byte aligned x / y / w.
__global__ __launch_bounds__(256) void dw_kernel_c4(const DwArgs a)
{
    set_f64_round_down();
    const long long tid = (long long)blockIdx.x * 256 + threadIdx.x;
    if (tid >= a.total) return;
    const int C4 = a.C >> 2;
    const int c4 = (int)(tid % C4);
    long long r = tid / C4;
    const int ox = (int)(r % a.Wo);
    r /= a.Wo;
    const int strip = (int)(r % a.strips);
    const int n = (int)(r / a.strips);
    const int c = c4 * 4;

    int wt[9][4];
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        const uint32_t v = *reinterpret_cast<const uint32_t *>(a.w + (long long)t * a.C + c);
#pragma unroll
        for (int q = 0; q < 4; ++q) wt[t][q] = sbyte(v, q);
    }
    int bias[4];
    double scale[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        bias[q] = a.bias[c + q];
        scale[q] = make_scale(a.mult[c + q], a.shift[c + q]);
    }

    const int oy0 = strip * a.strip_rows;
    const int oy1 = min(oy0 + a.strip_rows, a.Ho);
    const int8_t *xn = a.x + (long long)n * a.H * a.W * a.C + c;
    int8_t *yn = a.y + (long long)n * a.Ho * a.Wo * a.C + c;
    const int ix0 = ox * a.stride - 1;

    for (int oy = oy0; oy < oy1; ++oy) {
        int acc[4] = {bias[0], bias[1], bias[2], bias[3]};
        const int iy0 = oy * a.stride - 1;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int iy = iy0 + i;
            const bool rowok = iy >= 0 && iy < a.H;
#pragma unroll
            for (int jx = 0; jx < 3; ++jx) {
                const int ix = ix0 + jx;
                uint32_t v = 0;
                if (rowok && ix >= 0 && ix < a.W)
                    v = *reinterpret_cast<const uint32_t *>(xn + ((long long)iy * a.W + ix) * a.C);
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] += sbyte(v, q) * wt[i * 3 + jx][q];
            }
        }
        int o[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) o[q] = requant_to_biased(acc[q], scale[q], a.lo_b, a.hi_b);
        *reinterpret_cast<uint32_t *>(yn + ((long long)oy * a.Wo + ox) * a.C) =
            pack4_low_bytes(o[0], o[1], o[2], o[3]);
    }
}

// Any C and alignment: one thread per output element.
__global__ __launch_bounds__(256) void dw_kernel_generic(const DwArgs a)
{
    set_f64_round_down();
    const long long tid = (long long)blockIdx.x * 256 + threadIdx.x;
    if (tid >= a.total) return;
    const int c = (int)(tid % a.C);
    long long r = tid / a.C;
    const int ox = (int)(r % a.Wo);
    r /= a.Wo;
    const int oy = (int)(r % a.Ho);
    const int n = (int)(r / a.Ho);
    int acc = a.bias[c];
    for (int i = 0; i < 3; ++i) {
        const int iy = oy * a.stride + i - 1;
        if (iy < 0 || iy >= a.H) continue;
        for (int jx = 0; jx < 3; ++jx) {
            const int ix = ox * a.stride + jx - 1;
            if (ix < 0 || ix >= a.W) continue;
            acc += (int)a.x[(((long long)n * a.H + iy) * a.W + ix) * a.C + c] *
                   (int)a.w[(i * 3 + jx) * a.C + c];
        }
    }
    const int v = requant_to_biased(acc, make_scale(a.mult[c], a.shift[c]), a.lo_b, a.hi_b);
    a.y[tid] = (int8_t)(v - kQBias);
}

static bool overlaps(const void *p, size_t pn, const void *q, size_t qn)
{
    const uintptr_t a = (uintptr_t)p, b = (uintptr_t)q;
    return a < b + qn && b < a + pn;
}

}  // namespace prom

extern "C" int prom_dw_conv(const int8_t *x, int n, int h, int w, int c, const int8_t *w_dw, int stride,
                            const prom_requant_t *rq, int8_t *y, void *stream)
{
    using namespace prom;
    if (!x || !w_dw || !rq || !rq->bias || !rq->mult || !rq->shift || !y) return PROM_EINVAL;
    if (n <= 0 || h <= 0 || w <= 0 || c <= 0 || (stride != 1 && stride != 2)) return PROM_EINVAL;
    if (rq->act_min < -128 || rq->act_max > 127 || rq->act_min > rq->act_max) return PROM_EINVAL;
    DwArgs a;
    a.x = x; a.w = w_dw; a.bias = rq->bias; a.mult = rq->mult; a.shift = rq->shift; a.y = y;
    a.N = n; a.H = h; a.W = w; a.C = c; a.stride = stride;
    a.Ho = (h - 1) / stride + 1;
    a.Wo = (w - 1) / stride + 1;
    a.lo_b = rq->act_min + kQBias;
    a.hi_b = rq->act_max + kQBias;
    const size_t xbytes = (size_t)n * h * w * c, ybytes = (size_t)n * a.Ho * a.Wo * c;
    if (xbytes >= ((size_t)1 << 40)) return PROM_EUNSUPPORTED;
    if (overlaps(y, ybytes, x, xbytes) || overlaps(y, ybytes, w_dw, (size_t)9 * c)) return PROM_EALIAS;
    hipStream_t st = static_cast<hipStream_t>(stream);
    clear_hip_error();
    const bool fast = (c % 4 == 0) && ((((uintptr_t)x | (uintptr_t)y | (uintptr_t)w_dw) & 3) == 0);
    if (fast) {
        // enough threads to fill the chip, otherwise long strips to amortise the per-thread setup
        const long long cols = (long long)n * a.Wo * (c / 4);
        int strip_rows = a.Ho;
        while (strip_rows > 1 && cols * ((a.Ho + strip_rows - 1) / strip_rows) < 256LL * 256 * 8)
            strip_rows = (strip_rows + 1) / 2;
        a.strip_rows = strip_rows;
        a.strips = (a.Ho + strip_rows - 1) / strip_rows;
        a.total = cols * a.strips;
        const long long blocks = (a.total + 255) / 256;
        if (blocks > (1LL << 31) - 1) return PROM_EUNSUPPORTED;
        hipLaunchKernelGGL(dw_kernel_c4, dim3((unsigned)blocks), dim3(256), 0, st, a);
    } else {
        a.strips = a.strip_rows = 0;
        a.total = (long long)ybytes;
        const long long blocks = (a.total + 255) / 256;
        if (blocks > (1LL << 31) - 1) return PROM_EUNSUPPORTED;
        hipLaunchKernelGGL(dw_kernel_generic, dim3((unsigned)blocks), dim3(256), 0, st, a);
    }
    return check_launch();
}
