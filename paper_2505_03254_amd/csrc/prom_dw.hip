// int8 depthwise 3x3 convolution (pad 1, stride 1 or 2), NHWC, with the exact integer
// requantisation epilogue.  This is the 8-bit convolution that sits between the two ternary
// pointwise convolutions of a block (paper Section 2; Section 3.1 "Depthwise Convolutions").
// It is not a dense contraction (9 taps per output, channels independent), so it runs on the
// vector ALU, and the work per output byte decides its speed.
//
// dw_kernel_v4: a thread owns 4 consecutive channels (one dword of the NHWC row) of one output
// column and ROWS consecutive output rows (4, or 8 at stride 1 on maps at least 8 rows high);
// lanes run over channels, then columns, so every load and store instruction of a wavefront
// covers one contiguous run.  The input rows feeding the outputs (ROWS + 2 at stride 1,
// 2*ROWS + 1 at stride 2) are loaded for each of the 3 kernel columns as one
// dword per pixel and transposed in registers (v_perm_b32, 4x4 bytes) so that a dword holds 4
// vertically neighbouring pixels of ONE channel; the 3 vertical taps of an output are then one
// v_dot4_i32_i8 against the dword (w[0][j], w[1][j], w[2][j], 0) of that channel and kernel
// column.  At stride 2 the 4-row blocks are disjoint and the byte window of an output row is cut
// out with v_alignbyte_b32; at stride 1 the blocks start at every second input row, so that
// even output rows read their block at byte 0 and odd ones at byte 1, against a copy of the
// weight dword shifted by one byte.  About 15 vector instructions per output byte (8 rows per
// thread) against about 32 for one multiply-add per tap.  Requantisation as in the pointwise kernels:
// t = acc*mult + C (one v_mad_i64_i32, C = bias*mult + 2^(30+shift)), q = (t >> 31) >> shift.
#include "prom.h"
#include "prom_device.h"
#include "prom_launch.h"
#include <type_traits>
#include <algorithm>
#include <vector>

namespace prom {

struct DwArgs {
    const int8_t *x;
    const int8_t *w;  // [3][3][C]
    const int32_t *bias;
    const int32_t *mult;
    const int32_t *mult_neg;  // PReLU: multiplier for acc + bias < 0, or nullptr
    const int32_t *shift;
    int8_t *y;
    int N, H, W, C, Ho, Wo, stride;
    int strips;      // row strips per image
    int strip_rows;  // output rows per strip
    int lo, hi;
    long long total;  // threads with work
};

// 4x4 byte transpose: in[p] = 4 channels of pixel p  ->  out[q] = channel q of pixels 0..3.
__device__ __forceinline__ void transpose4x4(const uint32_t (&in)[4], uint32_t (&out)[4])
{
    const uint32_t t0 = __builtin_amdgcn_perm(in[1], in[0], 0x05010400u);  // a0 b0 a1 b1
    const uint32_t t1 = __builtin_amdgcn_perm(in[1], in[0], 0x07030602u);  // a2 b2 a3 b3
    const uint32_t u0 = __builtin_amdgcn_perm(in[3], in[2], 0x05010400u);  // c0 d0 c1 d1
    const uint32_t u1 = __builtin_amdgcn_perm(in[3], in[2], 0x07030602u);  // c2 d2 c3 d3
    out[0] = __builtin_amdgcn_perm(u0, t0, 0x05040100u);
    out[1] = __builtin_amdgcn_perm(u0, t0, 0x07060302u);
    out[2] = __builtin_amdgcn_perm(u1, t1, 0x05040100u);
    out[3] = __builtin_amdgcn_perm(u1, t1, 0x07060302u);
}

// C % 4 == 0, 4-byte aligned x / y / w, one image below 2^31 bytes.
// Grid: x over Wo * C/4 (channels fastest, then output columns: the lanes of a wavefront read and
// write contiguous runs), y = group of ROWS output rows, z = image.  Row and image indices are
// uniform per workgroup, so every address is a per-lane column offset plus a scalar row offset;
// the image is addressed through a buffer resource of its own, which makes rows above and below
// it read as zero (and such output rows vanish) without a test, and a column outside the image
// gets an offset beyond the resource.
// (bx, by, bz): the workgroup's place in that grid.
template <int S, int ROWS = 4>
__device__ __forceinline__ void dw_body_v4(const DwArgs &a, const int bx, const int by, const int bz)
{
    constexpr int NPIX = S * (ROWS - 1) + 3;  // input rows feeding ROWS output rows
    constexpr int NB = (NPIX + 3) / 4;        // transposed dwords per channel
    constexpr int kFlags = 0x00020000;
    constexpr int kOob = 0x7ffff000;
    const int C4 = a.C >> 2;
    const int t = bx * 256 + threadIdx.x;
    if (t >= a.Wo * C4) return;
    const int ox = t / C4;
    const int c = (t - ox * C4) * 4;
    const int oy0 = by * ROWS;
    const int n = bz;

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.x) + (long long)n * a.H * a.W * a.C, 0, a.H * a.W * a.C, kFlags);
    const __amdgpu_buffer_rsrc_t ry =
        __builtin_amdgcn_make_buffer_rsrc(a.y + (long long)n * a.Ho * a.Wo * a.C, 0, a.Ho * a.Wo * a.C, kFlags);
    const __amdgpu_buffer_rsrc_t rw =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a.w), 0, 9 * a.C, kFlags);

    // activations first: 3 columns x NPIX rows
    const int rowbytes = a.W * a.C;
    const int iy0 = oy0 * S - 1;
    uint32_t v[3][NB * 4];
#pragma unroll
    for (int jx = 0; jx < 3; ++jx) {
        const int ix = ox * S + jx - 1;
        const int coff = (ix >= 0 && ix < a.W) ? ix * a.C + c : kOob;
#pragma unroll
        for (int p = 0; p < NB * 4; ++p)
            v[jx][p] = p < NPIX ? (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rx, coff, (iy0 + p) * rowbytes, 0) : 0u;
    }
    // weights: wcol[jx][q] = (w[0][jx][c+q], w[1][jx][c+q], w[2][jx][c+q], 0)
    uint32_t wcol[3][4];
#pragma unroll
    for (int jx = 0; jx < 3; ++jx) {
        uint32_t in[4];
#pragma unroll
        for (int i = 0; i < 3; ++i) in[i] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rw, c, (i * 3 + jx) * a.C, 0);
        in[3] = 0;
        transpose4x4(in, wcol[jx]);
    }
    // requantisation: C = bias*mult + 2^(30+shift), mult, shift per channel
    const v4i pb = *reinterpret_cast<const v4i *>(a.bias + c);
    const v4i pm = *reinterpret_cast<const v4i *>(a.mult + c);
    const v4i ps = *reinterpret_cast<const v4i *>(a.shift + c);
    long long Cq[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) Cq[q] = (long long)pb[q] * pm[q] + (1LL << (30 + ps[q]));
    const int lo = in_vgpr(a.lo), hi = in_vgpr(a.hi);

    int acc[ROWS][4];  // [output row][channel]
    if constexpr (S == 1) {
        // Stride 1: blocks of 4 input rows that start at every second row (rows 0-3, 2-5, ...), so
        // that output row o finds its 3 rows in block o/2 at byte 0 (o even) or byte 1 (o odd),
        // and a second copy of the weight dwords shifted by one byte takes the odd rows: one more
        // transpose per column instead of a v_alignbyte_b32 for three of four windows.
        uint32_t wodd[3][4];
#pragma unroll
        for (int jx = 0; jx < 3; ++jx)
#pragma unroll
            for (int q = 0; q < 4; ++q) wodd[jx][q] = wcol[jx][q] << 8;
#pragma unroll
        for (int jx = 0; jx < 3; ++jx) {
#pragma unroll
            for (int b = 0; b < ROWS / 2; ++b) {
                const uint32_t in[4] = {v[jx][2 * b], v[jx][2 * b + 1], v[jx][2 * b + 2], v[jx][2 * b + 3]};
                uint32_t tr[4];
                transpose4x4(in, tr);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    acc[2 * b][q] = __builtin_amdgcn_sdot4((int)tr[q], (int)wcol[jx][q], jx == 0 ? 0 : acc[2 * b][q], false);
                    acc[2 * b + 1][q] =
                        __builtin_amdgcn_sdot4((int)tr[q], (int)wodd[jx][q], jx == 0 ? 0 : acc[2 * b + 1][q], false);
                }
            }
        }
    } else {
#pragma unroll
        for (int jx = 0; jx < 3; ++jx) {
            uint32_t tr[NB][4];
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const uint32_t in[4] = {v[jx][4 * b], v[jx][4 * b + 1], v[jx][4 * b + 2], v[jx][4 * b + 3]};
                transpose4x4(in, tr[b]);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
#pragma unroll
                for (int o = 0; o < ROWS; ++o) {
                    // byte window of channel q for output row o: input rows S*o .. S*o+3 of this column
                    const int first = S * o;
                    const int b = first >> 2, sh = first & 3;
                    const uint32_t w =
                        sh == 0 ? tr[b][q] : __builtin_amdgcn_alignbyte(tr[b + 1 < NB ? b + 1 : b][q], tr[b][q], sh);
                    acc[o][q] = __builtin_amdgcn_sdot4((int)w, (int)wcol[jx][q], jx == 0 ? 0 : acc[o][q], false);
                }
            }
        }
    }
    const int yoff = ox * a.C + c;
    const int yrow = a.Wo * a.C;
    if (a.mult_neg) {  // PReLU layer (uniform over the launch)
        const v4i pn = *reinterpret_cast<const v4i *>(a.mult_neg + c);
#pragma unroll
        for (int o = 0; o < ROWS; ++o) {
            int out[4];
#pragma unroll
            for (int q = 0; q < 4; ++q)
                out[q] = requant_prelu_i64(acc[o][q], v4i{pb[q], pm[q], pn[q], ps[q]}, lo, hi);
            __builtin_amdgcn_raw_buffer_store_b32((int)pack4_low_bytes(out[0], out[1], out[2], out[3]), ry, yoff,
                                                  (oy0 + o) * yrow, 0);
        }
        return;
    }
    // q = (t >> 31) >> shift; where every shift of the wavefront's channels is at least 1 the high
    // dword of t shifted by shift-1 is the same number and one instruction less per output.
    const bool any_shift0 =
        __builtin_amdgcn_ballot_w64((ps[0] == 0) | (ps[1] == 0) | (ps[2] == 0) | (ps[3] == 0)) != 0;
    auto epilogue = [&](auto general_tag) {
        constexpr bool GENERAL = decltype(general_tag)::value;
        int sh[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) sh[q] = GENERAL ? ps[q] : ps[q] - 1;
#pragma unroll
        for (int o = 0; o < ROWS; ++o) {
            int out[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const long long tq = (long long)acc[o][q] * (long long)pm[q] + Cq[q];
                out[q] = med3_i32((GENERAL ? (int)(tq >> 31) : (int)(tq >> 32)) >> sh[q], lo, hi);
            }
            // an output row below the image is beyond the resource and is dropped
            __builtin_amdgcn_raw_buffer_store_b32((int)pack4_low_bytes(out[0], out[1], out[2], out[3]), ry, yoff,
                                                  (oy0 + o) * yrow, 0);
        }
    };
    if (any_shift0)
        epilogue(std::true_type{});
    else
        epilogue(std::false_type{});
}

// xb == 0: the grid is (columns x channels, row strips, images).  xb > 0 (that many workgroups per row
// strip, images a multiple of 8): a 1-D grid in which 8 consecutive workgroups are the same place in
// 8 images -- workgroups go round-robin over the 8 XCDs, so each XCD has whole images and the
// workgroups that share input lines share its L2.
template <int S, int ROWS = 4>
__global__ __launch_bounds__(256) void dw_kernel_v4(const DwArgs a, const int xb)
{
    if (xb > 0) {
        const int l = blockIdx.x;
        const int per_img = xb * a.strips;
        const int k = l >> 3;
        const int within = k % per_img;
        dw_body_v4<S, ROWS>(a, within % xb, within / xb, (k / per_img) * 8 + (l & 7));
    } else {
        dw_body_v4<S, ROWS>(a, blockIdx.x, blockIdx.y, blockIdx.z);
    }
}

// Several independent depthwise layers in one launch: workgroups [start[i], start[i+1]) run layer i
// with the grid (xblocks, strips, images) it would have on its own.  The launch, first-load and
// write-back latencies of a small layer (5 us of a 7 us launch at 14x14 and 7x7) overlap with the
// other layers' work.
constexpr int kDwMaxBatch = 32;
struct DwBatchArgs {
    int count;
    int start[kDwMaxBatch + 1];
    int xblocks[kDwMaxBatch];
    DwArgs layer[kDwMaxBatch];
};

__global__ __launch_bounds__(256) void dw_batch_kernel(const DwBatchArgs b)
{
    const int bid = blockIdx.x;
    int i = 0;
    while (i + 1 < b.count && bid >= b.start[i + 1]) ++i;
    const DwArgs a = b.layer[i];  // a copy: a reference into the by-value argument can force all of it into scratch memory
    const int l = bid - b.start[i];
    const int xb = b.xblocks[i];
    // Workgroups go round-robin over the 8 XCDs, each with an L2 of its own.  With x fastest, the
    // workgroups that share input (column neighbours in a row strip, strips above and below) sit on
    // different XCDs and every shared line comes from HBM more than once (measured: 1.45 times the
    // input).  So 8 consecutive workgroups are the same place in 8 images: an XCD has whole images,
    // their workgroups one after the other.  (start[] are multiples of 8.)
    int bx, by, bz;
    if ((a.N & 7) == 0) {
        const int per_img = xb * a.strips;
        const int k = l >> 3;
        const int within = k % per_img;
        bz = (k / per_img) * 8 + (l & 7);
        bx = within % xb;
        by = within / xb;
    } else {
        const int r = l / xb;
        bx = l % xb;
        by = r % a.strips;
        bz = r / a.strips;
    }
    if (bz >= a.N) return;  // padding between the layers of the launch
    if (a.stride == 2)
        dw_body_v4<2, 4>(a, bx, by, bz);
    else if (a.strip_rows == 8)
        dw_body_v4<1, 8>(a, bx, by, bz);
    else
        dw_body_v4<1, 4>(a, bx, by, bz);
}

// Any C and alignment: one thread per output element.
__global__ __launch_bounds__(256) void dw_kernel_generic(const DwArgs a)
{
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
    const int m = (a.mult_neg && acc < 0) ? a.mult_neg[c] : a.mult[c];
    a.y[tid] = (int8_t)requant_s_i64(acc, m, a.shift[c], a.lo, a.hi);
}

static bool overlaps(const void *p, size_t pn, const void *q, size_t qn)
{
    const uintptr_t a = (uintptr_t)p, b = (uintptr_t)q;
    return a < b + qn && b < a + pn;
}

}  // namespace prom

// The limits of prom_dw_conv that depend on the shape alone (the vector kernel's grid is
// (columns x channels, strips of rows, images); the one-thread-per-output kernel has a 1-D grid).
int prom::dw_shape_check(int n, int h, int w, int c, int stride)
{
    if (n <= 0 || h <= 0 || w <= 0 || c <= 0 || (stride != 1 && stride != 2)) return PROM_EINVAL;
    const int ho = (h - 1) / stride + 1, wo = (w - 1) / stride + 1;
    const size_t xbytes = (size_t)n * h * w * c, ybytes = (size_t)n * ho * wo * c;
    if (xbytes >= ((size_t)1 << 40)) return PROM_EUNSUPPORTED;
    if (n > 65535 || (ho + 3) / 4 > 65535) return PROM_EUNSUPPORTED;  // (either kernel may be taken)
    if (((long long)wo * (c / 4) + 255) / 256 > (1LL << 31) - 1) return PROM_EUNSUPPORTED;
    if (((long long)ybytes + 255) / 256 > (1LL << 31) - 1) return PROM_EUNSUPPORTED;
    return PROM_OK;
}

namespace prom {

struct DwLaunch {
    DwArgs a;
    bool fast;
    dim3 grid;
    size_t xbytes, ybytes;
};

// Validate the arguments of one depthwise layer and fill its launch description; launches nothing.
static int dw_prepare(const int8_t *x, int n, int h, int w, int c, const int8_t *w_dw, int stride,
                      const prom_requant_t *rq, int8_t *y, DwLaunch &L)
{
    if (!x || !w_dw || !rq || !rq->bias || !rq->mult || !rq->shift || !y) return PROM_EINVAL;
    if (n <= 0 || h <= 0 || w <= 0 || c <= 0 || (stride != 1 && stride != 2)) return PROM_EINVAL;
    if (rq->act_min < -128 || rq->act_max > 127 || rq->act_min > rq->act_max) return PROM_EINVAL;
    DwArgs &a = L.a;
    a.x = x; a.w = w_dw; a.bias = rq->bias; a.mult = rq->mult; a.mult_neg = rq->mult_neg; a.shift = rq->shift; a.y = y;
    a.N = n; a.H = h; a.W = w; a.C = c; a.stride = stride;
    a.Ho = (h - 1) / stride + 1;
    a.Wo = (w - 1) / stride + 1;
    a.lo = rq->act_min;
    a.hi = rq->act_max;
    L.xbytes = (size_t)n * h * w * c;
    L.ybytes = (size_t)n * a.Ho * a.Wo * c;
    if (L.xbytes >= ((size_t)1 << 40)) return PROM_EUNSUPPORTED;
    if (overlaps(y, L.ybytes, x, L.xbytes) || overlaps(y, L.ybytes, w_dw, (size_t)9 * c)) return PROM_EALIAS;
    // the fast kernel addresses one image with 32-bit offsets and reads the parameters 16 bytes at a time
    L.fast = (c % 4 == 0) && ((((uintptr_t)x | (uintptr_t)y | (uintptr_t)w_dw) & 3) == 0) &&
             ((((uintptr_t)rq->bias | (uintptr_t)rq->mult | (uintptr_t)rq->mult_neg | (uintptr_t)rq->shift) & 15) == 0) &&
             (long long)h * w * c < (1LL << 31) - (1LL << 24) && n <= 65535;
    if (L.fast) {
        // stride 1: 8 output rows per thread where the map is high enough (fewer instructions per
        // output: the transposes and the weights are shared by twice as many rows)
        const int rows = (stride == 1 && a.Ho >= 8) ? 8 : 4;
        a.strip_rows = rows;
        a.strips = (a.Ho + rows - 1) / rows;
        a.total = 0;
        const long long xblocks = ((long long)a.Wo * (c / 4) + 255) / 256;
        if (xblocks > (1LL << 31) - 1 || a.strips > 65535 || n > 65535) return PROM_EUNSUPPORTED;
        L.grid = dim3((unsigned)xblocks, (unsigned)a.strips, (unsigned)n);
    } else {
        a.strips = a.strip_rows = 0;
        a.total = (long long)L.ybytes;
        const long long blocks = (a.total + 255) / 256;
        if (blocks > (1LL << 31) - 1) return PROM_EUNSUPPORTED;
        L.grid = dim3((unsigned)blocks);
    }
    return PROM_OK;
}

static void dw_launch(const DwLaunch &L, hipStream_t st)
{
    const DwArgs &a = L.a;
    if (!L.fast)
        hipLaunchKernelGGL(dw_kernel_generic, L.grid, dim3(256), 0, st, a);
    else {
        const long long blocks = (long long)L.grid.x * L.grid.y * L.grid.z;
        const bool flat = (a.N & 7) == 0 && blocks <= (1LL << 30);
        const dim3 grid = flat ? dim3((unsigned)blocks) : L.grid;
        const int xb = flat ? (int)L.grid.x : 0;
        if (a.stride == 1 && a.strip_rows == 8)
            hipLaunchKernelGGL((dw_kernel_v4<1, 8>), grid, dim3(256), 0, st, a, xb);
        else if (a.stride == 1)
            hipLaunchKernelGGL(dw_kernel_v4<1>, grid, dim3(256), 0, st, a, xb);
        else
            hipLaunchKernelGGL(dw_kernel_v4<2>, grid, dim3(256), 0, st, a, xb);
    }
}

// true if running `b` concurrently with `a` could change a result
static bool dw_conflicts(const DwLaunch &p, const DwLaunch &q)
{
    const DwArgs &a = p.a, &b = q.a;
    if (overlaps(a.y, p.ybytes, b.y, q.ybytes) || overlaps(a.y, p.ybytes, b.x, q.xbytes) ||
        overlaps(b.y, q.ybytes, a.x, p.xbytes))
        return true;
    auto writes_inputs = [](const DwArgs &w, size_t wn, const DwArgs &r) {
        if (overlaps(w.y, wn, r.w, (size_t)9 * r.C)) return true;
        const int32_t *arrs[4] = {r.bias, r.mult, r.shift, r.mult_neg};
        for (const int32_t *q4 : arrs)
            if (q4 && overlaps(w.y, wn, q4, (size_t)r.C * 4)) return true;
        return false;
    };
    return writes_inputs(a, p.ybytes, b) || writes_inputs(b, q.ybytes, a);
}

}  // namespace prom

extern "C" int prom_dw_conv(const int8_t *x, int n, int h, int w, int c, const int8_t *w_dw, int stride,
                            const prom_requant_t *rq, int8_t *y, void *stream)
{
    using namespace prom;
    DwLaunch L;
    const int rc = dw_prepare(x, n, h, w, c, w_dw, stride, rq, y, L);
    if (rc != PROM_OK) return rc;
    clear_hip_error();
    dw_launch(L, static_cast<hipStream_t>(stream));
    return check_launch();
}

extern "C" int prom_dw_conv_sequence(const prom_dw_layer_t *layers, int count, int *bad_layer, void *stream)
{
    using namespace prom;
    if (bad_layer) *bad_layer = -1;
    if (count < 0 || (count > 0 && !layers)) return PROM_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    static thread_local std::vector<DwLaunch> prepared;
    prepared.resize((size_t)count);
    for (int i = 0; i < count; ++i) {
        const prom_dw_layer_t &l = layers[i];
        const int rc = dw_prepare(l.x, l.n, l.h, l.w, l.c, l.w_dw, l.stride, &l.rq, l.y, prepared[(size_t)i]);
        if (rc != PROM_OK) {
            if (bad_layer) *bad_layer = i;
            return rc;
        }
    }
    // Consecutive layers the vector kernel takes and that do not touch each other's data share a
    // launch (at most kDwMaxBatch of them, and workgroup counts that fit a 1-D grid).
    static thread_local DwBatchArgs b;
    clear_hip_error();
    int i = 0;
    while (i < count) {
        int j = i;
        long long blocks = 0;
        while (j < count && j - i < kDwMaxBatch && prepared[(size_t)j].fast) {
            const DwLaunch &L = prepared[(size_t)j];
            bool clash = false;
            for (int k = i; k < j && !clash; ++k) clash = dw_conflicts(prepared[(size_t)k], L);
            const long long nb = (long long)L.grid.x * L.grid.y * L.grid.z;
            if (clash || blocks + nb > (1LL << 30)) break;
            blocks += nb;
            ++j;
        }
        if (j - i >= 2) {
            b.count = j - i;
            // the members with the least work first: a small layer is a latency chain per workgroup and
            // would otherwise end the launch alone
            int order[kDwMaxBatch];
            for (int k = 0; k < j - i; ++k) order[k] = i + k;
            std::stable_sort(order, order + (j - i), [&](int p, int q) {
                return prepared[(size_t)p].xbytes + prepared[(size_t)p].ybytes <
                       prepared[(size_t)q].xbytes + prepared[(size_t)q].ybytes;
            });
            int start = 0;
            for (int k = 0; k < j - i; ++k) {
                const DwLaunch &L = prepared[(size_t)order[k]];
                b.layer[k] = L.a;
                b.xblocks[k] = (int)L.grid.x;
                b.start[k] = start;
                start += (int)((L.grid.x * L.grid.y * L.grid.z + 7) / 8 * 8);
            }
            b.start[j - i] = start;
            hipLaunchKernelGGL(dw_batch_kernel, dim3((unsigned)start), dim3(256), 0, st, b);
            i = j;
        } else {
            dw_launch(prepared[(size_t)i], st);
            ++i;
        }
        if (check_launch() != PROM_OK) {
            if (bad_layer) *bad_layer = i - 1;
            return PROM_EHIP;
        }
    }
    return PROM_OK;
}
