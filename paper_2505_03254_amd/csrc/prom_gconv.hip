// int8 grouped 3x3 convolution (pad 1, stride 1 or 2), NHWC, as many output as input channels,
// groups of gs channels, with the integer requantisation epilogue (plain or PReLU).  RegNet and
// ResNeXt have this layer where MobileNetV2 has the depthwise convolution (paper Section 2); its
// weights are 8-bit with one scale per output channel (Section 3.1, Eq. 4-5).
//
// Kernels, by group size: 4, 8, 16 -> gconv_tapk_kernel (matrix cores, the kernel taps in the k
// dimension); 32, 64 -> gconv_mfma_kernel (matrix cores, one k step per tap); other multiples of 4
// -> gconv_kernel_v4 (vector ALU); anything else -> gconv_kernel_generic; 1 is prom_dw_conv.  The
// *_batch_kernel forms run several independent layers in one launch (prom_gconv3x3_sequence).
//
// gconv_kernel_v4: a thread owns 4 consecutive output channels (they lie in one group, gs being
// a multiple of 4) of one output column and 4 consecutive output rows; lanes run over channels,
// then columns.  For each of the 3 kernel columns it loads the gs input bytes of its group (in
// chunks of up to 16) for the 6 (stride 1) or 9 (stride 2) input rows that feed its outputs -- lanes of one group read
// the same bytes, lanes of neighbouring groups the bytes next to them, so a wavefront's load
// covers one contiguous run -- and, per kernel row, the 4*gs weight bytes of its 4 channels,
// which are reused for the 4 output rows.  The input channels of a group are contiguous in both
// operands, so 4 of them are one v_dot4_i32_i8 with no unpacking: 9*gs/4 instructions per
// output byte.  From gs = 16 on that is more vector ALU time than the HBM needs for the bytes
// (36 instructions per output byte at gs = 16), i.e. the kernel is ALU bound there.
#include "prom.h"
#include "prom_device.h"
#include "prom_launch.h"

#include <algorithm>
#include <mutex>
#include <type_traits>
#include <vector>

namespace prom {

struct GconvArgs {
    const int8_t *x;
    const int8_t *w;  // [3][3][C][gs]
    const v4i *wfrag;  // the same weights in MFMA operand order (prom_gconv_pack), or nullptr
    const int32_t *bias;
    const int32_t *mult;
    const int32_t *mult_neg;  // or nullptr
    const int32_t *shift;
    int8_t *y;
    int N, H, W, C, Ho, Wo, stride, gs;
    int lo, hi;
    long long total;  // outputs (generic kernel)
};

// n consecutive dwords at byte offset voff (+ scalar offset soff) of a buffer, with the widest
// loads n allows.  Out-of-range dwords read as zero.
template <int N>
__device__ __forceinline__ void load_dwords(const __amdgpu_buffer_rsrc_t r, int voff, int soff, uint32_t (&out)[N])
{
    constexpr int kOob = 0x7ffff000;
    if constexpr (N % 4 == 0) {
#pragma unroll
        for (int k = 0; k < N; k += 4) {
            const v4i v = __builtin_amdgcn_raw_buffer_load_b128(r, min((unsigned)voff + 4u * k, (unsigned)kOob), soff, 0);
            out[k] = v[0]; out[k + 1] = v[1]; out[k + 2] = v[2]; out[k + 3] = v[3];
        }
    } else if constexpr (N % 2 == 0) {
#pragma unroll
        for (int k = 0; k < N; k += 2) {
            const v2i v = __builtin_amdgcn_raw_buffer_load_b64(r, min((unsigned)voff + 4u * k, (unsigned)kOob), soff, 0);
            out[k] = v[0]; out[k + 1] = v[1];
        }
    } else {
#pragma unroll
        for (int k = 0; k < N; ++k)
            out[k] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(r, min((unsigned)voff + 4u * k, (unsigned)kOob), soff, 0);
    }
}

// C % 4 == 0, gs % 4 == 0, 4-byte aligned x / y / w, 16-byte aligned parameters, one image and
// the weights below 2^31 bytes.  The input channels of a group are taken in chunks of 4*KC
// (KC dwords per load); ONE: the group is a single chunk (gs == 4*KC), and the weights of the
// lane's 4 channels are then one contiguous run.  The loops over the kernel columns and the
// chunks stay loops: unrolled, the compiler issues every load of the thread up front and needs
// several hundred registers.
// Grid: x over Wo * C/4 (channels fastest, then output columns), y = group of 4 output rows,
// z = image.  Row and image indices are uniform per workgroup; the image is addressed through a
// buffer resource of its own, so rows above and below it read as zero and output rows below it
// are dropped, and a column outside the image gets an offset beyond the resource.
template <int S, int KC, bool ONE>
__global__ __launch_bounds__(256, (KC == 4 ? 3 : 4)) void gconv_kernel_v4(const GconvArgs a)
{
    constexpr int NPIX = S == 1 ? 6 : 9;  // input rows feeding 4 output rows
    constexpr int kFlags = 0x00020000;
    constexpr int kOob = 0x7ffff000;
    const int GS = ONE ? 4 * KC : a.gs;
    const int nchunk = ONE ? 1 : GS / (4 * KC);
    const int C4 = a.C >> 2;
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= a.Wo * C4) return;
    const int ox = t / C4;
    const int c = (t - ox * C4) * 4;  // the lane's first output channel
    const int first = (c / GS) * GS;  // first input channel of its group
    const int oy0 = blockIdx.y * 4;
    const int n = blockIdx.z;

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.x) + (long long)n * a.H * a.W * a.C, 0, a.H * a.W * a.C, kFlags);
    const __amdgpu_buffer_rsrc_t ry =
        __builtin_amdgcn_make_buffer_rsrc(a.y + (long long)n * a.Ho * a.Wo * a.C, 0, a.Ho * a.Wo * a.C, kFlags);
    const __amdgpu_buffer_rsrc_t rw =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a.w), 0, 9 * a.C * GS, kFlags);

    const int rowbytes = a.W * a.C;
    const int iy0 = oy0 * S - 1;
    int acc[4][4];  // [output row][channel]
#pragma unroll
    for (int o = 0; o < 4; ++o)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[o][r] = 0;

#pragma nounroll
    for (int jx = 0; jx < 3; ++jx) {
        const int ix = ox * S + jx - 1;
        const int coff0 = (ix >= 0 && ix < a.W) ? ix * a.C + first : kOob;
#pragma nounroll
        for (int kc = 0; kc < nchunk; ++kc) {
            const int coff = (int)min((unsigned)coff0 + (unsigned)(kc * 4 * KC), (unsigned)kOob);
            uint32_t v[NPIX][KC];
#pragma unroll
            for (int p = 0; p < NPIX; ++p) load_dwords<KC>(rx, coff, (iy0 + p) * rowbytes, v[p]);
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                uint32_t wr[4][KC];  // [channel r][k]
                const int wrow = (i * 3 + jx) * a.C * GS;  // uniform
                if constexpr (ONE) {
                    uint32_t flat[4 * KC];
                    load_dwords<4 * KC>(rw, c * GS, wrow, flat);
#pragma unroll
                    for (int r = 0; r < 4; ++r)
#pragma unroll
                        for (int k = 0; k < KC; ++k) wr[r][k] = flat[r * KC + k];
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) load_dwords<KC>(rw, (c + r) * GS + kc * 4 * KC, wrow, wr[r]);
                }
#pragma unroll
                for (int o = 0; o < 4; ++o)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
#pragma unroll
                        for (int k = 0; k < KC; ++k)
                            acc[o][r] = __builtin_amdgcn_sdot4((int)v[S * o + i][k], (int)wr[r][k], acc[o][r], false);
            }
        }
    }

    const v4i pb = *reinterpret_cast<const v4i *>(a.bias + c);
    const v4i pm = *reinterpret_cast<const v4i *>(a.mult + c);
    const v4i ps = *reinterpret_cast<const v4i *>(a.shift + c);
    v4i pn = {0, 0, 0, 0};
    const bool prelu = a.mult_neg != nullptr;  // uniform over the launch
    if (prelu) pn = *reinterpret_cast<const v4i *>(a.mult_neg + c);
    const int lo = in_vgpr(a.lo), hi = in_vgpr(a.hi);
    const int yoff = ox * a.C + c;
    const int yrow = a.Wo * a.C;
#pragma unroll
    for (int o = 0; o < 4; ++o) {
        int out[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const v4i pr = requant_params(pb[r], pm[r], pn[r], ps[r], prelu);
            out[r] = prelu ? requant_prelu_i64(acc[o][r], pr, lo, hi) : requant_i64<true>(acc[o][r], pr, lo, hi);
        }
        // an output row below the image is beyond the resource and is dropped
        __builtin_amdgcn_raw_buffer_store_b32((int)pack4_low_bytes(out[0], out[1], out[2], out[3]), ry, yoff,
                                              (oy0 + o) * yrow, 0);
    }
}

// ---- gconv_mfma_kernel: group sizes 4, 8, 16, 32, 64 on the matrix cores -------------------------
// A block of 64 output channels only sees the same 64 input channels (the groups divide 64), so
// per kernel tap the layer is a [64 x 64] block-diagonal int8 matrix applied to the 64 input bytes
// of the pixel under that tap: 9 k steps of v_mfma_i32_16x16x64_i8, one per tap.  The matrix cores
// do 64/gs times the necessary multiply-adds and are still far from being the limit; what has to
// be kept small is the number of times an input byte is fetched, 9 if every tap loads from
// global memory (measured: the texture addresser, which takes a 16-byte-per-lane load lane by
// lane, was then 70 % busy and set the time).  So a workgroup stages the input rows of a band of
// output rows once in LDS (64 channels per pixel, a zero column left and right, zero rows above
// and below the image), and the B operands of all 9 taps are 16-byte LDS reads at the lane's
// pixel plus the tap's offset; the block's weights are decoded once per workgroup into LDS
// fragments (zeros outside the groups) and serve every band the workgroup takes.
// Tile rows are permuted as in the pointwise kernels: row 4g + r of tile t is channel
// 16g + 4t + r of the block, so that a lane's 16 outputs of a pixel are 16 contiguous bytes.
// A wavefront iteration covers PT tiles of 16 consecutive output pixels of the band (in row-major
// order, so ragged widths waste nothing), a fragment read serving PT MFMAs.
// Requirements (host): gs in {4, 8, 16, 32, 64}, C % 4 == 0, x and y below 2^31 - 2^24 bytes,
// 4-byte aligned x / y / w, the band geometry of GconvBand.
struct GconvBand {
    int ncb;         // blocks of 64 channels
    int wgs_per_cb;  // workgroups per channel block
    int R;           // output rows per band
    int RI;          // input rows per band = (R-1)*stride + 3
    int bands;       // bands per image
    int G;           // images per unit of work (above 1 only when a band is the whole image)
    int units;       // units of work per channel block
    int swizzle;     // XCD-aware order of the workgroups (wgs_per_cb % 8 == 0)
    // floor(2^31 / d) + 1 for d = Wo and d = R * Wo: n / d = (n * this) >> 31 for every n with
    // n * d < 2^31 (the pixels of a unit are a few thousand at most)
    unsigned magic_wo, magic_img;
};

constexpr int kGconvFragBytes = 4 * 9 * 64 * 16;
constexpr int kGconvParBytes = 64 * 16;
constexpr int kGconvPieces = 9;  // 16-byte pieces of a staged band per thread

__device__ __forceinline__ void gconv_mfma_body(const GconvArgs &a, const GconvBand &bd, const int block)
{
    constexpr int kFlags = 0x00020000;
    constexpr int kOob = 0x7ffff000;
    constexpr int PT = 2;
    constexpr int NK = kGconvPieces;
    extern __shared__ __align__(16) unsigned char lds[];
    v4i *frag = reinterpret_cast<v4i *>(lds);                                    // [tile t][tap s][lane]
    v4i *lpar = reinterpret_cast<v4i *>(lds + kGconvFragBytes);                  // [64] parameters
    unsigned char *xt = lds + kGconvFragBytes + kGconvParBytes;                  // [G][RI][W+2][64] input band(s)
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, g = lane >> 4;
    // Workgroups go round-robin over the 8 XCDs, each with an L2 of its own.  A pixel's channel
    // blocks are neighbours in memory (two of them share a 128-byte line), so the workgroups of all
    // channel blocks with the same units sit on one XCD (grids that are a multiple of 8 per channel
    // block); otherwise every line comes from HBM once per channel block.
    int cb, wg;
    if (bd.swizzle) {
        const int k = block >> 3;
        cb = k % bd.ncb;
        wg = (k / bd.ncb) * 8 + (block & 7);
    } else {
        cb = block % bd.ncb;
        wg = block / bd.ncb;
    }
    if (wg >= bd.wgs_per_cb) return;  // padding of a shared launch
    const int C = a.C, GS = a.gs, S = a.stride, W = a.W, Wo = a.Wo;
    const int W2 = W + 2;
    const int cbase = cb * 64;
    const bool prelu = a.mult_neg != nullptr;
    const int row_items = W2 * 4;              // 16-byte pieces per staged input row
    const int img_items = bd.RI * row_items;   // pieces per staged image band
    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a.x), 0, a.N * a.H * W * C, kFlags);
    const __amdgpu_buffer_rsrc_t ry =
        __builtin_amdgcn_make_buffer_rsrc(a.y, 0, a.N * a.Ho * Wo * C, kFlags);

    // Unit of work u: one band of one image, or (small images) the whole of up to G images.
    struct Unit { int img0, count, ro0, rows_out; };
    auto unit_of = [&](int u) {
        Unit q;
        if (bd.G > 1) {
            q.img0 = u * bd.G;
            q.count = min(bd.G, a.N - q.img0);
            q.ro0 = 0;
        } else {
            q.img0 = u / bd.bands;
            q.count = 1;
            q.ro0 = (u - q.img0 * bd.bands) * bd.R;
        }
        q.rows_out = min(bd.R, a.Ho - q.ro0);
        return q;
    };
    // The band of a unit is fetched into registers, all 16-byte pieces of a thread back to back
    // (one memory latency per band, not one per row), and written to LDS later: the fetch of the
    // next unit is in flight while the current one is computed, and the first fetch while the
    // weights are staged.  Pixels outside the image and channels beyond C are zeros.
    v4i piece[NK];
    auto fetch_band = [&](int u) {
        const Unit q = unit_of(u);
        const int ri0 = q.ro0 * S - 1;  // first input row (may be -1)
        const int npiece = q.count * img_items;
#pragma unroll
        for (int k = 0; k < NK; ++k) {
            const int pc = k * 256 + tid;
            const int gi = pc / img_items;
            const int rem = pc - gi * img_items;
            const int row = rem / row_items;
            const int it = rem - row * row_items;
            const int col = it >> 2, qd = it & 3;  // staged column 0 is image column -1
            const int iy = ri0 + row;
            const bool ok = pc < npiece && iy >= 0 && iy < a.H && col >= 1 && col <= W && cbase + 16 * qd < C;
            const int off = (((q.img0 + gi) * a.H + iy) * W + col - 1) * C + cbase + 16 * qd;
            piece[k] = __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? off : kOob, 0, 0);
        }
    };
    // ---- weights of the block -> MFMA A fragments: a plain copy when the caller has prepared them,
    // else decoded here ----------------------------------------------------------------------------
    if (a.wfrag) {
        const v4i *src = a.wfrag + (long long)cb * (4 * 9 * 64);
        v4i tmp[9];
#pragma unroll
        for (int k = 0; k < 9; ++k) tmp[k] = src[k * 256 + tid];
#pragma unroll
        for (int k = 0; k < 9; ++k) frag[k * 256 + tid] = tmp[k];
    } else
    for (int idx = tid; idx < 4 * 9 * 64; idx += 256) {
        const int l = idx & 63, ts = idx >> 6, s = ts % 9, t = ts / 9;
        const int i = l & 15, kg = l >> 4;
        const int oc = cbase + 16 * (i >> 2) + 4 * t + (i & 3);
        const int gfirst = (oc / GS) * GS;  // first input channel of the output channel's group
        v4i e = {0, 0, 0, 0};
        if (oc < C) {
            const int8_t *wrow = a.w + ((long long)s * C + oc) * GS;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int ic = cbase + 16 * kg + 4 * d;  // 4 input channels; GS % 4 == 0: all in or all out
                if (ic >= gfirst && ic < gfirst + GS) e[d] = *reinterpret_cast<const int *>(wrow + (ic - gfirst));
            }
        }
        frag[idx] = e;
    }
    if (tid < 64) {
        const int c = cbase + tid;
        v4i p = {0, 0, 0, 1};
        if (c < C) p = requant_params(a.bias[c], a.mult[c], prelu ? a.mult_neg[c] : 0, a.shift[c], prelu);
        lpar[tid] = p;
    }
    if (wg < bd.units) fetch_band(wg);
    __syncthreads();

    v4i par[4][4];  // [tile t][r]: channel 16g + 4t + r
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) par[t][r] = lpar[16 * g + 4 * t + r];
    const int lo = in_vgpr(a.lo), hi = in_vgpr(a.hi);
    const int cl = cbase + 16 * g;  // the lane's first output channel

    // one instance of the loop per epilogue form: no branch per output
    auto run = [&](auto prelu_tag) {
        constexpr bool PRELU = decltype(prelu_tag)::value;
        for (int u = wg; u < bd.units; u += bd.wgs_per_cb) {
            const Unit q = unit_of(u);
            const int npiece = q.count * img_items;
            __syncthreads();  // the readers of the previous band are done
#pragma unroll
            for (int k = 0; k < NK; ++k) {
                const int pc = k * 256 + tid;
                if (pc < npiece) *reinterpret_cast<v4i *>(xt + pc * 16) = piece[k];
            }
            __syncthreads();
            if (u + bd.wgs_per_cb < bd.units) fetch_band(u + bd.wgs_per_cb);
            // ---- the unit's output pixels in tiles of 16, PT tiles per wavefront iteration ---------
            const int img_pix = q.rows_out * Wo;
            const int npix = q.count * img_pix;
            const int ngrp = (npix + 16 * PT - 1) / (16 * PT);
            for (int grp = wave; grp < ngrp; grp += 4) {
                int lbase[PT], yo[PT];
                bool valid[PT];
#pragma unroll
                for (int p = 0; p < PT; ++p) {
                    const int idx = (grp * PT + p) * 16 + j;
                    valid[p] = idx < npix;
                    const int ii = valid[p] ? idx : 0;
                    const int gi = ii / img_pix;
                    const int rem = ii - gi * img_pix;
                    const int r = rem / Wo;
                    const int ox = rem - r * Wo;
                    lbase[p] = ((gi * bd.RI + r * S) * W2 + ox * S) * 64 + 16 * g;  // tap (0, 0) of the pixel
                    yo[p] = (((q.img0 + gi) * a.Ho + q.ro0 + r) * Wo + ox) * C + cl;
                }
                v4i acc[PT][4];
#pragma unroll
                for (int p = 0; p < PT; ++p)
#pragma unroll
                    for (int t = 0; t < 4; ++t) acc[p][t] = v4i{0, 0, 0, 0};
                // opaque offset: the fragment reads stay inside the loop (4 registers in flight
                // each) instead of being hoisted out of it into 144 registers
                int fo = lane;
                asm volatile("" : "+v"(fo));
                const v4i *fl = frag + fo;
#pragma unroll
                for (int s = 0; s < 9; ++s) {
                    v4i b[PT];
#pragma unroll
                    for (int p = 0; p < PT; ++p)
                        b[p] = *reinterpret_cast<const v4i *>(xt + lbase[p] + ((s / 3) * W2 + s % 3) * 64);
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const v4i wf = fl[(t * 9 + s) * 64];
#pragma unroll
                        for (int p = 0; p < PT; ++p)
                            acc[p][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf, b[p], acc[p][t], 0, 0, 0);
                    }
                }
#pragma unroll
                for (int p = 0; p < PT; ++p) {
                    uint32_t out[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        int v[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            v[r] = PRELU ? requant_prelu_i64(acc[p][t][r], par[t][r], lo, hi)
                                         : requant_i64<true>(acc[p][t][r], par[t][r], lo, hi);
                        out[t] = pack4_low_bytes(v[0], v[1], v[2], v[3]);
                    }
                    // the lane's channels cl .. cl+15 of its pixel (C % 4 == 0: whole dwords are in or out)
                    if (valid[p] && cl + 16 <= C) {
                        store_b128_guarded(v4i{(int)out[0], (int)out[1], (int)out[2], (int)out[3]}, ry, yo[p]);
                    } else if (valid[p]) {
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            if (cl + 4 * t < C)
                                __builtin_amdgcn_raw_buffer_store_b32((int)out[t], ry, yo[p] + 4 * t, 0, 0);
                    }
                }
            }
        }
    };
    if (prelu)
        run(std::true_type{});
    else
        run(std::false_type{});
}

__global__ __launch_bounds__(256, 2) void gconv_mfma_kernel(const GconvArgs a, const GconvBand bd)
{
    gconv_mfma_body(a, bd, (int)blockIdx.x);
}

// ---- gconv_tapk_kernel: group sizes 4, 8, 16 with the kernel taps in the k dimension -------------
// A tile of 16 output channels of such a layer sees only the 16 input channels at the same
// positions (its groups lie inside them), so its contraction is 9 taps x 16 channels = 144 long:
// three k steps of v_mfma_i32_16x16x64_i8 in which k group kg of step s is tap 4s + kg (taps 9..11
// have zero weights), instead of the nine of the kernel above, and 12 KB of fragments per block of
// 64 channels instead of 36.  The B operand of a lane is then the 16-byte piece `t` of the pixel
// under its tap, so the band is staged as four planes of 16-byte pieces ([piece][pixel]): lanes of
// consecutive pixels read consecutive pieces.  Tile t holds channels 16t .. 16t+15 in their own
// order; a lane's four dwords (one per tile) are exchanged between the four lanes of a pixel with
// two pairs of lane-row swaps, after which lane (j, g) holds channels 16g .. 16g+15 of its pixel
// and stores them as one 16-byte piece, as above.  Band geometry, staging through registers and
// units of work are those of gconv_mfma_kernel.
#ifdef PROM_TIMELINE
// Developer build: workgroups 0 .. 255 record the 100 MHz clock at entry, after the prologue and
// per band (pieces in LDS, barrier passed, band computed), then after the last store is acknowledged.
__device__ unsigned long long g_gc_stamps[256 * 16];
#define GC_STAMP(i) do { if (threadIdx.x == 0 && blockIdx.x < 256 && (i) < 16) g_gc_stamps[blockIdx.x * 16 + (i)] = wall_clock64(); } while (0)
#else
#define GC_STAMP(i) do { } while (0)
#endif

constexpr int kTapkFragBytes = 4 * 3 * 64 * 16;
constexpr int kTapkParBytes = kGconvParBytes + 16;  // the parameters and the flag of the epilogue form
constexpr int kTapkPT = 2;          // pixel tiles per wavefront iteration
constexpr int kTapkThreads = 256;   // 4 wavefronts, two workgroups per compute unit
constexpr int kTapkPieces = 9;      // 16-byte pieces of a staged band per thread

// Rows of 16 lanes, registers o[0..3]: o[t] of row g  <->  o[g] of row t.
__device__ __forceinline__ void transpose_rows4(uint32_t (&o)[4])
{
    // rows 2, 3 of o[t] <-> rows 0, 1 of o[t + 2]: the off-diagonal 2x2 blocks change places
    auto a02 = __builtin_amdgcn_permlane32_swap(o[0], o[2], false, false);
    auto a13 = __builtin_amdgcn_permlane32_swap(o[1], o[3], false, false);
    // rows 1, 3 of the first <-> rows 0, 2 of the second: each 2x2 block is transposed
    auto b01 = __builtin_amdgcn_permlane16_swap(a02[0], a13[0], false, false);
    auto b23 = __builtin_amdgcn_permlane16_swap(a02[1], a13[1], false, false);
    o[0] = b01[0];
    o[1] = b01[1];
    o[2] = b23[0];
    o[3] = b23[1];
}

template <int PT>
__device__ __forceinline__ void gconv_tapk_body(const GconvArgs &a, const GconvBand &bd, const int block)
{
    constexpr int kFlags = 0x00020000;
    constexpr int kOob = 0x7ffff000;
    constexpr int NK = kTapkPieces;
    constexpr int NT = kTapkThreads;
    extern __shared__ __align__(16) unsigned char lds[];
    v4i *frag = reinterpret_cast<v4i *>(lds);                                  // [tile t][step s][lane]
    v4i *lpar = reinterpret_cast<v4i *>(lds + kTapkFragBytes);                 // [64] parameters, then a flag
    unsigned char *xt = lds + kTapkFragBytes + kTapkParBytes;                  // [piece 4][G][RI][W+2][16]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, g = lane >> 4;
    // Workgroups go round-robin over the 8 XCDs, each with an L2 of its own.  A pixel's channel
    // blocks are neighbours in memory (two of them share a 128-byte line), so the workgroups of all
    // channel blocks with the same units sit on one XCD (grids that are a multiple of 8 per channel
    // block); otherwise every line comes from HBM once per channel block.
    int cb, wg;
    if (bd.swizzle) {
        const int k = block >> 3;
        cb = k % bd.ncb;
        wg = (k / bd.ncb) * 8 + (block & 7);
    } else {
        cb = block % bd.ncb;
        wg = block / bd.ncb;
    }
    if (wg >= bd.wgs_per_cb) return;  // padding of a shared launch
    const int C = a.C, GS = a.gs, S = a.stride, W = a.W, Wo = a.Wo;
    const int W2 = W + 2;
    const int cbase = cb * 64;
    const bool prelu = a.mult_neg != nullptr;
    const int row_items = W2 * 4;
    const int img_items = bd.RI * row_items;
    const int PS = bd.G * bd.RI * W2 * 16;  // bytes of a plane of pieces
    GC_STAMP(0);
    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a.x), 0, a.N * a.H * W * C, kFlags);
    const __amdgpu_buffer_rsrc_t ry =
        __builtin_amdgcn_make_buffer_rsrc(a.y, 0, a.N * a.Ho * Wo * C, kFlags);

    struct Unit { int img0, count, ro0, rows_out; };
    auto unit_of = [&](int u) {
        Unit q;
        if (bd.G > 1) {
            q.img0 = u * bd.G;
            q.count = min(bd.G, a.N - q.img0);
            q.ro0 = 0;
        } else {
            q.img0 = u / bd.bands;
            q.count = 1;
            q.ro0 = (u - q.img0 * bd.bands) * bd.R;
        }
        q.rows_out = min(bd.R, a.Ho - q.ro0);
        return q;
    };
    // piece pc of a unit = piece (pc & 3) of staged pixel pc >> 2 (images, rows, columns in order)
    v4i piece[NK];
    auto fetch_band = [&](int u) {
        const Unit q = unit_of(u);
        const int ri0 = q.ro0 * S - 1;
        const int npiece = q.count * img_items;
#pragma unroll
        for (int k = 0; k < NK; ++k) {
            const int pc = k * NT + tid;
            const int gi = pc / img_items;
            const int rem = pc - gi * img_items;
            const int row = rem / row_items;
            const int it = rem - row * row_items;
            const int col = it >> 2, qd = it & 3;
            const int iy = ri0 + row;
            const bool ok = pc < npiece && iy >= 0 && iy < a.H && col >= 1 && col <= W && cbase + 16 * qd < C;
            const int off = (((q.img0 + gi) * a.H + iy) * W + col - 1) * C + cbase + 16 * qd;
            piece[k] = __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? off : kOob, 0, 0);
        }
    };
    // the first band is requested before anything else: one memory latency for it, the weights and
    // the parameters together
    if (wg < bd.units) fetch_band(wg);
    // ---- fragments: lane (i, kg) of tile t, step s holds, for output channel 16t + i of the block and
    // tap 4s + kg, the weights on input channels 16t .. 16t+15 (zero outside the channel's group)
    if (a.wfrag) {
        const v4i *src = a.wfrag + (long long)cb * (4 * 3 * 64);
        for (int idx = tid; idx < 4 * 3 * 64; idx += NT) frag[idx] = src[idx];
    } else
    for (int idx = tid; idx < 4 * 3 * 64; idx += NT) {
        const int l = idx & 63, ts = idx >> 6, s = ts % 3, t = ts / 3;
        const int i = l & 15, kg = l >> 4;
        const int tap = 4 * s + kg;
        const int oc = cbase + 16 * t + i;
        v4i e = {0, 0, 0, 0};
        if (oc < C && tap < 9) {
            const int gfirst = (oc / GS) * GS;
            const int8_t *wrow = a.w + ((long long)tap * C + oc) * GS;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int ic = cbase + 16 * t + 4 * d;
                if (ic >= gfirst && ic < gfirst + GS) e[d] = *reinterpret_cast<const int *>(wrow + (ic - gfirst));
            }
        }
        frag[idx] = e;
    }
    if (tid < 64) {
        const int c = cbase + tid;
        int shift = 1;
        v4i p = {0, 0, 0, 1};
        if (c < C) {
            shift = a.shift[c];
            p = requant_params(a.bias[c], a.mult[c], prelu ? a.mult_neg[c] : 0, shift, prelu);
        }
        lpar[tid] = p;
        // every shift of the block >= 1 (the usual case): the quotient comes from the high half of the
        // 64-bit sum and one 32-bit shift by shift - 1
        const bool all_ge1 = __builtin_amdgcn_ballot_w64(shift >= 1) == ~0ull;
        if (tid == 0) *reinterpret_cast<int *>(lpar + 64) = all_ge1 ? 1 : 0;
    }
    __syncthreads();

    const bool general = prelu || __builtin_amdgcn_readfirstlane(*reinterpret_cast<const int *>(lpar + 64)) == 0;
    v4i par[4][4];  // [tile t][r]: channel 16t + 4g + r; the fast form shifts by shift - 1
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            par[t][r] = lpar[16 * t + 4 * g + r];
            if (!general) par[t][r][3] -= 1;
        }
    GC_STAMP(1);
    [[maybe_unused]] int band_no = 0;
    const bool full_block = cbase + 64 <= C;
    // n / d by the band's magic numbers
    auto div_wo = [&](int n) { return (int)(((unsigned long long)(unsigned)n * bd.magic_wo) >> 31); };
    auto div_img = [&](int n) { return (int)(((unsigned long long)(unsigned)n * bd.magic_img) >> 31); };
    const int lo = in_vgpr(a.lo), hi = in_vgpr(a.hi);
    const int cl = cbase + 16 * g;  // the lane's first output channel after the exchange
    int toff[3];                    // the lane's tap of each k step, as a byte offset in a plane
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        const int tap = min(4 * s + g, 8);
        toff[s] = ((tap / 3) * W2 + tap % 3) * 16;
    }

    auto run = [&](auto mode_tag) {
        constexpr int MODE = decltype(mode_tag)::value;
        for (int u = wg; u < bd.units; u += bd.wgs_per_cb) {
            const Unit q = unit_of(u);
            const int npiece = q.count * img_items;
            __syncthreads();  // the readers of the previous band are done
#pragma unroll
            for (int k = 0; k < NK; ++k) {
                const int pc = k * NT + tid;
                if (pc < npiece) *reinterpret_cast<v4i *>(xt + (pc & 3) * PS + (pc >> 2) * 16) = piece[k];
            }
            GC_STAMP(2 + 3 * band_no);
            __syncthreads();
            GC_STAMP(3 + 3 * band_no);
            if (u + bd.wgs_per_cb < bd.units) fetch_band(u + bd.wgs_per_cb);
            const int img_pix = q.rows_out * Wo;
            const int npix = q.count * img_pix;
            const int ngrp = (npix + 16 * PT - 1) / (16 * PT);
            for (int grp = wave; grp < ngrp; grp += NT / 64) {
                int pix[PT], yo[PT];
                bool valid[PT];
#pragma unroll
                for (int p = 0; p < PT; ++p) {
                    const int idx = (grp * PT + p) * 16 + j;
                    valid[p] = idx < npix;
                    const int ii = valid[p] ? idx : 0;
                    // img_pix = R * Wo except in an image's last band, where a unit is one image and idx < img_pix
                    const int gi = div_img(ii);
                    const int rem = ii - gi * img_pix;
                    const int r = div_wo(rem);
                    const int ox = rem - r * Wo;
                    pix[p] = ((gi * bd.RI + r * S) * W2 + ox * S) * 16;  // tap (0, 0) of the pixel
                    yo[p] = (((q.img0 + gi) * a.Ho + q.ro0 + r) * Wo + ox) * C + cl;
                }
                v4i acc[PT][4];
#pragma unroll
                for (int p = 0; p < PT; ++p)
#pragma unroll
                    for (int t = 0; t < 4; ++t) acc[p][t] = v4i{0, 0, 0, 0};
                int fo = lane;
                asm volatile("" : "+v"(fo));  // keeps the fragment reads inside the loop
                const v4i *fl = frag + fo;
#pragma unroll
                for (int s = 0; s < 3; ++s) {
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const v4i wf = fl[(t * 3 + s) * 64];
#pragma unroll
                        for (int p = 0; p < PT; ++p) {
                            const v4i b = *reinterpret_cast<const v4i *>(xt + t * PS + pix[p] + toff[s]);
                            acc[p][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf, b, acc[p][t], 0, 0, 0);
                        }
                    }
                }
#pragma unroll
                for (int p = 0; p < PT; ++p) {
                    uint32_t out[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        int v[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) v[r] = requant_mode<MODE>(acc[p][t][r], par[t][r], lo, hi);
                        out[t] = pack4_low_bytes(v[0], v[1], v[2], v[3]);
                    }
                    transpose_rows4(out);  // now channels cl .. cl+15 of the lane's pixel
                    if (full_block) {
                        store_b128_guarded(v4i{(int)out[0], (int)out[1], (int)out[2], (int)out[3]}, ry,
                                           valid[p] ? yo[p] : kOob);
                    } else if (valid[p]) {
#pragma unroll
                        for (int t = 0; t < 4; ++t)
                            if (cl + 4 * t < C)
                                __builtin_amdgcn_raw_buffer_store_b32((int)out[t], ry, yo[p] + 4 * t, 0, 0);
                    }
                }
            }
            GC_STAMP(4 + 3 * band_no);
            ++band_no;

        }
    };
    if (prelu)
        run(std::integral_constant<int, 2>{});
    else if (general)
        run(std::integral_constant<int, 1>{});
    else
        run(std::integral_constant<int, 0>{});
#ifdef PROM_TIMELINE
    __builtin_amdgcn_s_waitcnt(0);
    GC_STAMP(15);
#endif
}

template <int PT>
__global__ __launch_bounds__(kTapkThreads, 2) void gconv_tapk_kernel(const GconvArgs a, const GconvBand bd)
{
    gconv_tapk_body<PT>(a, bd, (int)blockIdx.x);
}

// ---- several layers in one launch (prom_gconv3x3_sequence) ----------------------------------------
// The kernel argument is a table of layers and of the first workgroup of each; a workgroup finds
// its layer and runs that layer's body with its index inside the layer.
constexpr int kGconvMaxBatch = 24;
constexpr int kGconvBatchSlots = 512;  // workgroups of a shared launch: two per compute unit
struct GconvBatchArgs {
    GconvArgs a[kGconvMaxBatch];
    GconvBand bd[kGconvMaxBatch];
    int start[kGconvMaxBatch + 1];
    int count;
};
static_assert(sizeof(GconvBatchArgs) <= 4096, "kernel arguments are limited to 4 KB");

__device__ __forceinline__ int gconv_batch_member(const GconvBatchArgs &b)
{
    int m = 0;
    for (int k = 1; k < b.count; ++k)
        if ((int)blockIdx.x >= b.start[k]) m = k;
    return m;
}

#ifdef PROM_TIMELINE
// Developer build: member, entry and exit clock of the first 2048 workgroups of a shared launch.
__device__ unsigned long long g_gcb_stamps[2048 * 3];
#endif

template <int PT>
__global__ __launch_bounds__(kTapkThreads, 2) void gconv_tapk_batch_kernel(const GconvBatchArgs b)
{
    const int m = gconv_batch_member(b);
#ifdef PROM_TIMELINE
    if (threadIdx.x == 0 && blockIdx.x < 2048) {
        g_gcb_stamps[blockIdx.x * 3] = (unsigned long long)m;
        g_gcb_stamps[blockIdx.x * 3 + 1] = wall_clock64();
    }
#endif
    gconv_tapk_body<PT>(b.a[m], b.bd[m], (int)blockIdx.x - b.start[m]);
#ifdef PROM_TIMELINE
    __builtin_amdgcn_s_waitcnt(0);
    if (threadIdx.x == 0 && blockIdx.x < 2048) g_gcb_stamps[blockIdx.x * 3 + 2] = wall_clock64();
#endif
}

__global__ __launch_bounds__(256, 2) void gconv_mfma_batch_kernel(const GconvBatchArgs b)
{
    const int m = gconv_batch_member(b);
    gconv_mfma_body(b.a[m], b.bd[m], (int)blockIdx.x - b.start[m]);
}

// Any C, group size and alignment: one thread per output element.
__global__ __launch_bounds__(256) void gconv_kernel_generic(const GconvArgs a)
{
    const long long tid = (long long)blockIdx.x * 256 + threadIdx.x;
    if (tid >= a.total) return;
    const int c = (int)(tid % a.C);
    long long r = tid / a.C;
    const int ox = (int)(r % a.Wo);
    r /= a.Wo;
    const int oy = (int)(r % a.Ho);
    const int n = (int)(r / a.Ho);
    const int first = (c / a.gs) * a.gs;
    int acc = a.bias[c];
    for (int i = 0; i < 3; ++i) {
        const int iy = oy * a.stride + i - 1;
        if (iy < 0 || iy >= a.H) continue;
        for (int jx = 0; jx < 3; ++jx) {
            const int ix = ox * a.stride + jx - 1;
            if (ix < 0 || ix >= a.W) continue;
            const int8_t *xp = a.x + (((long long)n * a.H + iy) * a.W + ix) * a.C + first;
            const int8_t *wp = a.w + ((long long)(i * 3 + jx) * a.C + c) * a.gs;
            for (int k = 0; k < a.gs; ++k) acc += (int)xp[k] * (int)wp[k];
        }
    }
    const int m = (a.mult_neg && acc < 0) ? a.mult_neg[c] : a.mult[c];
    a.y[tid] = (int8_t)requant_s_i64(acc, m, a.shift[c], a.lo, a.hi);
}

using GconvFn = void (*)(const GconvArgs);

// gs % 4 == 0: the widest chunk that divides the group.
template <int S> static GconvFn pick_gconv(int gs)
{
    if (gs == 4) return &gconv_kernel_v4<S, 1, true>;
    if (gs == 8) return &gconv_kernel_v4<S, 2, true>;
    if (gs == 16) return &gconv_kernel_v4<S, 4, true>;
    if (gs % 16 == 0) return &gconv_kernel_v4<S, 4, false>;
    if (gs % 8 == 0) return &gconv_kernel_v4<S, 2, false>;
    return &gconv_kernel_v4<S, 1, false>;
}

static bool ranges_overlap(const void *p, size_t pn, const void *q, size_t qn)
{
    const uintptr_t a = (uintptr_t)p, b = (uintptr_t)q;
    return a < b + qn && b < a + pn;
}

}  // namespace prom

namespace prom {

// A validated, planned layer.
struct GconvLaunch {
    enum Kind { DEPTHWISE, TAPK, MFMA, V4, GENERIC } kind;
    GconvArgs a;
    GconvBand bd;       // TAPK, MFMA
    size_t lds;         // TAPK, MFMA
    unsigned grid;      // TAPK, MFMA: workgroups
    const prom_requant_t *rq;  // DEPTHWISE: the caller's struct, valid during the call
    size_t xbytes, ybytes, wbytes, fbytes;
    const void *w_frag;
};

static int gconv_prepare(const int8_t *x, int n, int h, int w, int c, const int8_t *w_g, const void *w_frag,
                         int group_size, int stride, const prom_requant_t *rq, int8_t *y, GconvLaunch &L)
{
    if (!x || !w_g || !rq || !rq->bias || !rq->mult || !rq->shift || !y) return PROM_EINVAL;
    if (n <= 0 || h <= 0 || w <= 0 || c <= 0 || (stride != 1 && stride != 2)) return PROM_EINVAL;
    if (group_size <= 0 || c % group_size != 0) return PROM_EINVAL;
    if (rq->act_min < -128 || rq->act_max > 127 || rq->act_min > rq->act_max) return PROM_EINVAL;
    // |acc| <= 9 * gs * 128 * 128 must stay well inside the int32 accumulator and the
    // precondition |acc + bias| < 2^30 of the requantisation
    if (group_size > 4096) return PROM_EUNSUPPORTED;
    GconvArgs &a = L.a;
    a.x = x; a.w = w_g; a.wfrag = nullptr; a.bias = rq->bias; a.mult = rq->mult; a.mult_neg = rq->mult_neg; a.shift = rq->shift;
    a.y = y;
    a.N = n; a.H = h; a.W = w; a.C = c; a.stride = stride; a.gs = group_size;
    a.Ho = (h - 1) / stride + 1;
    a.Wo = (w - 1) / stride + 1;
    a.lo = rq->act_min;
    a.hi = rq->act_max;
    L.rq = rq;
    L.w_frag = w_frag;
    const size_t xbytes = (size_t)n * h * w * c, ybytes = (size_t)n * a.Ho * a.Wo * c;
    const size_t wbytes = (size_t)9 * c * group_size;
    L.xbytes = xbytes; L.ybytes = ybytes; L.wbytes = wbytes; L.fbytes = 0;
    if (group_size == 1) {  // same weight layout: prom_dw_conv validates the rest
        L.kind = GconvLaunch::DEPTHWISE;
        return PROM_OK;
    }
    if (xbytes >= ((size_t)1 << 40)) return PROM_EUNSUPPORTED;
    if (ranges_overlap(y, ybytes, x, xbytes) || ranges_overlap(y, ybytes, w_g, wbytes)) return PROM_EALIAS;
    a.total = (long long)ybytes;
    const bool fast = (group_size % 4 == 0) && (c % 4 == 0) && ((((uintptr_t)x | (uintptr_t)y | (uintptr_t)w_g) & 3) == 0) &&
                      ((((uintptr_t)rq->bias | (uintptr_t)rq->mult | (uintptr_t)rq->mult_neg |
                         (uintptr_t)rq->shift) & 15) == 0) &&
                      (long long)h * w * c < (1LL << 31) - (1LL << 24) && wbytes < ((size_t)1 << 30) && n <= 65535;
    const bool mfma = fast && (group_size == 4 || group_size == 8 || group_size == 16 || group_size == 32 ||
                               group_size == 64) &&
                      xbytes < ((size_t)1 << 31) - ((size_t)1 << 24) && ybytes < ((size_t)1 << 31) - ((size_t)1 << 24);
    if (w_frag) {
        L.fbytes = prom_gconv_frag_size(c, group_size);
        if (((uintptr_t)w_frag & 15) != 0 || L.fbytes == 0) return PROM_EINVAL;
        if (ranges_overlap(y, ybytes, w_frag, L.fbytes)) return PROM_EALIAS;
    }
    if (mfma) {
        // band height: as many output rows as keep the staged input rows within the band's bytes
        const bool tapk = group_size <= 16;
        const int kBandBytes = tapk ? kTapkPieces * kTapkThreads * 16 : kGconvPieces * 256 * 16;
        const int row_bytes = (w + 2) * 64;
        const int ri = kBandBytes / row_bytes;
        if (ri >= 3) {  // else an image row is too wide for the staged band: the dot4 kernel takes it
            a.wfrag = static_cast<const v4i *>(w_frag);
            GconvBand &bd = L.bd;
            bd.ncb = (c + 63) / 64;
            bd.R = (ri - 3) / stride + 1;
            if (bd.R > a.Ho) bd.R = a.Ho;
            if (bd.R < a.Ho) {
                // bands of equal height rather than a short last one
                const int nb = (a.Ho + bd.R - 1) / bd.R;
                bd.R = (a.Ho + nb - 1) / nb;
            }
            bd.RI = (bd.R - 1) * stride + 3;
            bd.bands = (a.Ho + bd.R - 1) / bd.R;
            bd.G = 1;
            if (bd.bands == 1) {
                // small images: several per unit (a workgroup copies its block's weights whatever it
                // computes), as far as they fit, but no more than leaves a workgroup for every
                // compute unit
                bd.G = kBandBytes / (bd.RI * row_bytes);
                const long long spare = (long long)n * bd.ncb / 256;
                if (bd.G > spare) bd.G = (int)spare;
                if (bd.G > 16) bd.G = 16;
                if (bd.G < 1) bd.G = 1;
            }
            const long long units = bd.G > 1 ? ((long long)n + bd.G - 1) / bd.G : (long long)n * bd.bands;
            bd.units = (int)units;
            const unsigned d_img = (unsigned)bd.R * (unsigned)a.Wo;
            bd.magic_wo = (unsigned)((1ull << 31) / (unsigned)a.Wo) + 1u;
            bd.magic_img = (unsigned)((1ull << 31) / d_img) + 1u;
            // two workgroups per compute unit, and not one more: a workgroup that does not fit in the
            // first round starts when another has finished all its units and doubles the run time
            long long per_cb = (2 * 256) / bd.ncb;
            if (per_cb > units) per_cb = units;
            if (per_cb < 1) per_cb = 1;
            if (per_cb >= 64) per_cb -= per_cb % 8;  // for the XCD-aware order; small grids keep every workgroup
            bd.wgs_per_cb = (int)per_cb;
            bd.swizzle = per_cb % 8 == 0;
            L.lds = (size_t)(tapk ? kTapkFragBytes + kTapkParBytes : kGconvFragBytes + kGconvParBytes) +
                    (size_t)bd.G * bd.RI * row_bytes;
            L.grid = (unsigned)(per_cb * bd.ncb);
            L.kind = tapk ? GconvLaunch::TAPK : GconvLaunch::MFMA;
            return PROM_OK;
        }
    }
    if (fast) {
        const long long xblocks = ((long long)a.Wo * (c / 4) + 255) / 256;
        const int strips = (a.Ho + 3) / 4;
        if (xblocks > (1LL << 31) - 1 || strips > 65535) return PROM_EUNSUPPORTED;
        L.kind = GconvLaunch::V4;
    } else {
        if ((a.total + 255) / 256 > (1LL << 31) - 1) return PROM_EUNSUPPORTED;
        L.kind = GconvLaunch::GENERIC;
    }
    return PROM_OK;
}

// The matrix-core kernels stage up to 96 KB in LDS.
static int gconv_set_attributes()
{
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {
        const void *fns[4] = {reinterpret_cast<const void *>(&gconv_mfma_kernel),
                              reinterpret_cast<const void *>(&gconv_tapk_kernel<kTapkPT>),
                              reinterpret_cast<const void *>(&gconv_mfma_batch_kernel),
                              reinterpret_cast<const void *>(&gconv_tapk_batch_kernel<kTapkPT>)};
        for (const void *fn : fns)
            if (attr_err == hipSuccess)
                attr_err = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
    });
    if (attr_err != hipSuccess) {
        last_hip_error() = attr_err;
        (void)hipGetLastError();
        return PROM_EHIP;
    }
    return PROM_OK;
}

static int gconv_launch(const GconvLaunch &L, hipStream_t st)
{
    const GconvArgs &a = L.a;
    if (L.kind == GconvLaunch::DEPTHWISE)
        return prom_dw_conv(a.x, a.N, a.H, a.W, a.C, a.w, a.stride, L.rq, a.y, st);
    if (L.kind == GconvLaunch::TAPK || L.kind == GconvLaunch::MFMA) {
        const int rc = gconv_set_attributes();
        if (rc != PROM_OK) return rc;
    }
    clear_hip_error();
    switch (L.kind) {
    case GconvLaunch::TAPK:
        hipLaunchKernelGGL((gconv_tapk_kernel<kTapkPT>), dim3(L.grid), dim3(kTapkThreads), L.lds, st, a, L.bd);
        break;
    case GconvLaunch::MFMA:
        hipLaunchKernelGGL(gconv_mfma_kernel, dim3(L.grid), dim3(256), L.lds, st, a, L.bd);
        break;
    case GconvLaunch::V4: {
        const GconvFn fn = a.stride == 1 ? pick_gconv<1>(a.gs) : pick_gconv<2>(a.gs);
        const long long xblocks = ((long long)a.Wo * (a.C / 4) + 255) / 256;
        const int strips = (a.Ho + 3) / 4;
        hipLaunchKernelGGL(fn, dim3((unsigned)xblocks, (unsigned)strips, (unsigned)a.N), dim3(256), 0, st, a);
        break;
    }
    default:
        hipLaunchKernelGGL(gconv_kernel_generic, dim3((unsigned)((a.total + 255) / 256)), dim3(256), 0, st, a);
        break;
    }
    return check_launch();
}

// True if one of the two layers writes what the other reads or writes.
static bool gconv_conflicts(const GconvLaunch &p, const GconvLaunch &q)
{
    auto reads_or_writes = [](const GconvLaunch &l, const void *y, size_t yn) {
        const size_t pn = (size_t)l.a.C * sizeof(int32_t);
        return ranges_overlap(y, yn, l.a.x, l.xbytes) || ranges_overlap(y, yn, l.a.y, l.ybytes) ||
               ranges_overlap(y, yn, l.a.w, l.wbytes) || (l.w_frag && ranges_overlap(y, yn, l.w_frag, l.fbytes)) ||
               ranges_overlap(y, yn, l.a.bias, pn) || ranges_overlap(y, yn, l.a.mult, pn) ||
               ranges_overlap(y, yn, l.a.shift, pn) || (l.a.mult_neg && ranges_overlap(y, yn, l.a.mult_neg, pn));
    };
    return reads_or_writes(q, p.a.y, p.ybytes) || reads_or_writes(p, q.a.y, q.ybytes);
}

}  // namespace prom

extern "C" int prom_gconv3x3(const int8_t *x, int n, int h, int w, int c, const int8_t *w_g, const void *w_frag,
                             int group_size, int stride, const prom_requant_t *rq, int8_t *y, void *stream)
{
    prom::GconvLaunch L;
    const int rc = prom::gconv_prepare(x, n, h, w, c, w_g, w_frag, group_size, stride, rq, y, L);
    if (rc != PROM_OK) return rc;
    return prom::gconv_launch(L, static_cast<hipStream_t>(stream));
}

extern "C" int prom_gconv3x3_sequence(const prom_gconv_layer_t *layers, int count, int *bad_layer, void *stream)
{
    using namespace prom;
    if (bad_layer) *bad_layer = -1;
    if (count < 0 || (count > 0 && !layers)) return PROM_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    static thread_local std::vector<GconvLaunch> prepared;
    prepared.resize((size_t)count);
    for (int i = 0; i < count; ++i) {
        const prom_gconv_layer_t &l = layers[i];
        const int rc = gconv_prepare(l.x, l.n, l.h, l.w, l.c, l.w_g, l.w_frag, l.group_size, l.stride, &l.rq, l.y,
                                     prepared[(size_t)i]);
        if (rc != PROM_OK) {
            if (bad_layer) *bad_layer = i;
            return rc;
        }
    }
    // Consecutive layers of one matrix-core kernel that do not touch each other's data share a launch
    // (at most kGconvMaxBatch of them), the members with the least work first: a small layer is one
    // latency chain per workgroup and would otherwise end the launch alone.
    static thread_local GconvBatchArgs b;
    int i = 0;
    while (i < count) {
        const GconvLaunch::Kind kind = prepared[(size_t)i].kind;
        int j = i;
        if (kind == GconvLaunch::TAPK || kind == GconvLaunch::MFMA) {
            long long blocks = 0;
            while (j < count && j - i < kGconvMaxBatch && prepared[(size_t)j].kind == kind) {
                const GconvLaunch &L = prepared[(size_t)j];
                bool clash = false;
                for (int k = i; k < j && !clash; ++k) clash = gconv_conflicts(prepared[(size_t)k], L);
                if (clash || blocks + L.grid > (1LL << 30)) break;
                blocks += L.grid;
                ++j;
            }
        }
        int rc;
        if (j - i >= 2) {
            rc = gconv_set_attributes();
            if (rc == PROM_OK) {
                // The launch has as many workgroups as are resident at once (two per compute unit):
                // alone, a small layer spreads over the chip for the sake of latency; here that would
                // queue thousands of workgroups that each live one latency chain long.  They are shared
                // out so that every layer's workgroups live about equally long, by an estimate of a
                // workgroup's time per unit of work (a fixed part for staging, barriers and the fetch
                // latency, plus the rounds in which its four wavefronts take the unit's groups of 32
                // pixels; fitted to the per-workgroup lifetimes of such a launch): the layer whose
                // workgroups would live longest gets the next ones.  Shares by the bytes alone leave the
                // layers with small images far behind (a unit of three 7x7 images takes as long as a
                // band of 112 pixels), shares by the rounds alone the large ones.
                const int n = j - i;
                double cost[kGconvMaxBatch];
                int per_cb[kGconvMaxBatch], step[kGconvMaxBatch];
                double cost_sum = 0;
                // Small images: a layer alone takes no more images per unit of work than leaves a
                // workgroup for every compute unit; here a layer has a dozen workgroups whatever it
                // does, and takes as many images per unit as cost least per image by the same
                // estimate (7x7: seven instead of three, 14x14: two instead of one).
                for (int k = 0; k < n; ++k) {
                    GconvLaunch &L = prepared[(size_t)(i + k)];
                    GconvBand &bd = L.bd;
                    if (bd.bands != 1) continue;
                    const int band_bytes = kind == GconvLaunch::TAPK ? kTapkPieces * kTapkThreads * 16 : kGconvPieces * 256 * 16;
                    const int image_bytes = bd.RI * (L.a.W + 2) * 64;
                    int gmax = band_bytes / image_bytes;
                    if (gmax > 16) gmax = 16;
                    if (gmax > L.a.N) gmax = L.a.N;
                    auto per_image = [&](int g) {
                        const int rounds = ((g * bd.R * L.a.Wo + 31) / 32 + 3) / 4;
                        return (2.0 + 1.3 * rounds) / g;
                    };
                    int best = bd.G;
                    for (int g = 1; g <= gmax; ++g)
                        if (per_image(g) < 0.98 * per_image(best)) best = g;
                    if (best != bd.G) {
                        L.lds = L.lds - (size_t)bd.G * image_bytes + (size_t)best * image_bytes;
                        bd.G = best;
                        bd.units = (L.a.N + best - 1) / best;
                    }
                }
                for (int k = 0; k < n; ++k) {
                    const GconvLaunch &L = prepared[(size_t)(i + k)];
                    const int npix = (L.bd.G > 1 ? L.bd.G : 1) * L.bd.R * L.a.Wo;
                    const int rounds = ((npix + 31) / 32 + 3) / 4;
                    cost[k] = (double)L.bd.ncb * L.bd.units * (2.0 + 1.3 * rounds);
                    cost_sum += cost[k];
                }
                // (three per compute unit would fit LDS and registers of the tap-in-k kernel: 108-114
                // against 91 us for RegNetX-400MF's 22 layers, 301-313 against 264 for ResNeXt-50's)
                constexpr int slots = kGconvBatchSlots;
                int used = 0;
                for (int k = 0; k < n; ++k) {
                    const GconvBand &bd = prepared[(size_t)(i + k)].bd;
                    const double ideal = slots * cost[k] / cost_sum / bd.ncb;
                    // several channel blocks and enough workgroups: multiples of 8, for the XCD-aware order
                    step[k] = (bd.ncb > 1 && ideal >= 8 && bd.units >= 8) ? 8 : 1;
                    int w = (int)(ideal / step[k]) * step[k];
                    if (w < step[k]) w = step[k];
                    if (w > bd.units) w = bd.units / step[k] * step[k];
                    per_cb[k] = w;
                    used += w * bd.ncb;
                }
                for (;;) {  // the remaining workgroups, one step at a time, to the layer that would end last
                    int best = -1;
                    double best_life = 0;
                    for (int k = 0; k < n; ++k) {
                        const GconvBand &bd = prepared[(size_t)(i + k)].bd;
                        if (per_cb[k] + step[k] > bd.units || used + step[k] * bd.ncb > slots) continue;
                        const double life = cost[k] / ((double)per_cb[k] * bd.ncb);
                        if (best < 0 || life > best_life) {
                            best = k;
                            best_life = life;
                        }
                    }
                    if (best < 0) break;
                    per_cb[best] += step[best];
                    used += step[best] * prepared[(size_t)(i + best)].bd.ncb;
                }
                // A layer that takes its workgroups 8 per channel block at a time can be left with
                // half of what it needs when the others' minimum shares have used up the launch: while
                // the layer that would end last can still grow, it takes workgroups from layers
                // that would end a quarter sooner even without them (RegNetX-400MF at batch 256: 174
                // against 223 us; with any gain taken, batch 32 and 128 lose 3-6 %: the estimate is
                // no finer than that).
                for (int pass = 0; pass < 4 * slots; ++pass) {
                    int last = -1;
                    double last_life = 0;
                    for (int k = 0; k < n; ++k) {
                        const double life = cost[k] / ((double)per_cb[k] * prepared[(size_t)(i + k)].bd.ncb);
                        if (life > last_life) {
                            last_life = life;
                            last = k;
                        }
                    }
                    const GconvBand &lb = prepared[(size_t)(i + last)].bd;
                    if (per_cb[last] + step[last] > lb.units) break;
                    int trial[kGconvMaxBatch];
                    for (int k = 0; k < n; ++k) trial[k] = per_cb[k];
                    int need = step[last] * lb.ncb - (slots - used);
                    while (need > 0) {
                        int donor = -1;
                        double donor_life = 0;
                        for (int k = 0; k < n; ++k) {
                            if (k == last || trial[k] < 2 * step[k]) continue;
                            const double life =
                                cost[k] / ((double)(trial[k] - step[k]) * prepared[(size_t)(i + k)].bd.ncb);
                            if (donor < 0 || life < donor_life) {
                                donor = k;
                                donor_life = life;
                            }
                        }
                        if (donor < 0 || donor_life * 1.25 >= last_life) break;
                        trial[donor] -= step[donor];
                        need -= step[donor] * prepared[(size_t)(i + donor)].bd.ncb;
                    }
                    if (need > 0) break;
                    trial[last] += step[last];
                    used = 0;
                    for (int k = 0; k < n; ++k) {
                        per_cb[k] = trial[k];
                        used += per_cb[k] * prepared[(size_t)(i + k)].bd.ncb;
                    }
                }
                // Order: the layers without the XCD-aware order first, packed without gaps (padding
                // blocks would leave some XCDs with more workgroups than they can hold at once), then,
                // from a multiple of 8 on, the others; within each kind the least bytes first (a small
                // layer is one latency chain per workgroup and would otherwise end the launch alone).
                int order[kGconvMaxBatch];
                for (int k = 0; k < n; ++k) order[k] = k;
                std::stable_sort(order, order + n, [&](int p, int q) {
                    const bool sp = step[p] == 8, sq = step[q] == 8;
                    if (sp != sq) return !sp;
                    return prepared[(size_t)(i + p)].xbytes + prepared[(size_t)(i + p)].ybytes <
                           prepared[(size_t)(i + q)].xbytes + prepared[(size_t)(i + q)].ybytes;
                });
                b.count = n;
                int start = 0;
                size_t lds = 0;
                for (int k = 0; k < n; ++k) {
                    const int m = order[k];
                    const GconvLaunch &L = prepared[(size_t)(i + m)];
                    b.a[k] = L.a;
                    b.bd[k] = L.bd;
                    b.bd[k].wgs_per_cb = per_cb[m];
                    b.bd[k].swizzle = step[m] == 8;
                    if (step[m] == 8) start = (start + 7) / 8 * 8;  // a member's workgroup index tells its XCD
                    b.start[k] = start;
                    start += per_cb[m] * L.bd.ncb;
                    if (L.lds > lds) lds = L.lds;
                }
                b.start[j - i] = start;
                clear_hip_error();
                if (kind == GconvLaunch::TAPK)
                    hipLaunchKernelGGL((gconv_tapk_batch_kernel<kTapkPT>), dim3((unsigned)start), dim3(kTapkThreads), lds, st, b);
                else
                    hipLaunchKernelGGL(gconv_mfma_batch_kernel, dim3((unsigned)start), dim3(256), lds, st, b);
                rc = check_launch();
            }
            i = j;
        } else {
            rc = gconv_launch(prepared[(size_t)i], st);
            ++i;
        }
        if (rc != PROM_OK) {
            if (bad_layer) *bad_layer = i - 1;
            return rc;
        }
    }
    return PROM_OK;
}

#ifdef PROM_TIMELINE
extern "C" int prom_debug_gcb_stamps(unsigned long long *host)
{
    if (hipDeviceSynchronize() != hipSuccess) return PROM_EHIP;
    return hipMemcpyFromSymbol(host, HIP_SYMBOL(prom::g_gcb_stamps), sizeof(unsigned long long) * 2048 * 3) == hipSuccess ? PROM_OK : PROM_EHIP;
}
extern "C" int prom_debug_gc_stamps(unsigned long long *host)
{
    if (hipDeviceSynchronize() != hipSuccess) return PROM_EHIP;
    return hipMemcpyFromSymbol(host, HIP_SYMBOL(prom::g_gc_stamps), sizeof(unsigned long long) * 256 * 16) == hipSuccess ? PROM_OK : PROM_EHIP;
}
#endif
