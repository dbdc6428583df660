// Depthwise 3x3 followed by the ternary pointwise projection in one kernel: the second half of the
// inverted-residual block (paper Section 2; Figure 4), for blocks whose hidden tensor is too deep
// for the fully fused kernel (384 to 960 hidden channels at 14x14 and 7x7).  The depthwise output
// never reaches HBM: one intermediate round trip and one launch less per block.
//
// A workgroup owns a band of R output rows of one image and walks over the hidden channels in
// chunks of 64:
//   - the chunk's slice of the band's input rows (with halo) comes from HBM as 16-byte pieces
//     (two chunks ahead, held in registers) into a double-buffered LDS tile of 4 planes of 16
//     channels with a zero border, which is the padding of the convolution;
//   - the depthwise 3x3 runs on the matrix cores: for 16 channels the 64-deep k dimension of
//     v_mfma_i32_16x16x64_i8 holds 4 taps x 16 channels (B operand of lane (pixel, g): the 16
//     channel bytes of the pixel under tap 4q + g; A operand: zero except the weight of the lane's
//     channel and tap), 3 MFMAs for the 9 taps of 16 pixels x 16 channels;
//   - the requantised depthwise outputs of a lane (its pixel, 16 of the chunk's 64 channels) are,
//     packed, a B operand of the projection MFMA, whose A operands are decoded per chunk and
//     wavefront from the 2-bit codes, which sit in LDS for the whole layer (cout x chid / 4 bytes);
//     the projection accumulators stay in registers across the chunks.
// Everything a chunk needs except its activation slice is staged once per workgroup, so a chunk
// costs no memory latency of its own.  One workgroup barrier per chunk.
#include "prom_pw_stream.h"
#include "prom_launch.h"

#include <mutex>
#include <vector>

namespace prom {

struct DwProjArgs {
    const int8_t *t;     // [N][H][W][C] input of the depthwise layer (the expanded tensor)
    const int8_t *wd;    // [3][3][C]
    const uint32_t *wp;  // packed [cout][C]
    const int32_t *bd, *md, *sd, *nd;  // depthwise bias / mult / shift / mult_neg (or nullptr) [C]
    const int32_t *bp, *mp, *sp, *np;  // projection [cout]
    const int8_t *res;   // [N][Ho][Wo][cout] or nullptr
    int8_t *y;           // [N][Ho][Wo][cout]
    int N, H, W, Ho, Wo, C, cout, stride;
    int R, bands, RI;    // output rows per band, bands per image, input rows per band
    int nch;             // chunks of 64 hidden channels
    int lo_d, hi_d, lo_p, hi_p;
    int rsw;             // bytes per row of the packed projection weights in LDS
    int wp_vec;          // the packed rows are whole 16-byte pieces and 16-byte aligned
    int off_wd, off_pd, off_pp, off_t1, plane;  // LDS byte offsets; bytes of one 16-channel plane
};

constexpr int kDpCH = 64;     // hidden channels per chunk
constexpr int kDpPieces = 4;  // 16-byte pieces of a slice per thread (a slice is at most 256 pixels)
constexpr int kDpAhead = 2;   // slices in flight (three were measured: no faster, the chunk loop is not waiting on memory)

#ifdef PROM_TIMELINE
// Developer build: workgroup 0 .. 63 record the 100 MHz clock at up to 32 points of their life.
__device__ unsigned long long g_dp_stamps[64 * 32];
#define DP_STAMP(i) do { if (threadIdx.x == 0 && blockIdx.x < 64 && (i) < 32) g_dp_stamps[blockIdx.x * 32 + (i)] = wall_clock64(); } while (0)
#else
#define DP_STAMP(i) do { } while (0)
#endif

template <int COT, int TPW, bool PRELU>
__global__ __launch_bounds__(256) void dwproj_kernel(const DwProjArgs a)
{
    DP_STAMP(0);
    extern __shared__ __align__(16) unsigned char lds[];
    unsigned char *wpl = lds;                                          // [16*COT][rsw] packed projection weights
    int8_t *wdl = reinterpret_cast<int8_t *>(lds + a.off_wd);          // [nch][9][64]
    v4i *pd = reinterpret_cast<v4i *>(lds + a.off_pd);                 // [nch*64]
    v4i *pp = reinterpret_cast<v4i *>(lds + a.off_pp);                 // [16*COT]
    unsigned char *t1 = lds + a.off_t1;                                // [2][4 planes][RI][W+2][16], then 16 spare bytes

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, g = lane >> 4;

    const int img = blockIdx.x / a.bands;
    const int band = blockIdx.x - img * a.bands;
    const int ro0 = band * a.R;
    const int rows_out = min(a.R, a.Ho - ro0);
    const int iy0 = ro0 * a.stride - 1;  // first input row of the band (may be -1)
    const int W = a.W, Wo = a.Wo, C = a.C, cout = a.cout, s = a.stride, nch = a.nch;
    const int W2 = W + 2;
    const int plane = a.plane;
    const int slice = 4 * plane;  // bytes of one buffer of t1
    const int npix2 = rows_out * Wo;
    unsigned char *dump = t1 + 2 * slice;

    const __amdgpu_buffer_rsrc_t rt =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a.t), 0, a.N * a.H * W * C, kBufFlags);

    // ---- this thread's pieces of a slice: piece p = tid + 256*r is channels 16*(p & 3).. of pixel
    // p >> 2 of the band's input rows -------------------------------------------------------------
    unsigned g_off[kDpPieces];
    int l_off[kDpPieces];
#pragma unroll
    for (int r = 0; r < kDpPieces; ++r) {
        const int p = tid + 256 * r;
        const int ct = p & 3, pix = p >> 2;
        const int row = pix / W, col = pix - row * W;
        const int iy = iy0 + row;
        const bool ok = row < a.RI && iy >= 0 && iy < a.H;
        g_off[r] = ok ? (unsigned)(((img * a.H + iy) * W + col) * C + 16 * ct) : (unsigned)kOobOffset;
        l_off[r] = ok ? ct * plane + (row * W2 + col + 1) * 16 : -1;
    }
    v4i S[kDpAhead][kDpPieces];
    auto load_slice = [&](v4i(&slot)[kDpPieces], int c) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < kDpPieces; ++r) {
            // channels beyond C (ragged last chunk) and chunks beyond the last read as zero
            const bool in = kDpCH * c + 16 * ((tid + 256 * r) & 3) < C;
            const unsigned off = in ? min(g_off[r] + (unsigned)(kDpCH * c), (unsigned)kOobOffset) : (unsigned)kOobOffset;
            slot[r] = __builtin_amdgcn_raw_buffer_load_b128(rt, (int)off, 0, 0);
        }
    };
    auto put_slice = [&](const v4i(&slot)[kDpPieces], int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < kDpPieces; ++r) {
            unsigned char *dst = l_off[r] >= 0 ? t1 + buf * slice + l_off[r] : dump;
            *reinterpret_cast<v4i *>(dst) = slot[r];
        }
    };
#pragma unroll
    for (int u = 0; u < kDpAhead; ++u) load_slice(S[u], u);

    // ---- staged once per workgroup: packed projection weights, depthwise weights, parameters; the
    // activation tile zeroed (its border and the rows outside the image stay zero).  Every loop
    // issues a batch of global loads before it stores the first of them to LDS: a load-store pair
    // per iteration would pay one memory latency per iteration ------------------------------------
    {
        const v4i zero4 = {0, 0, 0, 0};
        for (int idx = tid; idx < 2 * slice / 16; idx += 256) reinterpret_cast<v4i *>(t1)[idx] = zero4;
        const int KWp = (C + 15) >> 4;
        if (a.wp_vec) {
            // rows of whole 16-byte pieces, 16-byte aligned
            const int rq = a.rsw >> 4, gq = KWp >> 2;
            const int count = 16 * COT * rq;
            constexpr int U = 10;
            for (int base = 0; base < count; base += 256 * U) {
                v4i v[U];
#pragma unroll
                for (int q = 0; q < U; ++q) {
                    const int idx = base + q * 256 + tid;
                    const int row = idx / rq, k4 = idx - row * rq;
                    const bool ok = idx < count && row < cout && k4 < gq;
                    const v4i w = *reinterpret_cast<const v4i *>(a.wp + (ok ? (long long)row * KWp + 4 * k4 : 0));
                    v[q] = ok ? w : zero4;
                }
#pragma unroll
                for (int q = 0; q < U; ++q) {
                    const int idx = base + q * 256 + tid;
                    if (idx < count) reinterpret_cast<v4i *>(wpl)[idx] = v[q];
                }
            }
        } else {
            const int rsw4 = a.rsw >> 2;
            const int count = 16 * COT * rsw4;
            constexpr int U = 16;
            for (int base = 0; base < count; base += 256 * U) {
                uint32_t v[U];
#pragma unroll
                for (int q = 0; q < U; ++q) {
                    const int idx = base + q * 256 + tid;
                    const int row = idx / rsw4, kw = idx - row * rsw4;
                    const bool ok = idx < count && row < cout && kw < KWp;
                    const uint32_t w = a.wp[ok ? (long long)row * KWp + kw : 0];
                    v[q] = ok ? w : 0u;
                }
#pragma unroll
                for (int q = 0; q < U; ++q) {
                    const int idx = base + q * 256 + tid;
                    if (idx < count) reinterpret_cast<uint32_t *>(wpl)[idx] = v[q];
                }
            }
        }
        {
            // depthwise weights [9][C] -> [chunk][9][64], four channels (one dword) at a time
            const int c4n = C >> 2;  // dwords per tap row (C % 16 == 0)
            const int count = nch * 9 * (kDpCH / 4);
            const uint32_t *wd4 = reinterpret_cast<const uint32_t *>(a.wd);
            constexpr int U = 10;
            for (int base = 0; base < count; base += 256 * U) {
                uint32_t v[U];
#pragma unroll
                for (int q = 0; q < U; ++q) {
                    const int idx = base + q * 256 + tid;
                    const int ch = idx / (9 * 16), rem = idx - ch * (9 * 16);
                    const int tap = rem >> 4, c4 = ch * 16 + (rem & 15);
                    const bool ok = idx < count && c4 < c4n;
                    const uint32_t w = wd4[ok ? tap * c4n + c4 : 0];
                    v[q] = ok ? w : 0u;
                }
#pragma unroll
                for (int q = 0; q < U; ++q) {
                    const int idx = base + q * 256 + tid;
                    if (idx < count) reinterpret_cast<uint32_t *>(wdl)[idx] = v[q];
                }
            }
        }
        {
            constexpr int U = 4;
            const int count = nch * kDpCH;
            for (int base = 0; base < count; base += 256 * U) {
                int pb[U], pm[U], pn[U], ps[U];
#pragma unroll
                for (int q = 0; q < U; ++q) {
                    const int idx = base + q * 256 + tid;
                    const int ci = idx < C ? idx : 0;
                    pb[q] = a.bd[ci]; pm[q] = a.md[ci]; ps[q] = a.sd[ci];
                    pn[q] = a.nd ? a.nd[ci] : pm[q];
                }
#pragma unroll
                for (int q = 0; q < U; ++q) {
                    const int idx = base + q * 256 + tid;
                    if (idx < count) pd[idx] = idx < C ? requant_params(pb[q], pm[q], pn[q], ps[q], PRELU) : v4i{0, 0, 0, 1};
                }
            }
        }
        for (int idx = tid; idx < 16 * COT; idx += 256) {
            v4i p = {0, 0, 0, 1};
            if (idx < cout) p = requant_params(a.bp[idx], a.mp[idx], a.np ? a.np[idx] : a.mp[idx], a.sp[idx], a.np != nullptr);
            pp[idx] = p;
        }
    }
    DP_STAMP(1);
    __syncthreads();  // the zeroing is done before the first slice lands
    DP_STAMP(2);
    put_slice(S[0], 0);
    load_slice(S[0], kDpAhead);

    v4i acc[TPW][COT];
#pragma unroll
    for (int k = 0; k < TPW; ++k)
#pragma unroll
        for (int u = 0; u < COT; ++u) acc[k][u] = v4i{0, 0, 0, 0};
    const int lo_d = in_vgpr(a.lo_d), hi_d = in_vgpr(a.hi_d);

    // LDS offsets of this lane's pixels (tap (0,0), plane 0) and of its tap in each tap group
    int poff[TPW];
#pragma unroll
    for (int k = 0; k < TPW; ++k) {
        // tiles beyond the band are computed on its last pixel and never stored
        const int p = min((wave + 4 * k) * 16 + j, npix2 - 1);
        const int oy = p / Wo, ox = p - oy * Wo;
        poff[k] = ((oy * s) * W2 + ox * s) * 16;
    }
    int toff[3];
#pragma unroll
    for (int q = 0; q < 3; ++q) {
        const int tap = min(4 * q + g, 8);  // lanes whose tap does not exist read tap 8 again, against zero weights
        toff[q] = ((tap / 3) * W2 + tap % 3) * 16;
    }
    const int dsel = j >> 2, dsh = 8 * (j & 3);  // where the lane's one weight sits in its A operand
    const int my_tiles = (npix2 + 15) >> 4;      // pixel tiles of the band
    __syncthreads();
    DP_STAMP(3);

    auto chunk = [&](const int c, v4i(&slot)[kDpPieces]) __attribute__((always_inline)) {
        if (c >= nch) return;  // uniform: every wavefront skips the same chunks and barriers
        const unsigned char *tb = t1 + (c & 1) * slice;
        const int8_t *wdl_c = wdl + c * (9 * kDpCH);
        const v4i *pd_c = pd + c * kDpCH;
        // A operands of the depthwise MFMAs: for channel tile t and tap group q the weight of channel
        // 16t + j under tap 4q + g at byte j of the 16, zero elsewhere
        v4i adw[4][3];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int q = 0; q < 3; ++q) {
                const int tap = 4 * q + g;
                const uint32_t wb = tap < 9 ? (uint32_t)(uint8_t)wdl_c[min(tap, 8) * kDpCH + 16 * t + j] : 0u;
                const int val = (int)(wb << dsh);
                adw[t][q] = v4i{dsel == 0 ? val : 0, dsel == 1 ? val : 0, dsel == 2 ? val : 0, dsel == 3 ? val : 0};
            }
        v4i b2[TPW];
#pragma unroll
        for (int k = 0; k < TPW; ++k) {
            if ((wave + 4 * k) < my_tiles) {  // uniform per wavefront
                // the four channel tiles are four independent MFMA chains: tap groups outermost, so
                // that a chain's next MFMA finds the previous one finished
                const unsigned char *src = tb + poff[k];
                v4i accd[4];
                const v4i zero4 = {0, 0, 0, 0};
#pragma unroll
                for (int q = 0; q < 3; ++q) {
                    v4i bq[4];
#pragma unroll
                    for (int t = 0; t < 4; ++t) bq[t] = *reinterpret_cast<const v4i *>(src + t * plane + toff[q]);
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        accd[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(adw[t][q], bq[t], q == 0 ? zero4 : accd[t], 0, 0, 0);
                }
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    int v[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const v4i pr = pd_c[16 * t + 4 * g + r];
                        v[r] = PRELU ? requant_prelu_i64(accd[t][r], pr, lo_d, hi_d) : requant_i64<true>(accd[t][r], pr, lo_d, hi_d);
                    }
                    b2[k][t] = (int)pack4_low_bytes(v[0], v[1], v[2], v[3]);
                }
            }
        }
        // ---- projection: one k step per chunk.  k order of the step: lane g, byte 4t + r <-> hidden
        // channel 64c + 16t + 4g + r, which is where the depthwise stage left its outputs.  The
        // packed rows of two output tiles are read ahead of their decode ----------------------------
        const unsigned char *wrow = wpl + j * a.rsw + 16 * c;
        v4i q4n[2];
        q4n[0] = *reinterpret_cast<const v4i *>(wrow);
        if constexpr (COT > 1) q4n[1] = *reinterpret_cast<const v4i *>(wrow + 16 * a.rsw);
#pragma unroll
        for (int u = 0; u < COT; ++u) {
            const v4i q4 = q4n[u & 1];
            if (u + 2 < COT) q4n[u & 1] = *reinterpret_cast<const v4i *>(wrow + (u + 2) * 16 * a.rsw);
            v4i ap;
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
                const uint32_t sel = (((uint32_t)q4[tt] >> (2 * g)) & 0x03030303u) << 1;
                ap[tt] = (int)__builtin_amdgcn_perm(0x00FF0000u, 0x00010000u, sel);
            }
#pragma unroll
            for (int k = 0; k < TPW; ++k)
                if ((wave + 4 * k) < my_tiles)
                    acc[k][u] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ap, b2[k], acc[k][u], 0, 0, 0);
        }
        // ---- the next chunk's slice into the other buffer (last read one chunk ago, behind the
        // barrier), a new slice on its way ----------------------------------------------------------
        put_slice(slot, (c + 1) & 1);
        load_slice(slot, c + 1 + kDpAhead);
        __syncthreads();
        DP_STAMP(4 + c);
    };
    for (int c = 0; c < nch; c += kDpAhead) {
#pragma unroll
        for (int d = 0; d < kDpAhead; ++d) chunk(c + d, S[(d + 1) % kDpAhead]);
    }

    // ---- projection epilogue: requantise, skip connection, store ------------------------------
    const int lo_p = in_vgpr(a.lo_p), hi_p = in_vgpr(a.hi_p);
    const int m128 = in_vgpr(-128), p127 = in_vgpr(127);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, a.N * a.Ho * Wo * cout, kBufFlags);
    const __amdgpu_buffer_rsrc_t rres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.res ? a.res : a.y), 0, a.N * a.Ho * Wo * cout, kBufFlags);
#pragma unroll
    for (int k = 0; k < TPW; ++k) {
        const int p = (wave + 4 * k) * 16 + j;
        const bool pvalid = p < npix2;
        const int oy = p / Wo, ox = p - oy * Wo;
        const int opix = (img * a.Ho + ro0 + oy) * Wo + ox;
#pragma unroll
        for (int u = 0; u < COT; ++u) {
            const int cc = 16 * u + 4 * g;
            if (cc < cout) {
                int v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    v[r] = a.np ? requant_prelu_i64(acc[k][u][r], pp[cc + r], lo_p, hi_p)
                                : requant_i64<true>(acc[k][u][r], pp[cc + r], lo_p, hi_p);
                if (a.res) {
                    const uint32_t res = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(
                        rres, pvalid ? opix * cout + cc : kOobOffset, 0, 0);
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = med3_i32(v[r] + sbyte(res, r), m128, p127);
                }
                __builtin_amdgcn_raw_buffer_store_b32((int)pack4_low_bytes(v[0], v[1], v[2], v[3]), ry,
                                                      pvalid ? opix * cout + cc : kOobOffset, 0, 0);
            }
        }
    }
    DP_STAMP(30);
#ifdef PROM_TIMELINE
    __builtin_amdgcn_s_waitcnt(0);
    DP_STAMP(31);
#endif
}

using DwProjFn = void (*)(const DwProjArgs);

inline int dp_align16(int v) { return (v + 15) & ~15; }

// Output-channel tiles and pixel tiles per wavefront of the instantiation for a cout (the
// projection accumulators are 4 * COT * TPW registers); COT = 0: no instantiation.
static void dwproj_shape(int cout, int *cot, int *tpw)
{
    *cot = cout <= 32 ? 2 : cout <= 64 ? 4 : cout <= 96 ? 6 : cout <= 160 ? 10 : cout <= 320 ? 20 : 0;
    *tpw = *cot <= 6 ? 4 : *cot == 10 ? 2 : 1;
}

constexpr int kDpLdsMax = 150 * 1024;

// Plans the kernel for a shape: band height, LDS layout, kernel, grid.  false if it does not apply.
static bool plan_dwproj(DwProjArgs &a, DwProjFn &fn, size_t &lds, int &grid, bool prelu)
{
    int cot = 0, tpw = 0;
    dwproj_shape(a.cout, &cot, &tpw);
    if (cot == 0 || a.C % 16 != 0 || a.cout % 4 != 0) return false;
    if ((long long)a.N * a.H * a.W * a.C >= (long long)kOobOffset) return false;
    if ((long long)a.N * a.Ho * a.Wo * a.cout >= (long long)kOobOffset) return false;
    a.nch = (a.C + kDpCH - 1) / kDpCH;
    a.rsw = 16 * (a.nch | 1);  // an odd number of 16-byte slots per row spreads the rows over the banks
    const int s = a.stride;
    // Band height, within what a workgroup can hold (16 * 4 * TPW output pixels, a slice of 256
    // input pixels, the LDS limit): the highest band that still gives every CU two workgroups;
    // failing that (small batches) the lowest band that keeps all four wavefronts busy.
    const long long fixed = (long long)16 * cot * a.rsw + (long long)a.nch * (9 * kDpCH + kDpCH * 16) + 16 * cot * 16 + 16;
    int best = 0, best_full = 0, best_busy = 0;
    for (int R = 1; R <= a.Ho; ++R) {
        const int RI = (R - 1) * s + 3;
        if (R * a.Wo > 64 * tpw || RI * a.W > 64 * kDpPieces) break;
        const long long bytes = fixed + 2LL * 4 * RI * (a.W + 2) * 16;
        if (bytes > kDpLdsMax) break;
        const int bands = (a.Ho + R - 1) / R;
        best = R;
        if ((long long)a.N * bands >= 512) best_full = R;
        if (best_busy == 0 && (R * a.Wo + 15) / 16 >= 4) best_busy = R;
    }
    if (best_full)
        best = best_full;
    else if (best_busy)
        best = best_busy;
    if (best == 0) return false;
    a.R = best;
    a.RI = (best - 1) * s + 3;
    a.bands = (a.Ho + best - 1) / best;
    a.plane = a.RI * (a.W + 2) * 16;
    int off = 16 * cot * a.rsw;
    a.off_wd = off; off += dp_align16(a.nch * 9 * kDpCH);
    a.off_pd = off; off += a.nch * kDpCH * 16;
    a.off_pp = off; off += 16 * cot * 16;
    a.off_t1 = off; off += 2 * 4 * a.plane + 16;
    lds = (size_t)off;
    fn = cot == 2    ? (prelu ? &dwproj_kernel<2, 4, true> : &dwproj_kernel<2, 4, false>)
         : cot == 4  ? (prelu ? &dwproj_kernel<4, 4, true> : &dwproj_kernel<4, 4, false>)
         : cot == 6  ? (prelu ? &dwproj_kernel<6, 4, true> : &dwproj_kernel<6, 4, false>)
         : cot == 10 ? (prelu ? &dwproj_kernel<10, 2, true> : &dwproj_kernel<10, 2, false>)
                     : (prelu ? &dwproj_kernel<20, 1, true> : &dwproj_kernel<20, 1, false>);
    const long long gsz = (long long)a.N * a.bands;
    if (gsz > (1LL << 30)) return false;
    grid = (int)gsz;
    return true;
}

static bool dp_overlaps(const void *p, size_t pn, const void *q, size_t qn)
{
    const uintptr_t a = (uintptr_t)p, b = (uintptr_t)q;
    return a < b + qn && b < a + pn;
}

}  // namespace prom

extern "C" int prom_dw_pw_can_fuse(int n, int h, int w, int c, int cout, int stride)
{
    using namespace prom;
    if (n <= 0 || h <= 0 || w <= 0 || c <= 0 || cout <= 0 || (stride != 1 && stride != 2)) return PROM_EINVAL;
    DwProjArgs a = {};
    a.N = n; a.H = h; a.W = w; a.Ho = (h - 1) / stride + 1; a.Wo = (w - 1) / stride + 1;
    a.C = c; a.cout = cout; a.stride = stride;
    DwProjFn fn = nullptr;
    size_t lds = 0;
    int grid = 0;
    return plan_dwproj(a, fn, lds, grid, false) ? 1 : 0;
}

extern "C" int prom_dw_pw_conv(const int8_t *x, int n, int h, int w, int c, const int8_t *w_dw, int stride,
                               const prom_requant_t *rq_dw, const void *w_project_packed, int cout,
                               const prom_requant_t *rq_project, const int8_t *residual, int8_t *y, void *stream)
{
    using namespace prom;
    if (!x || !w_dw || !w_project_packed || !rq_dw || !rq_project || !y) return PROM_EINVAL;
    if (n <= 0 || h <= 0 || w <= 0 || c <= 0 || cout <= 0 || (stride != 1 && stride != 2)) return PROM_EINVAL;
    const prom_requant_t *rqs[2] = {rq_dw, rq_project};
    for (const prom_requant_t *rq : rqs) {
        if (!rq->bias || !rq->mult || !rq->shift) return PROM_EINVAL;
        if (rq->act_min < -128 || rq->act_max > 127 || rq->act_min > rq->act_max) return PROM_EINVAL;
    }
    if ((((uintptr_t)x | (uintptr_t)y | (uintptr_t)residual | (uintptr_t)w_project_packed | (uintptr_t)w_dw) & 3) != 0)
        return PROM_EUNSUPPORTED;
    DwProjArgs a = {};
    a.t = x; a.wd = w_dw; a.wp = static_cast<const uint32_t *>(w_project_packed);
    a.bd = rq_dw->bias; a.md = rq_dw->mult; a.sd = rq_dw->shift; a.nd = rq_dw->mult_neg;
    a.bp = rq_project->bias; a.mp = rq_project->mult; a.sp = rq_project->shift; a.np = rq_project->mult_neg;
    a.res = residual; a.y = y;
    a.N = n; a.H = h; a.W = w; a.Ho = (h - 1) / stride + 1; a.Wo = (w - 1) / stride + 1;
    a.C = c; a.cout = cout; a.stride = stride;
    a.lo_d = rq_dw->act_min; a.hi_d = rq_dw->act_max;
    a.lo_p = rq_project->act_min; a.hi_p = rq_project->act_max;
    {
        const size_t xb = (size_t)n * h * w * c, yb = (size_t)n * a.Ho * a.Wo * cout;
        if (dp_overlaps(y, yb, x, xb)) return PROM_EALIAS;
        if (residual && residual != y && dp_overlaps(y, yb, residual, yb)) return PROM_EALIAS;
    }
    DwProjFn fn = nullptr;
    size_t lds = 0;
    int grid = 0;
    if (!plan_dwproj(a, fn, lds, grid, a.nd != nullptr)) return PROM_EUNSUPPORTED;
    a.wp_vec = (((c + 15) / 16) % 4 == 0 && ((uintptr_t)w_project_packed & 15) == 0) ? 1 : 0;
    {
        static std::mutex mu;
        static std::vector<DwProjFn> attr_done;
        std::lock_guard<std::mutex> lock(mu);
        bool done = false;
        for (DwProjFn f : attr_done) done |= f == fn;
        if (!done) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(fn),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess && lds > 64 * 1024) {
                last_hip_error() = e;
                (void)hipGetLastError();
                return PROM_EHIP;
            }
            attr_done.push_back(fn);
        }
    }
    clear_hip_error();
    DwProjArgs args = a;
    void *kargs[] = {&args};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(fn), dim3(grid), dim3(256), kargs, lds,
                                         static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        last_hip_error() = e;
        (void)hipGetLastError();
        return PROM_EHIP;
    }
    return check_launch();
}

#ifdef PROM_TIMELINE
extern "C" int prom_debug_dp_stamps(unsigned long long *host)
{
    if (hipDeviceSynchronize() != hipSuccess) return PROM_EHIP;
    return hipMemcpyFromSymbol(host, HIP_SYMBOL(prom::g_dp_stamps), sizeof(unsigned long long) * 64 * 32) == hipSuccess ? PROM_OK : PROM_EHIP;
}
#endif
