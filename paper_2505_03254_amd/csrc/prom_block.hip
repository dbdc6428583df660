// Inverted-residual block: ternary pointwise expand -> int8 depthwise 3x3 -> ternary pointwise
// project (+ saturating skip), paper Section 2 and Figure 4.
//
// Fused kernel.  The expanded tensor is 6x wider than the block's input and output; written to
// HBM between the three layers it is >90 % of the block's traffic.  The fused kernel keeps it in
// LDS: a workgroup owns a band of R output rows of one image and walks over the hidden
// channels in chunks of 64:
//   stage 1  expand the band's input rows (R*stride + 2 with the halo) for 64 hidden channels
//            with int8 MFMA, requantise, store as int8 into an LDS tile with a zero border;
//   stage 2  depthwise 3x3 on that tile, also on the matrix cores: for 16 channels the 64-deep k
//            dimension holds 4 taps x 16 channels (the B operand of lane (pixel, g) is the 16
//            channel bytes of the pixel under tap 4q + g, one LDS read; the A operand is zero
//            except the one weight of the lane's channel and tap), so 3 MFMAs cover the 9 taps
//            of 16 pixels x 16 channels, against 144 vector-ALU multiply-adds per lane;
//   stage 3  the requantised depthwise outputs of a lane (its pixel, 16 of the 64 hidden
//            channels) are, packed, exactly a B operand of the projection MFMA: one 64-deep k
//            step per chunk with the projection weights decoded in the matching channel order;
//            nothing goes back to LDS, the accumulators live in registers across chunks.
// After the last chunk the projection is requantised, the block input is added (skip) and the
// band is written.  HBM traffic is the block input (rows of the halo are read twice) and output.
// Shapes the fused kernel does not take run as three launches through the caller's workspace.
#include "prom_pw_stream.h"
#include "prom_launch.h"
#include "prom_block_planes.h"

#include <mutex>
#include <vector>

namespace prom {

struct BlockArgs {
    const int8_t *x;
    int8_t *y;
    const uint32_t *we;  // packed expand weights [chid][cin]
    const int8_t *wd;    // depthwise weights [3][3][chid]
    const uint32_t *wp;  // packed project weights [cout][chid]
    const int32_t *be, *me, *se;  // expand bias / mult / shift [chid]
    const int32_t *bd, *md, *sd;  // depthwise [chid]
    const int32_t *bp, *mp, *sp;  // project [cout]
    const int32_t *ne, *nd, *np;  // PReLU negative-side multipliers of the three layers, or nullptr
    int N, H, W, Ho, Wo, cin, chid, cout, stride;
    int R;        // output rows per band
    int bands;    // bands per image
    int RI;       // input rows per band = (R-1)*stride + 3
    int add_res;
    int lo_e, hi_e, lo_d, hi_d, lo_p, hi_p;
    // LDS byte offsets
    int off_t1, off_t2, off_fe, off_fp, off_pe, off_pd, off_pp, off_wd;
};

constexpr int kCH = 64;  // hidden channels per chunk = one k step of the projection

// Parameters of channel c of a layer in the form its epilogue takes (mneg == nullptr: plain).
__device__ __forceinline__ v4i make_par(const int32_t *b, const int32_t *m, const int32_t *mneg,
                                        const int32_t *s, int c)
{
    return requant_params(b[c], m[c], mneg ? mneg[c] : 0, s[c], mneg != nullptr);
}

// prelu is uniform over the launch.
__device__ __forceinline__ int requant_sel(bool prelu, int accv, const v4i &pr, int lo, int hi)
{
    return prelu ? requant_prelu_i64(accv, pr, lo, hi) : requant_i64<true>(accv, pr, lo, hi);
}

// COT: 16-channel output tiles (cout <= 16*COT); TPW: projection pixel tiles per wavefront;
// PRELU: the expand and depthwise epilogues take the PReLU form (a layer of the two without
// negative-side multipliers then runs it with mult_neg = mult, which is the plain form), so that
// neither hot loop has a branch per output.
template <int COT, int TPW, bool PRELU>
__global__ __launch_bounds__(256, 2) void block_fused_kernel(const BlockArgs a)
{
    extern __shared__ __align__(16) unsigned char lds[];
    int8_t *xs = reinterpret_cast<int8_t *>(lds);                      // [RI][W][cin padded to 16] (+64 pad)
    // the expanded band as 4 planes of 16 channels, [4][RI][W+2][16]: a wavefront's 16-byte reads
    // of one plane (consecutive pixels) then fall into different banks
    int8_t *t1 = reinterpret_cast<int8_t *>(lds + a.off_t1);
    v4i *fe = reinterpret_cast<v4i *>(lds + a.off_fe);                 // [chunk][4 tiles][KSe][64 lanes]
    v4i *fp = reinterpret_cast<v4i *>(lds + a.off_fp);                 // [chunk][COT][64 lanes]
    v4i *pe = reinterpret_cast<v4i *>(lds + a.off_pe);                 // [chunk][64] expand parameters
    v4i *pd = reinterpret_cast<v4i *>(lds + a.off_pd);                 // [chunk][64] depthwise parameters
    v4i *pp = reinterpret_cast<v4i *>(lds + a.off_pp);                 // [16*COT] project parameters
    int8_t *wdl = reinterpret_cast<int8_t *>(lds + a.off_wd);          // [chunk][9][64] depthwise weights

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, g = lane >> 4;

    const int img = blockIdx.x / a.bands;
    const int band = blockIdx.x - img * a.bands;
    const int ro0 = band * a.R;                       // first output row of the band
    const int rows_out = min(a.R, a.Ho - ro0);        // valid output rows
    const int ri0 = ro0 * a.stride - 1;               // first input row (may be -1)
    const int W = a.W, Wo = a.Wo, cin = a.cin, chid = a.chid, cout = a.cout, s = a.stride;
    const int KSe = (cin + 63) >> 6, KWe = (cin + 15) >> 4, KWp = (chid + 15) >> 4;
    const int W2 = W + 2;
    const int plane = a.RI * W2 * 16;  // bytes of one 16-channel plane of t1
    const int npix1 = a.RI * W;                       // pixels expanded per chunk
    const int npix2 = rows_out * Wo;                  // output pixels of the band

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.x), 0, a.N * a.H * W * cin, kBufFlags);

    // ---- stage 0: the band's input rows into LDS, pixels padded to a multiple of 16 bytes (rows
    // outside the image read as zero or as a neighbouring image; the expanded rows are forced to
    // zero below, so either is fine; the padding bytes meet zero weights) ------------------------
    const int cinp = (cin + 15) & ~15;
    {
        const int row_bytes = W * cin;
        const int total = a.RI * row_bytes;  // multiple of 8
        const long long base = ((long long)img * a.H + ri0) * row_bytes;
        const int pieces = cin >> 3;  // 8-byte pieces per pixel
        for (int o = tid * 8; o < total; o += 256 * 8) {
            const long long go = base + o;
            const int off = (go >= 0 && go < (long long)kOobOffset) ? (int)go : kOobOffset;
            const v2i v = __builtin_amdgcn_raw_buffer_load_b64(rx, off, 0, 0);
            const int pc = o >> 3;
            const int px = pc / pieces;
            *reinterpret_cast<v2i *>(xs + px * cinp + 8 * (pc - px * pieces)) = v;
        }
        // project parameters (used after the last chunk)
        if (tid < 16 * COT) {
            v4i p = {0, 0, 0, 1};
            if (tid < cout) p = make_par(a.bp, a.mp, a.np, a.sp, tid);
            pp[tid] = p;
        }
    }

    v4i acc[TPW][COT];
#pragma unroll
    for (int q = 0; q < TPW; ++q)
#pragma unroll
        for (int t = 0; t < COT; ++t) acc[q][t] = v4i{0, 0, 0, 0};

    const int lo_e = in_vgpr(a.lo_e), hi_e = in_vgpr(a.hi_e);
    const int lo_d = in_vgpr(a.lo_d), hi_d = in_vgpr(a.hi_d);

    // ---- weights and parameters of all chunks (one memory latency for the whole block) ----------
    const int nchunks = (chid + kCH - 1) / kCH;
    const int fe_chunk = 4 * KSe * 64;  // expand fragments per chunk
    for (int idx = tid; idx < nchunks * fe_chunk; idx += 256) {
        const int ch = idx / fe_chunk, rem = idx - ch * fe_chunk;
        const int l = rem & 63, tk = rem >> 6, ks = tk % KSe, t = tk / KSe;
        const int c = ch * kCH + 16 * t + (l & 15);
        const int kw = 4 * ks + (l >> 4);
        const bool ok = c < chid && kw < KWe;
        const uint32_t wv = a.we[ok ? (long long)c * KWe + kw : 0];
        fe[idx] = decode_word(ok ? wv : 0u);
    }
    for (int idx = tid; idx < nchunks * COT * 64; idx += 256) {
        // project fragments, one k step per chunk.  k order of the step: lane kg, byte 4t + b  <->
        // hidden channel c0 + 16t + 4kg + b, which is where stage 2 leaves the depthwise outputs
        const int ch = idx / (COT * 64), rem = idx - ch * (COT * 64);
        const int l = rem & 63, t = rem >> 6;
        const int c = 16 * t + (l & 15);
        const int kg = l >> 4;
        v4i e = {0, 0, 0, 0};
        if (c < cout) {
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
                const int kw = 4 * ch + tt;
                if (kw < KWp) {
                    const uint32_t wv = a.wp[(long long)c * KWp + kw];
                    const uint32_t sel = ((wv >> (2 * kg)) & 0x03030303u) << 1;
                    e[tt] = (int)__builtin_amdgcn_perm(0x00FF0000u, 0x00010000u, sel);
                }
            }
        }
        fp[idx] = e;
    }
    for (int idx = tid; idx < nchunks * kCH; idx += 256) {
        v4i e = {0, 0, 0, 1}, d = {0, 0, 0, 1};
        if (idx < chid) {
            e = requant_params(a.be[idx], a.me[idx], a.ne ? a.ne[idx] : a.me[idx], a.se[idx], PRELU);
            d = requant_params(a.bd[idx], a.md[idx], a.nd ? a.nd[idx] : a.md[idx], a.sd[idx], PRELU);
        }
        pe[idx] = e;
        pd[idx] = d;
    }
    for (int idx = tid; idx < nchunks * 9 * kCH; idx += 256) {
        const int ch = idx / (9 * kCH), rem = idx - ch * (9 * kCH);
        const int tap = rem >> 6, c = ch * kCH + (rem & 63);
        wdl[idx] = c < chid ? a.wd[tap * chid + c] : (int8_t)0;
    }
    // zero border columns of t1 (col -1 and col W of every row, in each of the 4 planes); stage 1
    // never writes them
    for (int idx = tid; idx < a.RI * 2 * (kCH / 4); idx += 256) {
        const int q = idx % (kCH / 4), rc = idx / (kCH / 4);
        const int row = rc >> 1, col = (rc & 1) ? W + 1 : 0;
        *reinterpret_cast<uint32_t *>(t1 + (q >> 2) * plane + (row * W2 + col) * 16 + 4 * (q & 3)) = 0u;
    }
    __syncthreads();

    for (int ch = 0; ch < nchunks; ++ch) {
        const v4i *fe_c = fe + ch * fe_chunk;
        const v4i *fp_c = fp + ch * (COT * 64);
        const v4i *pe_c = pe + ch * kCH;
        const v4i *pd_c = pd + ch * kCH;
        const int8_t *wdl_c = wdl + ch * (9 * kCH);
        if (ch) __syncthreads();  // the depthwise reads of the previous chunk are done with t1

        // ---- stage 1: expand 64 hidden channels for every pixel of the band's input rows; the
        // activation fragment of a pixel tile serves the 4 channel tiles ------------------------
        {
            v4i pare[4][4];  // channel 16t + 4g + r
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) pare[t][r] = pe_c[16 * t + 4 * g + r];
            for (int pt = wave; pt * 16 < npix1; pt += 4) {
                const int p = pt * 16 + j;
                v4i d4[4];
                const int8_t *xp = xs + min(p, npix1 - 1) * cinp + 16 * g;
                {
                    // 16 k-bytes of pixel p; bytes beyond cin meet zero weights
                    const v4i b = *reinterpret_cast<const v4i *>(xp);
                    const v4i zero4 = {0, 0, 0, 0};
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        d4[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fe_c[(t * KSe) * 64 + lane], b, zero4, 0, 0, 0);
                }
                for (int ks = 1; ks < KSe; ++ks) {
                    const v4i b = *reinterpret_cast<const v4i *>(xp + 64 * ks);
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        d4[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fe_c[(t * KSe + ks) * 64 + lane], b, d4[t], 0, 0, 0);
                }
                if (p < npix1) {
                    const int row = p / W, col = p - row * W;
                    const int ri = ri0 + row;
                    const bool inimg = ri >= 0 && ri < a.H;
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        int v[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) v[r] = requant_sel(PRELU, d4[t][r], pare[t][r], lo_e, hi_e);
                        const uint32_t o = inimg ? pack4_low_bytes(v[0], v[1], v[2], v[3]) : 0u;
                        *reinterpret_cast<uint32_t *>(t1 + t * plane + (row * W2 + col + 1) * 16 + 4 * g) = o;
                    }
                }
            }
        }
        __syncthreads();

        // ---- stages 2 and 3: depthwise 3x3 by MFMA on the LDS tile, then the projection -----------
        {
            // the lane's A operands of the depthwise MFMAs: for channel tile t and tap group q
            // the weight of channel 16t + (lane & 15) under tap 4q + (lane >> 4), at byte
            // (lane & 15) of the 16, zero elsewhere
            const int li = lane & 15;
            v4i adw[4][3];
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int q = 0; q < 3; ++q) {
                    const int tap = 4 * q + g;
                    const uint32_t wb = tap < 9 ? (uint32_t)(uint8_t)wdl_c[tap * kCH + 16 * t + li] : 0u;
                    const uint32_t val = wb << (8 * (li & 3));
                    adw[t][q] = v4i{(li >> 2) == 0 ? (int)val : 0, (li >> 2) == 1 ? (int)val : 0,
                                    (li >> 2) == 2 ? (int)val : 0, (li >> 2) == 3 ? (int)val : 0};
                }
            v4i pard[4][4];  // channel 16t + 4g + r
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) pard[t][r] = pd_c[16 * t + 4 * g + r];
            int toff[3];  // LDS offset of the lane's tap in each tap group (tap 8 again where there is none)
#pragma unroll
            for (int q = 0; q < 3; ++q) {
                const int tap = min(4 * q + g, 8);
                toff[q] = ((tap / 3) * W2 + tap % 3) * 16;
            }
#pragma unroll
            for (int q2 = 0; q2 < TPW; ++q2) {
                const int pt = wave + 4 * q2;
                {   // tiles beyond the band are computed on its last pixel and never stored: no
                    // branch, so that the tiles of a wavefront can overlap
                    const int p = min(pt * 16 + j, npix2 - 1);
                    const int oy = p / Wo, ox = p - oy * Wo;
                    const int8_t *src = t1 + ((oy * s) * W2 + ox * s) * 16;  // tap (0, 0) of the pixel, plane 0
                    v4i accd[4];
                    const v4i zero4 = {0, 0, 0, 0};
#pragma unroll
                    for (int q = 0; q < 3; ++q) {
#pragma unroll
                        for (int t = 0; t < 4; ++t) {
                            // lanes whose tap does not exist (9..11) read tap 8 again, against zero weights
                            const v4i b = *reinterpret_cast<const v4i *>(src + toff[q] + t * plane);
                            accd[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(adw[t][q], b, q == 0 ? zero4 : accd[t], 0, 0, 0);
                        }
                    }
                    v4i b2;
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        int v[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) v[r] = requant_sel(PRELU, accd[t][r], pard[t][r], lo_d, hi_d);
                        b2[t] = (int)pack4_low_bytes(v[0], v[1], v[2], v[3]);
                    }
#pragma unroll
                    for (int t = 0; t < COT; ++t)
                        acc[q2][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fp_c[t * 64 + lane], b2, acc[q2][t], 0, 0, 0);
                }
            }
        }
    }

    // ---- projection epilogue: requantise, skip connection, store ------------------------------
    const int lo_p = in_vgpr(a.lo_p), hi_p = in_vgpr(a.hi_p);
    const int m128 = in_vgpr(-128), p127 = in_vgpr(127);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, a.N * a.Ho * Wo * cout, kBufFlags);
#pragma unroll
    for (int q = 0; q < TPW; ++q) {
        const int p = (wave + 4 * q) * 16 + j;
        const bool pvalid = p < npix2;
        const int oy = p / Wo, ox = p - oy * Wo;
        const int opix = (img * a.Ho + ro0 + oy) * Wo + ox;  // output pixel index
#pragma unroll
        for (int t = 0; t < COT; ++t) {
            const int c = 16 * t + 4 * g;
            if (c < cout) {
                int v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = requant_sel(a.np != nullptr, acc[q][t][r], pp[c + r], lo_p, hi_p);
                if (a.add_res) {
                    // stride 1 and cin == cout: the block input at the same pixel and channels
                    const uint32_t res = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(
                        rx, pvalid ? opix * cin + c : kOobOffset, 0, 0);
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = med3_i32(v[r] + sbyte(res, r), m128, p127);
                }
                __builtin_amdgcn_raw_buffer_store_b32((int)pack4_low_bytes(v[0], v[1], v[2], v[3]), ry,
                                                      pvalid ? opix * cout + c : kOobOffset, 0, 0);
            }
        }
    }
}

using BlockFn = void (*)(const BlockArgs);

inline size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }
inline int align16(int v) { return (v + 15) & ~15; }

// Plans the fused kernel; returns false if the shape does not fit it or (unless `forced`) if the
// three launches are expected to be faster.
static bool plan_fused(BlockArgs &a, BlockFn &fn, size_t &lds, int &grid, bool forced)
{
    const int cin = a.cin, chid = a.chid, cout = a.cout, s = a.stride;
    if (cin % 8 != 0 || chid % 4 != 0 || cout % 4 != 0 || cout > 160) return false;
    if ((long long)a.N * a.H * a.W * (cin > cout ? cin : cout) >= (long long)kOobOffset) return false;
    if (a.W > 1024) return false;
    // projection tiles per pixel tile, and pixel tiles per wavefront so that the projection
    // accumulators stay within 64 registers
    const int cot = cout <= 32 ? 2 : cout <= 64 ? 4 : cout <= 96 ? 6 : 10;
    const int tpw = cot == 2 ? 4 : cot == 4 ? 4 : cot == 6 ? 2 : 1;
    const int kse = (cin + 63) / 64;
    const int nch = (chid + kCH - 1) / kCH;  // every chunk's weights are resident
    // Measured in GPU time (calls replayed from a HIP graph; MobileNetV2 blocks, batch 8 to 128):
    // the fused launch beats the three launches through the workspace on mid-sized hidden tensors
    // (28x28x192 at batch 128: 27 us against 42; 112x112x96 at batch 8: 21 against 24).  Small
    // ones are done in three short kernels of 5 us each before the fused kernel, which has two
    // workgroups per CU and a serial chunk loop, has finished (28x28x192 at batch 8: 18 against
    // 16), although a host that pays 10 us per call sees the opposite; on large ones the unfused
    // kernels stream at 4-5 TB/s and win (112x112x96 at batch 128: 166 against 87).  With more
    // than 3 chunks the resident weights leave no room for a band, and streaming them through two
    // LDS slots was measured too: a chunk then costs the latency of its weight fetch, 5-6 us, and
    // the kernel loses everywhere.
    if (nch > 3) return false;
    const long long hidden = (long long)a.N * a.H * a.W * chid;
    if (!forced && (hidden < (4LL << 20) || hidden > (32LL << 20))) return false;
    // the band: at most tpw projection pixel tiles per wavefront, LDS <= 72 KB (two workgroups per CU)
    // Band height by a cost estimate: rounds of workgroups over the chip (two per CU) times the
    // rows a workgroup expands and filters plus a fixed part (weights, barriers) worth about 4 rows.
    int best = 0;
    long long best_cost = 0;
    for (int R = 1; R <= a.Ho; ++R) {
        if (R * a.Wo > 64 * tpw) break;
        const int RI = (R - 1) * s + 3;
        const long long bytes = (long long)align16(RI * a.W * align16(cin) + 64) + (long long)RI * (a.W + 2) * kCH +
                                (long long)nch * (4 * kse * 1024 + cot * 1024 + 2 * kCH * 16 + 9 * kCH) +
                                16 * cot * 16 + 64;
        if (bytes > 72 * 1024) break;
        const int bands = (a.Ho + R - 1) / R;
        const long long rounds = ((long long)a.N * bands + 511) / 512;
        const long long cost = rounds * ((long long)(4 + RI) * a.W + (long long)R * a.Wo);
        if (best == 0 || cost <= best_cost) {
            best = R;
            best_cost = cost;
        }
    }
    if (best == 0) return false;
    const int R = best;
    a.R = R;
    a.RI = (R - 1) * s + 3;
    a.bands = (a.Ho + R - 1) / R;
    int off = align16(a.RI * a.W * align16(cin) + 64);
    a.off_t1 = off; off += align16(a.RI * (a.W + 2) * kCH);
    a.off_t2 = 0;
    a.off_fe = off; off += nch * 4 * kse * 1024;
    a.off_fp = off; off += nch * cot * 1024;
    a.off_pe = off; off += nch * kCH * 16;
    a.off_pd = off; off += nch * kCH * 16;
    a.off_pp = off; off += 16 * cot * 16;
    a.off_wd = off; off += align16(nch * 9 * kCH);
    lds = (size_t)off;
    const bool prelu = a.ne != nullptr || a.nd != nullptr;
    fn = cot == 2   ? (prelu ? &block_fused_kernel<2, 4, true> : &block_fused_kernel<2, 4, false>)
         : cot == 4 ? (prelu ? &block_fused_kernel<4, 4, true> : &block_fused_kernel<4, 4, false>)
         : cot == 6 ? (prelu ? &block_fused_kernel<6, 2, true> : &block_fused_kernel<6, 2, false>)
                    : (prelu ? &block_fused_kernel<10, 1, true> : &block_fused_kernel<10, 1, false>);
    const long long g = (long long)a.N * a.bands;
    if (g > (1LL << 30)) return false;
    grid = (int)g;
    return true;
}

}  // namespace prom

// Whether PROM_BLOCK_AUTO takes the two-launch form (expand; depthwise + projection fused) instead
// of three launches: at present never.  Measured (GPU time of depthwise + projection as two kernels
// against the one fused kernel): a workgroup of the fused kernel walks over the hidden channels in
// chunks of 64 at 1.3 to 1.8 us per chunk (instruction latency of one wavefront per SIMD, not
// memory) plus 8 us of staging and epilogue.  It is level with the two kernels at 14x14x384 (18 to
// 22 against 18 to 19 us), loses from 576 hidden channels on (27 to 37 against 19 to 22) and on large
// maps (56x56x144 at batch 128: 106 against 44), and where it wins under eager launches (28x28x192 at
// batch 8: 11.8 against 18.4; at batch 128: 19.8 against 23.7) the 17-block chain replayed from a HIP
// graph is slower with it (316 against 291 us at batch 8), because two short kernels cost less there
// than the serial chunk loop.  The form stays available through PROM_BLOCK_DWPROJ and
// prom_dw_pw_conv: it moves one intermediate tensor less through HBM.
// Whether PROM_BLOCK_AUTO takes the plane-resident kernel where it applies.  Measured (GPU time per
// call, MobileNetV2 blocks): with at least 12 planes of hidden channels on maps up to 28x28 the one
// kernel beats the three launches and the chunk-interleaved fused kernel (batch 128: 28x28x192
// 26 against 27 us fused, stride 2 18 against 28; 14x14x384 15 against 29; 14x14x576 21 against 34;
// 7x7x960 20 to 25 against 29).  On larger maps the band's halo rows and the vector ALU's
// requantisation of the expanded tensor cost more than the three streaming kernels (56x56x144: 89
// against 66 us; 112x112x96: 109 against 88).
static bool planes_is_faster(int n, int h, int w, int cin, int chid, int cout, int stride)
{
    (void)cin; (void)cout; (void)stride;
    if (chid >= 192 && (long long)h * w <= 28 * 28) return true;
    // small problems are bound by launches, not by work: one kernel instead of three (the 17-block
    // chain at batch 8 replayed from a HIP graph: 201 us with this kernel throughout, 230 with it on
    // the deep blocks only, 281 with three launches per block)
    return (long long)n * h * w * chid <= (48LL << 20);
}

static bool dwproj_is_faster(int n, int h, int w, int chid, int cout, int stride)
{
    (void)n; (void)h; (void)w; (void)chid; (void)cout; (void)stride;
    return false;
}

extern "C" size_t prom_block_workspace_size(int n, int h, int w, int cin, int chid, int cout, int stride)
{
    if (n <= 0 || h <= 0 || w <= 0 || cin <= 0 || chid <= 0 || cout <= 0 || (stride != 1 && stride != 2))
        return 0;
    const size_t ho = (size_t)(h - 1) / stride + 1, wo = (size_t)(w - 1) / stride + 1;
    return prom::round256((size_t)n * h * w * chid) + prom::round256((size_t)n * ho * wo * chid);
}

static int fused_query(int n, int h, int w, int cin, int chid, int cout, int stride, bool forced)
{
    using namespace prom;
    if (n <= 0 || h <= 0 || w <= 0 || cin <= 0 || chid <= 0 || cout <= 0 || (stride != 1 && stride != 2))
        return PROM_EINVAL;
    BlockArgs a = {};
    a.N = n; a.H = h; a.W = w; a.Ho = (h - 1) / stride + 1; a.Wo = (w - 1) / stride + 1;
    a.cin = cin; a.chid = chid; a.cout = cout; a.stride = stride;
    BlockFn fn = nullptr;
    size_t lds = 0;
    int grid = 0;
    return plan_fused(a, fn, lds, grid, forced) ? 1 : 0;
}

extern "C" int prom_block_is_fused(int n, int h, int w, int cin, int chid, int cout, int stride)
{
    const int planes = prom_block_planes_applies(n, h, w, cin, chid, cout, stride);
    if (planes < 0) return planes;
    if (planes == 1 && planes_is_faster(n, h, w, cin, chid, cout, stride)) return 1;
    return fused_query(n, h, w, cin, chid, cout, stride, false);
}

extern "C" int prom_block_can_fuse(int n, int h, int w, int cin, int chid, int cout, int stride)
{
    return fused_query(n, h, w, cin, chid, cout, stride, true);
}

extern "C" int prom_block_planes_applies(int n, int h, int w, int cin, int chid, int cout, int stride)
{
    using namespace prom;
    if (n <= 0 || h <= 0 || w <= 0 || cin <= 0 || chid <= 0 || cout <= 0 || (stride != 1 && stride != 2))
        return PROM_EINVAL;
    PlanesArgs a = {};
    a.N = n; a.H = h; a.W = w; a.Ho = (h - 1) / stride + 1; a.Wo = (w - 1) / stride + 1;
    a.cin = cin; a.chid = chid; a.cout = cout; a.stride = stride;
    size_t lds = 0;
    int grid = 0, kse = 0;
    return plan_planes(a, lds, grid, kse) ? 1 : 0;
}

extern "C" int prom_block(const int8_t *x, int n, int h, int w, int cin, int chid, int cout, int stride,
                          const void *w_expand_packed, const prom_requant_t *rq_expand,
                          const int8_t *w_dw, const prom_requant_t *rq_dw,
                          const void *w_project_packed, const prom_requant_t *rq_project,
                          int add_residual, void *workspace, size_t workspace_bytes, int8_t *y,
                          void *stream)
{
    return prom_block_ex(x, n, h, w, cin, chid, cout, stride, w_expand_packed, rq_expand, w_dw, rq_dw,
                         w_project_packed, rq_project, add_residual, workspace, workspace_bytes, y,
                         PROM_BLOCK_AUTO, stream);
}

extern "C" int prom_block_ex(const int8_t *x, int n, int h, int w, int cin, int chid, int cout, int stride,
                             const void *w_expand_packed, const prom_requant_t *rq_expand,
                             const int8_t *w_dw, const prom_requant_t *rq_dw,
                             const void *w_project_packed, const prom_requant_t *rq_project,
                             int add_residual, void *workspace, size_t workspace_bytes, int8_t *y,
                             int path, void *stream)
{
    using namespace prom;
    if (path != PROM_BLOCK_AUTO && path != PROM_BLOCK_FUSED && path != PROM_BLOCK_UNFUSED &&
        path != PROM_BLOCK_DWPROJ && path != PROM_BLOCK_PLANES)
        return PROM_EINVAL;
    if (!x || !y || !w_expand_packed || !w_dw || !w_project_packed || !rq_expand || !rq_dw || !rq_project)
        return PROM_EINVAL;
    if (n <= 0 || h <= 0 || w <= 0 || cin <= 0 || chid <= 0 || cout <= 0 || (stride != 1 && stride != 2))
        return PROM_EINVAL;
    if (add_residual && !(stride == 1 && cin == cout)) return PROM_EINVAL;
    const size_t need = prom_block_workspace_size(n, h, w, cin, chid, cout, stride);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255) != 0) return PROM_EWORKSPACE;
    const int ho = (h - 1) / stride + 1, wo = (w - 1) / stride + 1;
    int8_t *t1 = static_cast<int8_t *>(workspace);
    int8_t *t2 = t1 + round256((size_t)n * h * w * chid);
    {
        const uintptr_t ya = (uintptr_t)y, wa = (uintptr_t)workspace, xa = (uintptr_t)x;
        const size_t yb = (size_t)n * ho * wo * cout, xb = (size_t)n * h * w * cin;
        if (ya < wa + need && wa < ya + yb) return PROM_EALIAS;
        if (ya < xa + xb && xa < ya + yb) return PROM_EALIAS;
    }
    const prom_requant_t *rqs[3] = {rq_expand, rq_dw, rq_project};
    for (const prom_requant_t *rq : rqs) {
        if (!rq->bias || !rq->mult || !rq->shift) return PROM_EINVAL;
        if (rq->act_min < -128 || rq->act_max > 127 || rq->act_min > rq->act_max) return PROM_EINVAL;
    }
    if (cin > 4096 || chid > 4096) return PROM_EUNSUPPORTED;

    const bool aligned = ((((uintptr_t)x | (uintptr_t)y | (uintptr_t)w_dw) & 7) == 0) &&
                         ((((uintptr_t)w_expand_packed | (uintptr_t)w_project_packed) & 3) == 0);
    BlockArgs a;
    a.x = x; a.y = y;
    a.we = static_cast<const uint32_t *>(w_expand_packed);
    a.wd = w_dw;
    a.wp = static_cast<const uint32_t *>(w_project_packed);
    a.be = rq_expand->bias; a.me = rq_expand->mult; a.se = rq_expand->shift;
    a.bd = rq_dw->bias; a.md = rq_dw->mult; a.sd = rq_dw->shift;
    a.bp = rq_project->bias; a.mp = rq_project->mult; a.sp = rq_project->shift;
    a.ne = rq_expand->mult_neg; a.nd = rq_dw->mult_neg; a.np = rq_project->mult_neg;
    a.N = n; a.H = h; a.W = w; a.Ho = ho; a.Wo = wo;
    a.cin = cin; a.chid = chid; a.cout = cout; a.stride = stride;
    a.add_res = add_residual;
    a.lo_e = rq_expand->act_min; a.hi_e = rq_expand->act_max;
    a.lo_d = rq_dw->act_min; a.hi_d = rq_dw->act_max;
    a.lo_p = rq_project->act_min; a.hi_p = rq_project->act_max;
    if (path == PROM_BLOCK_PLANES || path == PROM_BLOCK_AUTO) {
        // one kernel, the expanded band resident in LDS as 16-channel planes
        PlanesArgs pa = {};
        pa.x = x; pa.y = y;
        pa.we = a.we; pa.wd = a.wd; pa.wp = a.wp;
        pa.be = a.be; pa.me = a.me; pa.se = a.se;
        pa.bd = a.bd; pa.md = a.md; pa.sd = a.sd;
        pa.bp = a.bp; pa.mp = a.mp; pa.sp = a.sp;
        pa.ne = a.ne; pa.nd = a.nd; pa.np = a.np;
        pa.N = n; pa.H = h; pa.W = w; pa.Ho = ho; pa.Wo = wo;
        pa.cin = cin; pa.chid = chid; pa.cout = cout; pa.stride = stride;
        pa.add_res = add_residual;
        pa.lo_e = a.lo_e; pa.hi_e = a.hi_e; pa.lo_d = a.lo_d; pa.hi_d = a.hi_d; pa.lo_p = a.lo_p; pa.hi_p = a.hi_p;
        size_t plds = 0;
        int pgrid = 0, kse = 0;
        // (the per-channel arrays of the first two layers are read four channels at a time)
        uintptr_t par_bits = (uintptr_t)pa.be | (uintptr_t)pa.me | (uintptr_t)pa.se | (uintptr_t)pa.bd |
                             (uintptr_t)pa.md | (uintptr_t)pa.sd | (uintptr_t)pa.ne | (uintptr_t)pa.nd;
        const bool ok = aligned && (par_bits & 15) == 0 && plan_planes(pa, plds, pgrid, kse) &&
                        (path == PROM_BLOCK_PLANES || planes_is_faster(n, h, w, cin, chid, cout, stride));
        if (path == PROM_BLOCK_PLANES && !ok) return PROM_EUNSUPPORTED;
        if (ok) return launch_planes(pa, plds, pgrid, kse, stream);
    }
    BlockFn fn = nullptr;
    size_t lds = 0;
    int grid = 0;
    const bool fuse = path != PROM_BLOCK_UNFUSED && path != PROM_BLOCK_DWPROJ && aligned &&
                      plan_fused(a, fn, lds, grid, path == PROM_BLOCK_FUSED);
    if (path == PROM_BLOCK_FUSED && !fuse) return PROM_EUNSUPPORTED;
    if (fuse) {
        static std::mutex mu;
        static std::vector<BlockFn> attr_done;
        {
            std::lock_guard<std::mutex> lock(mu);
            bool done = false;
            for (BlockFn f : attr_done) done |= f == fn;
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
        BlockArgs args = a;
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

    // the multi-launch forms: refuse now what one of the later layers would refuse
    {
        int rc0 = pw_shape_check(n, h, w, cin, chid);
        if (rc0 == PROM_OK) rc0 = dw_shape_check(n, h, w, chid, stride);
        if (rc0 == PROM_OK) rc0 = pw_shape_check(n, ho, wo, chid, cout);
        if (rc0 != PROM_OK) return rc0;
    }
    // two launches: expand, then depthwise and projection in one kernel
    const bool can_dwproj = prom_dw_pw_can_fuse(n, h, w, chid, cout, stride) == 1 &&
                            ((((uintptr_t)x | (uintptr_t)y | (uintptr_t)w_project_packed | (uintptr_t)w_dw) & 3) == 0);
    if (path == PROM_BLOCK_DWPROJ && !can_dwproj) return PROM_EUNSUPPORTED;
    if (path == PROM_BLOCK_DWPROJ || (path == PROM_BLOCK_AUTO && can_dwproj && dwproj_is_faster(n, h, w, chid, cout, stride))) {
        const int rc2 = prom_pw_conv(x, n, h, w, cin, w_expand_packed, chid, rq_expand, nullptr, t1, stream);
        if (rc2 != PROM_OK) return rc2;
        return prom_dw_pw_conv(t1, n, h, w, chid, w_dw, stride, rq_dw, w_project_packed, cout, rq_project,
                               add_residual ? x : nullptr, y, stream);
    }
    // three launches through the workspace
    int rc = prom_pw_conv(x, n, h, w, cin, w_expand_packed, chid, rq_expand, nullptr, t1, stream);
    if (rc != PROM_OK) return rc;
    rc = prom_dw_conv(t1, n, h, w, chid, w_dw, stride, rq_dw, t2, stream);
    if (rc != PROM_OK) return rc;
    return prom_pw_conv(t2, n, ho, wo, chid, w_project_packed, cout, rq_project,
                        add_residual ? x : nullptr, y, stream);
}

// ---- the block for callers that cannot allocate -------------------------------------------------
// The three-launch form needs the two intermediates somewhere.  prom_block takes them from the
// caller's workspace; prom_block_noalloc keeps them in a fixed array in the library's own device
// image, so that a caller under graph capture or in a loop that must not call hipMalloc needs no
// workspace of its own.  The array exists once per GPU the library runs on, from the moment the
// code object is loaded there until the process ends.
namespace prom {

constexpr size_t kNoAllocScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];

constexpr int kMaxDevices = 64;

// Device address of `scratch` on the current device (the name `scratch` in host code is only a
// handle for the runtime, not an address a kernel could use).  Looked up once per device.
static int noalloc_scratch(void **out)
{
    static std::mutex mu;
    static void *ptr[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        last_hip_error() = e != hipSuccess ? e : hipErrorInvalidDevice;
        (void)hipGetLastError();
        return PROM_EHIP;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            last_hip_error() = e != hipSuccess ? e : hipErrorInvalidSymbol;
            (void)hipGetLastError();
            return PROM_EHIP;
        }
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return PROM_OK;
}

}  // namespace prom

extern "C" size_t prom_block_noalloc_max_workspace(void) { return prom::kNoAllocScratchBytes; }

extern "C" int prom_block_noalloc(const int8_t *x, int n, int h, int w, int cin, int chid, int cout, int stride,
                                  const void *w_expand_packed, const prom_requant_t *rq_expand,
                                  const int8_t *w_dw, const prom_requant_t *rq_dw,
                                  const void *w_project_packed, const prom_requant_t *rq_project,
                                  int add_residual, int8_t *y, void *stream)
{
    if (n <= 0 || h <= 0 || w <= 0 || cin <= 0 || chid <= 0 || cout <= 0 || (stride != 1 && stride != 2))
        return PROM_EINVAL;
    const size_t need = prom_block_workspace_size(n, h, w, cin, chid, cout, stride);
    if (need > prom::kNoAllocScratchBytes) return PROM_ESCRATCH;
    void *ws = nullptr;
    const int rc = prom::noalloc_scratch(&ws);
    if (rc != PROM_OK) return rc;
    return prom_block_ex(x, n, h, w, cin, chid, cout, stride, w_expand_packed, rq_expand, w_dw, rq_dw,
                         w_project_packed, rq_project, add_residual, ws, prom::kNoAllocScratchBytes, y,
                         PROM_BLOCK_AUTO, stream);
}
