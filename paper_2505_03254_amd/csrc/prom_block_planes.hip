// Inverted-residual block (paper Section 2 and Figure 4: ternary pointwise expansion -> int8
// depthwise 3x3 -> ternary pointwise projection, + skip) as ONE kernel with the expanded tensor
// of a band of rows resident in LDS as 16-channel planes.
//
// The chunk-interleaved fused kernel of prom_block.hip keeps every weight of the block decoded in
// LDS and walks the hidden channels in barrier-separated chunks; beyond 192 hidden channels its
// weights no longer fit.  This kernel turns the ownership round so that NO weight matrix passes
// through LDS and the workgroup meets at two or three barriers in all:
//   phase 0  the band's input rows, the per-channel parameters of the expansion and the depthwise
//            layer and the depthwise weights go to LDS; the borders of the planes are zeroed;
//   phase 1  expansion.  A wavefront owns 16-channel planes of the hidden tensor (plane p, p + 8,
//            ...): it fetches the 16 x cin packed ternary codes of its plane straight from global
//            memory into registers (one dword per lane and k step, the next plane's one plane
//            ahead), decodes them once, and runs every 16-pixel tile of the band through
//            v_mfma_i32_16x16x64_i8 with the pixels as the B operand (a 16-byte LDS read), the
//            requantised outputs go to the plane [row][col + 1][16 channels] with a zero border;
//   phase 2  depthwise 3x3 of the same planes on the matrix cores (k = 4 taps x 16 channels; the A
//            operand holds the lane's one weight per tap group), by the same owner, so that a
//            plane needs no barrier between its expansion and its filter; the requantised outputs
//            go to the compact plane [pixel][16 channels];
//   phase 3  projection.  A wavefront owns an output-channel tile (and a group of up to 4 pixel
//            tiles), fetches and decodes that tile's rows of packed codes itself and reads the B
//            operands (pixel, 16 hidden channels) from the planes; epilogue, skip (the block input
//            is still in LDS), store.
// With at least as many planes as wavefronts a plane's depthwise output overwrites the slot of a
// plane its owner has already consumed (plane p -> slot p, its expansion sits in slot p + 8), so
// the hidden tensor takes (planes + 8) slots in all; with fewer planes the pixel tiles of a plane
// are spread over wavefronts, there is a barrier between phases 1 and 2 and the depthwise output
// has a region of its own.
#include "prom_pw_stream.h"
#include "prom_launch.h"
#include "prom_block_planes.h"

#include <cstdlib>
#include <mutex>
#include <vector>

namespace prom {

// Wavefronts per workgroup: 8, 12 or 16 (the planner takes the count that divides the planes best).

#ifdef PROM_TIMELINE
// Developer build: workgroups 0 .. 255 record the 100 MHz clock at the phase boundaries.
__device__ unsigned long long g_pl_stamps[256 * 8];
#define PL_STAMP(i) do { if (threadIdx.x == 0 && blockIdx.x < 256) g_pl_stamps[blockIdx.x * 8 + (i)] = wall_clock64(); } while (0)
#else
#define PL_STAMP(i) do { } while (0)
#endif

// Epilogue forms: 0 = every shift of the lane's channels >= 1 (pr.w holds shift - 1), 1 = any
// shift, 2 = PReLU.
template <int MODE> struct PlMode { static constexpr int value = MODE; };

// Bias, multiplier(s) and shift of a lane's four channels (16*plane + 4*g + 0..3) as loaded.
struct PlRawPar { v4i b, m, n, s; };

// KSE: 64-wide k steps of the expansion (cin <= 64*KSE).  PRELU: the expansion and depthwise
// epilogues take the PReLU form (a layer of the two without negative-side multipliers runs it with
// mult_neg = mult, which is the plain form).
template <int KSE, bool PRELU, int NW>
__global__ __launch_bounds__(64 * NW, 1) void block_planes_kernel(const PlanesArgs a)
{
    constexpr int kPlWaves = NW, kPlThreads = 64 * NW;
    extern __shared__ __align__(16) unsigned char lds[];
    PL_STAMP(0);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, g = lane >> 4;
    const int W = a.W, Wo = a.Wo, W2 = W + 2, s = a.stride;
    const int cin = a.cin, chid = a.chid, cout = a.cout, cinp = a.cinp;
    const int NP = a.NP;

    const int img = blockIdx.x / a.bands;
    const int band = blockIdx.x - img * a.bands;
    const int ro0 = band * a.R;                                // first output row of the band
    const int rows_out = min(a.R, a.Ho - ro0);
    const int ri0 = ro0 * s - 1;                               // first input row under a tap (may be -1)
    const int ri_last = ri0 + (rows_out - 1) * s + 2;          // last one (may be H)
    const int rlo = max(ri0, 0), rhi = min(ri_last, a.H - 1);  // the rows that exist
    const int rv0 = rlo - ri0;                                 // plane row of the first existing input row
    const int nvr = rhi - rlo + 1;
    const int rib = ri_last - ri0 + 1;                         // plane rows in use
    const int np1 = nvr * W;                                   // pixels to expand
    const int np2 = rows_out * Wo;                             // output pixels of the band
    const int nt1 = (np1 + 15) >> 4, nt2 = (np2 + 15) >> 4;

    int8_t *xs = reinterpret_cast<int8_t *>(lds);
    uint16_t *o1 = reinterpret_cast<uint16_t *>(lds + a.off_o1);  // pixel of phase 1 -> 16-byte cell of its plane
    uint16_t *o2 = reinterpret_cast<uint16_t *>(lds + a.off_o2);  // output pixel -> cell of its tap (0, 0)
    v4i *pp = reinterpret_cast<v4i *>(lds + a.off_pp);            // [16*COT] projection parameters
    int8_t *wdl = reinterpret_cast<int8_t *>(lds + a.off_wd);     // [9][chid] depthwise weights
    uint32_t *w3l = reinterpret_cast<uint32_t *>(lds + a.off_w3); // [16*COT][S3] packed projection codes
    unsigned char *t1 = lds + a.off_t1;
    unsigned char *t2 = lds + a.off_t2;
    const int slot1 = a.slot1, slot2 = a.slot2;

    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a.x), 0, a.N * a.H * W * cin, kBufFlags);

    const int KWe = a.KWe, KWp = a.KWp, S3 = a.S3;
    const int G1 = a.G1, G2 = a.G2, G3 = a.G3;
    const int units1 = NP * G1, units2 = NP * G2;
    const bool prelu_p = a.np != nullptr;

    // ---- phase 0: every global load of the prologue leaves first, the index tables and the zero
    // cells are made while they fly, then the loaded values go to LDS -------------------------------
    // the band's existing input rows: one contiguous run of the NHWC tensor, 8-byte pieces
    constexpr int NX = 4;
    const int xtotal = np1 * cin;  // multiple of 8
    const int xbase = ((img * a.H + rlo) * W) * cin;
    v2i xv[NX];
#pragma unroll
    for (int q = 0; q < NX; ++q) {
        const int o = (tid + q * kPlThreads) * 8;
        xv[q] = __builtin_amdgcn_raw_buffer_load_b64(rx, o < xtotal ? xbase + o : kOobOffset, 0, 0);
    }
    // the packed codes and the parameters of this wavefront's first plane
    auto load_w1 = [&](int u, uint32_t(&w)[KSE]) __attribute__((always_inline)) {
        const int pl = G1 == 1 ? u : u / G1;
        const uint32_t *row = a.we + (long long)(16 * pl + j) * KWe;
#pragma unroll
        for (int ks = 0; ks < KSE; ++ks) {
            const int kw = 4 * ks + g;
            const bool ok = kw < KWe;
            const uint32_t v = row[ok ? kw : 0];
            w[ks] = ok ? v : 0u;
        }
    };
    auto load_par = [&](const int32_t *B, const int32_t *M, const int32_t *Nn, const int32_t *S, int pl,
                        PlRawPar &r) __attribute__((always_inline)) {
        const int c = 16 * pl + 4 * g;
        r.b = *reinterpret_cast<const v4i *>(B + c);
        r.m = *reinterpret_cast<const v4i *>(M + c);
        r.s = *reinterpret_cast<const v4i *>(S + c);
        if (PRELU && Nn) r.n = *reinterpret_cast<const v4i *>(Nn + c);
        else r.n = r.m;
    };
    auto make_par = [&](const PlRawPar &r, v4i(&par)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) par[i] = requant_params(r.b[i], r.m[i], r.n[i], r.s[i], PRELU);
    };
    uint32_t w1n[KSE];
    PlRawPar rawe, rawd;
    {
        const int u = min(wave, units1 - 1);
        load_w1(u, w1n);
        load_par(a.be, a.me, a.ne, a.se, G1 == 1 ? u : u / G1, rawe);
        const int u2 = min(wave, units2 - 1);
        load_par(a.bd, a.md, a.nd, a.sd, G2 == 1 ? u2 : u2 / G2, rawd);
    }
    // the projection's parameters: one channel per thread
    int pbp, pmp, pnp, psp;
    {
        const int c = min(tid, cout - 1);
        pbp = a.bp[c]; pmp = a.mp[c]; psp = a.sp[c];
        pnp = prelu_p ? a.np[c] : 0;
    }
    // depthwise weights, dword pieces
    constexpr int NWD = 5;
    const uint32_t *wd4 = reinterpret_cast<const uint32_t *>(a.wd);
    const int nwd = (9 * chid) >> 2;
    uint32_t wdv[NWD];
#pragma unroll
    for (int q = 0; q < NWD; ++q) wdv[q] = wd4[min(tid + q * kPlThreads, nwd - 1)];

    {
        // (pixels beyond the band land in a spare cell behind the plane's rows)
        for (int p = tid; p < nt1 * 16; p += kPlThreads) {
            const int row = p / W, col = p - row * W;
            o1[p] = (uint16_t)(p < np1 ? (rv0 + row) * W2 + col + 1 : a.RI * W2);
        }
        for (int p = tid; p < nt2 * 16; p += kPlThreads) {
            const int pc = min(p, np2 - 1);
            const int oy = pc / Wo, ox = pc - oy * Wo;
            o2[p] = (uint16_t)((oy * s) * W2 + ox * s);
        }
        // zero cells of the expansion planes: the two border columns of every row in use and the
        // rows outside the image
        const int ninv = rib - nvr;
        const int per = 2 * rib + ninv * W;
        const v4i zero4 = {0, 0, 0, 0};
        for (int e = tid; e < per; e += kPlThreads) {
            int cell;
            if (e < 2 * rib) {
                cell = (e >> 1) * W2 + ((e & 1) ? W + 1 : 0);
            } else {
                const int q = e - 2 * rib;
                const int ir = q / W, col = q - ir * W;
                // invalid rows: those before rv0, then those from rv0 + nvr on
                const int row = ir < rv0 ? ir : ir + nvr;
                cell = row * W2 + col + 1;
            }
            unsigned char *dst = t1 + cell * 16;
            for (int pl = 0; pl < NP; ++pl) *reinterpret_cast<v4i *>(dst + pl * slot1) = zero4;
        }
    }
    {
        const int pieces = cin >> 3;
#pragma unroll
        for (int q = 0; q < NX; ++q) {
            const int pc = tid + q * kPlThreads;
            if (pc * 8 < xtotal) {
                const int px = pc / pieces;
                *reinterpret_cast<v2i *>(xs + px * cinp + 8 * (pc - px * pieces)) = xv[q];
            }
        }
        for (int o = (tid + NX * kPlThreads) * 8; o < xtotal; o += kPlThreads * 8) {
            const v2i v = __builtin_amdgcn_raw_buffer_load_b64(rx, xbase + o, 0, 0);
            const int pc = o >> 3;
            const int px = pc / pieces;
            *reinterpret_cast<v2i *>(xs + px * cinp + 8 * (pc - px * pieces)) = v;
        }
        if (tid < 16 * a.COT) pp[tid] = tid < cout ? requant_params(pbp, pmp, pnp, psp, prelu_p) : v4i{0, 0, 0, 1};
#pragma unroll
        for (int q = 0; q < NWD; ++q) {
            const int i = tid + q * kPlThreads;
            if (i < nwd) reinterpret_cast<uint32_t *>(wdl)[i] = wdv[q];
        }
        for (int i = tid + NWD * kPlThreads; i < nwd; i += kPlThreads) reinterpret_cast<uint32_t *>(wdl)[i] = wd4[i];
    }
    __syncthreads();
    PL_STAMP(1);

    const int lo_e = in_vgpr(a.lo_e), hi_e = in_vgpr(a.hi_e);
    const int lo_d = in_vgpr(a.lo_d), hi_d = in_vgpr(a.hi_d);
    const v4i zero4 = {0, 0, 0, 0};

    // ---- phase 1: expansion of the owned planes -----------------------------------------------------
    {
        const int tpg = G1 == 1 ? nt1 : (nt1 + G1 - 1) / G1;
        for (int u = wave; u < units1; u += kPlWaves) {
            v4i A[KSE];
#pragma unroll
            for (int ks = 0; ks < KSE; ++ks) A[ks] = decode_word(w1n[ks]);
            v4i par[4];
            make_par(rawe, par);
            const int pl = G1 == 1 ? u : u / G1;
            const int grp = u - pl * G1;
            {   // the next unit's codes and parameters fly during this one
                const int un = min(u + kPlWaves, units1 - 1);
                load_w1(un, w1n);
                load_par(a.be, a.me, a.ne, a.se, G1 == 1 ? un : un / G1, rawe);
            }
            unsigned char *t1p = t1 + pl * slot1 + 4 * g;
            const int pt0 = grp * tpg, pt1 = min((grp + 1) * tpg, nt1);
            // NTL pixel tiles at once: independent chains for the matrix cores and the epilogue
            auto tiles = [&](auto mode, auto ntl, int pt) __attribute__((always_inline)) {
                constexpr int MODE = decltype(mode)::value;
                constexpr int NTL = decltype(ntl)::value;
                v4i d[NTL];
                int cell[NTL], p[NTL];
#pragma unroll
                for (int i = 0; i < NTL; ++i) {
                    p[i] = (pt + i) * 16 + j;
                    const int8_t *xp = xs + __umul24(p[i], cinp) + 16 * g;
                    cell[i] = o1[p[i]];
                    d[i] = zero4;
#pragma unroll
                    for (int ks = 0; ks < KSE; ++ks)
                        d[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[ks], *reinterpret_cast<const v4i *>(xp + 64 * ks), d[i], 0, 0, 0);
                }
#pragma unroll
                for (int i = 0; i < NTL; ++i) {
                    int v[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = requant_mode<MODE>(d[i][r], par[r], lo_e, hi_e);
                    *reinterpret_cast<uint32_t *>(t1p + cell[i] * 16) = pack4_low_bytes(v[0], v[1], v[2], v[3]);
                }
            };
            auto run = [&](auto mode) __attribute__((always_inline)) {
                int pt = pt0;
                for (; pt + 4 <= pt1; pt += 4) tiles(mode, PlMode<4>{}, pt);
                if (pt + 2 <= pt1) {
                    tiles(mode, PlMode<2>{}, pt);
                    pt += 2;
                }
                if (pt < pt1) tiles(mode, PlMode<1>{}, pt);
            };
            if constexpr (PRELU) {
                run(PlMode<2>{});
            } else {
                const bool shift0 = par[0][3] == 0 || par[1][3] == 0 || par[2][3] == 0 || par[3][3] == 0;
                if (__builtin_amdgcn_ballot_w64(shift0) == 0) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) par[r][3] -= 1;
                    run(PlMode<0>{});
                } else {
                    run(PlMode<1>{});
                }
            }
        }
    }
    PL_STAMP(2);
    if (G1 != 1 || G2 != 1) __syncthreads();

    // The projection's packed codes go to LDS while phase 2 runs: loads now, stores behind the loop.
    // Wide rows (whole 16-byte pieces): the matrix is one flat run of pieces.
    constexpr int NW3 = 10;
    const bool w3wide = (KWp & 3) == 0 && (reinterpret_cast<uintptr_t>(a.wp) & 15) == 0;
    const int kq3 = KWp >> 2;
    const int n3 = w3wide ? cout * kq3 : cout * KWp;  // pieces: 16 bytes or one word
    v4i w3v[NW3];
    if (w3wide) {
#pragma unroll
        for (int q = 0; q < NW3; ++q)
            w3v[q] = *reinterpret_cast<const v4i *>(a.wp + 4 * (long long)min(tid + q * kPlThreads, n3 - 1));
    } else {
#pragma unroll
        for (int q = 0; q < NW3; ++q) w3v[q][0] = (int)a.wp[min(tid + q * kPlThreads, n3 - 1)];
    }

    // ---- phase 2: depthwise 3x3 of the owned planes on the matrix cores ------------------------------
    {
        const int li = lane & 15;
        int toff[3];  // byte offset of the lane's tap in each tap group (tap 8 again where there is none)
#pragma unroll
        for (int q = 0; q < 3; ++q) {
            const int tap = min(4 * q + g, 8);
            toff[q] = ((tap / 3) * W2 + tap % 3) * 16;
        }
        const int tpg = G2 == 1 ? nt2 : (nt2 + G2 - 1) / G2;
        for (int u = wave; u < units2; u += kPlWaves) {
            const int pl = G2 == 1 ? u : u / G2;
            const int grp = u - pl * G2;
            // A operands: for tap group q the weight of channel 16*pl + li under tap 4q + g at byte li
            // of the lane's 16, zero elsewhere
            v4i adw[3];
#pragma unroll
            for (int q = 0; q < 3; ++q) {
                const int tap = 4 * q + g;
                const uint32_t wb = tap < 9 ? (uint32_t)(uint8_t)wdl[tap * chid + 16 * pl + li] : 0u;
                const uint32_t val = wb << (8 * (li & 3));
                adw[q] = v4i{(li >> 2) == 0 ? (int)val : 0, (li >> 2) == 1 ? (int)val : 0,
                             (li >> 2) == 2 ? (int)val : 0, (li >> 2) == 3 ? (int)val : 0};
            }
            v4i par[4];
            make_par(rawd, par);
            {
                const int un = min(u + kPlWaves, units2 - 1);
                load_par(a.bd, a.md, a.nd, a.sd, G2 == 1 ? un : un / G2, rawd);
            }
            const unsigned char *t1p = t1 + pl * slot1;
            unsigned char *t2p = t2 + pl * slot2 + 4 * g;
            const int pt0 = grp * tpg, pt1 = min((grp + 1) * tpg, nt2);
            auto tiles = [&](auto mode, auto ntl, int pt) __attribute__((always_inline)) {
                constexpr int MODE = decltype(mode)::value;
                constexpr int NTL = decltype(ntl)::value;
                v4i d[NTL];
#pragma unroll
                for (int i = 0; i < NTL; ++i) {
                    const unsigned char *src = t1p + o2[(pt + i) * 16 + j] * 16;
                    d[i] = zero4;
#pragma unroll
                    for (int q = 0; q < 3; ++q)
                        d[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(adw[q], *reinterpret_cast<const v4i *>(src + toff[q]), d[i], 0, 0, 0);
                }
                // (the reads of every tile are complete before the first write: with one owner per
                // plane the output may land in a slot this wavefront has consumed, never in its own)
#pragma unroll
                for (int i = 0; i < NTL; ++i) {
                    int v[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = requant_mode<MODE>(d[i][r], par[r], lo_d, hi_d);
                    *reinterpret_cast<uint32_t *>(t2p + ((pt + i) * 16 + j) * 16) = pack4_low_bytes(v[0], v[1], v[2], v[3]);
                }
            };
            auto run = [&](auto mode) __attribute__((always_inline)) {
                int pt = pt0;
                for (; pt + 4 <= pt1; pt += 4) tiles(mode, PlMode<4>{}, pt);
                if (pt + 2 <= pt1) {
                    tiles(mode, PlMode<2>{}, pt);
                    pt += 2;
                }
                if (pt < pt1) tiles(mode, PlMode<1>{}, pt);
            };
            if constexpr (PRELU) {
                run(PlMode<2>{});
            } else {
                const bool shift0 = par[0][3] == 0 || par[1][3] == 0 || par[2][3] == 0 || par[3][3] == 0;
                if (__builtin_amdgcn_ballot_w64(shift0) == 0) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) par[r][3] -= 1;
                    run(PlMode<0>{});
                } else {
                    run(PlMode<1>{});
                }
            }
        }
    }
    // the projection's codes: rows of S3 words in LDS
    if (w3wide) {
#pragma unroll
        for (int q = 0; q < NW3; ++q) {
            const int i = tid + q * kPlThreads;
            if (i < n3) {
                const int row = i / kq3;
                *reinterpret_cast<v4i *>(w3l + row * S3 + 4 * (i - row * kq3)) = w3v[q];
            }
        }
        for (int i = tid + NW3 * kPlThreads; i < n3; i += kPlThreads) {
            const int row = i / kq3;
            *reinterpret_cast<v4i *>(w3l + row * S3 + 4 * (i - row * kq3)) = *reinterpret_cast<const v4i *>(a.wp + 4 * (long long)i);
        }
    } else {
#pragma unroll
        for (int q = 0; q < NW3; ++q) {
            const int i = tid + q * kPlThreads;
            if (i < n3) {
                const int row = i / KWp;
                w3l[row * S3 + (i - row * KWp)] = (uint32_t)w3v[q][0];
            }
        }
        for (int i = tid + NW3 * kPlThreads; i < n3; i += kPlThreads) {
            const int row = i / KWp;
            w3l[row * S3 + (i - row * KWp)] = a.wp[i];
        }
        // words between the row's end and the next multiple of four are read as codes: zero
        for (int r = tid; r < cout; r += kPlThreads)
            for (int w = KWp; w < ((KWp + 3) & ~3); ++w) w3l[r * S3 + w] = 0u;
    }
    PL_STAMP(3);
    __syncthreads();
    PL_STAMP(4);

    // ---- phase 3: projection ---------------------------------------------------------------------------
    // The k dimension is walked in groups of 16 packed words (256 hidden channels): k step 4*gi + e
    // of lane group kg covers plane 16*gi + 4*kg + e, so that a lane's codes of four k steps are one
    // 16-byte LDS read.
    {
        const int lo_p = in_vgpr(a.lo_p), hi_p = in_vgpr(a.hi_p);
        const int m128 = in_vgpr(-128), p127 = in_vgpr(127);
        const __amdgpu_buffer_rsrc_t ry =
            __builtin_amdgcn_make_buffer_rsrc(a.y, 0, a.N * a.Ho * Wo * cout, kBufFlags);
        const int obase = (img * a.Ho + ro0) * Wo;  // first output pixel of the band
        const int TPG3 = a.TPG3;
        const int units3 = a.COT * G3;
        const int R4 = (KWp + 3) & ~3;
        const int ng3 = (KWp + 15) >> 4;
        // TPG pixel tiles of one output-channel tile per unit (tiles beyond the band are computed on
        // whatever the planes hold there and never stored: no branch in the k loop)
        auto unit = [&](auto tpg, int ct, int pt0) __attribute__((always_inline)) {
            constexpr int TPG = decltype(tpg)::value;
            v4i acc[TPG];
#pragma unroll
            for (int i = 0; i < TPG; ++i) acc[i] = zero4;
            const unsigned char *bq = t2 + (pt0 * 16 + j) * 16;
            const uint32_t *wrow = w3l + (16 * ct + j) * S3;
            // One k step ahead: the B operands of the next step and the codes of the next group are
            // on their way while this step's codes are decoded and its MFMAs issue.  Steps past the
            // last plane read the last plane against zero codes (the rows are zero-padded to R4 and
            // groups past R4 take zeros), the reads past the last step go nowhere.
            auto load_b = [&](v4i(&B)[TPG], int plane) __attribute__((always_inline)) {
                const unsigned char *bp = bq + min(plane, NP - 1) * slot2;
#pragma unroll
                for (int i = 0; i < TPG; ++i) B[i] = *reinterpret_cast<const v4i *>(bp + i * 256);
            };
            auto load_w = [&](int wo) __attribute__((always_inline)) {
                v4i wv = *reinterpret_cast<const v4i *>(wrow + min(wo, R4 - 4));
                if (wo >= R4) wv = zero4;
                return wv;
            };
            v4i Bn[TPG];
            load_b(Bn, 4 * g);
            v4i wn = load_w(4 * g);
            for (int gi = 0; gi < ng3; ++gi) {
                const int wo = 16 * gi + 4 * g;
                const v4i wv = wn;
                wn = load_w(wo + 16);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v4i Bc[TPG];
#pragma unroll
                    for (int i = 0; i < TPG; ++i) Bc[i] = Bn[i];
                    load_b(Bn, e < 3 ? wo + e + 1 : wo + 16);
                    const v4i A = decode_word((uint32_t)wv[e]);
#pragma unroll
                    for (int i = 0; i < TPG; ++i)
                        acc[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A, Bc[i], acc[i], 0, 0, 0);
                }
            }
            const int c = 16 * ct + 4 * g;
            const bool cok = c < cout;
            v4i pr[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) pr[r] = pp[c + r];
#pragma unroll
            for (int i = 0; i < TPG; ++i) {
                if (pt0 + i < nt2) {
                    const int p = (pt0 + i) * 16 + j;
                    const bool pvalid = cok && p < np2;
                    int v[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        v[r] = prelu_p ? requant_prelu_i64(acc[i][r], pr[r], lo_p, hi_p)
                                       : requant_i64<true>(acc[i][r], pr[r], lo_p, hi_p);
                    if (a.add_res) {
                        // stride 1 and cin == cout: the block input at the same pixel, still in LDS
                        const uint32_t res = *reinterpret_cast<const uint32_t *>(
                            xs + ((1 - rv0) * W + min(p, np2 - 1)) * cinp + (cok ? c : 0));
#pragma unroll
                        for (int r = 0; r < 4; ++r) v[r] = med3_i32(v[r] + sbyte(res, r), m128, p127);
                    }
                    __builtin_amdgcn_raw_buffer_store_b32((int)pack4_low_bytes(v[0], v[1], v[2], v[3]), ry,
                                                          pvalid ? (obase + p) * cout + c : kOobOffset, 0, 0);
                }
            }
        };
        for (int u = wave; u < units3; u += kPlWaves) {
            const int ct = G3 == 1 ? u : u / G3;
            const int pt0 = (u - ct * G3) * TPG3;
            if (pt0 >= nt2) continue;
            if (TPG3 == 8) unit(PlMode<8>{}, ct, pt0);
            else if (TPG3 == 4) unit(PlMode<4>{}, ct, pt0);
            else if (TPG3 == 2) unit(PlMode<2>{}, ct, pt0);
            else unit(PlMode<1>{}, ct, pt0);
        }
    }
    PL_STAMP(6);
    __builtin_amdgcn_s_waitcnt(0);
    PL_STAMP(7);
}

using PlanesFn = void (*)(const PlanesArgs);

static inline int align16i(int v) { return (v + 15) & ~15; }

// Plans the kernel for the shape in `a` (N, H, W, Ho, Wo, cin, chid, cout, stride set): band height,
// unit split of the three phases, LDS layout.  False if the shape does not fit.
bool plan_planes(PlanesArgs &a, size_t &lds, int &grid, int &kse)
{
    const int cin = a.cin, chid = a.chid, cout = a.cout, s = a.stride;
    if (cin % 8 != 0 || chid % 16 != 0 || cout % 4 != 0 || cin > 192) return false;
    if ((long long)a.N * a.H * a.W * cin >= (long long)kOobOffset) return false;
    if ((long long)a.N * a.Ho * a.Wo * cout >= (long long)kOobOffset) return false;
    if (a.W > 4096) return false;
    kse = (cin + 63) / 64;
    const int NP = chid / 16, COT = (cout + 15) / 16;
    const int KS3 = (chid + 63) / 64;
    const int KWp = chid / 16;
    int cinp = align16i(cin);
    if (((cinp >> 4) & 1) == 0) cinp += 16;  // odd number of 16-byte pieces per pixel: no bank conflicts
    const int W2 = a.W + 2;
    const int kLdsMax = 160 * 1024;
    int only_nw = 0;
#ifdef PROM_TIMELINE
    if (const char *env = getenv("PROM_PLANES_NW")) only_nw = atoi(env);
#endif

    // Candidates: wavefronts per workgroup (more of them keep the vector ALU busier while others
    // wait on LDS and the matrix cores; the planes must divide among them), the padding of the
    // projection's code rows in LDS (against bank conflicts; dropped where LDS is short), the band
    // height.  The estimate counts wavefront instructions: a SIMD issues one every `cpi` cycles.
    struct Pick { int nw, pad, R, G, G3, TPG3; double cost; } best = {0, 0, 0, 0, 0, 0, 0};
    for (int nw : {8, 12, 16}) {
        if (only_nw && nw != only_nw) continue;
        if (cout > 64 * nw) continue;
        const double cpi = nw == 8 ? 4.9 : nw == 12 ? 4.45 : 3.95;  // measured: phases 1 and 2 of 14x14x384
        // few planes: spread the pixel tiles of a plane over wavefronts (about 3 units per wavefront)
        const int G = NP >= nw ? 1 : (3 * nw + NP - 1) / NP;
        for (int pad : {4, 0}) {
            const int s3 = ((KWp + 3) & ~3) + pad;
            for (int R = 1; R <= a.Ho; ++R) {
                const int RI = (R - 1) * s + 3;
                const long long np1 = (long long)RI * a.W, np2 = (long long)R * a.Wo;
                if (np1 > 8192 || (long long)RI * W2 >= 65535) break;
                const int nt1 = (int)((np1 + 15) / 16), nt2 = (int)((np2 + 15) / 16);
                const int plane1 = (RI * W2 + 1) * 16, plane2 = nt2 * 256;
                long long bytes = align16i(nt1 * 16 * cinp + 64 * kse + 64);  // xs
                bytes += align16i(nt1 * 32) + align16i(nt2 * 32);             // o1, o2
                bytes += COT * 256;                                           // pp
                bytes += 16LL * COT * s3 * 4;                                 // w3l
                bytes += align16i(9 * chid);                                  // wdl
                if (G == 1) bytes += (long long)(NP + nw) * (plane1 > plane2 ? plane1 : plane2);
                else bytes += (long long)NP * (plane1 + plane2);
                if (bytes + 2048 > kLdsMax) break;
                // phase 3: 1, 2, 4 or 8 pixel tiles of one output-channel tile per unit
                int g3 = 1, tpg3 = 1;
                double c3 = 0;
                for (int t = 1; t <= 8; t *= 2) {
                    const int gg = (nt2 + t - 1) / t;
                    const long long rounds = ((long long)COT * gg + nw - 1) / nw;
                    const double c = (double)rounds * (KS3 * (20.0 + 3.0 * t) + 40.0 * t + 40.0);
                    if (t == 1 || c < c3) {
                        c3 = c;
                        g3 = gg;
                        tpg3 = t;
                    }
                }
                // phases 1 and 2: the SIMDs share the units' instructions (a wavefront that is done
                // leaves its SIMD to the others, so uneven plane counts cost little); spread planes
                // pay a barrier
                const double per1 = 60.0 + ((nt1 + G - 1) / G) * (38.0 + 3.0 * kse);
                const double per2 = 80.0 + ((nt2 + G - 1) / G) * 42.0;
                const double units = (double)NP * G;
                double work = cpi * units * (per1 + per2) / 4.0 + (nw / 4) * cpi * c3;
                if (G > 1) work *= 1.15;
                const int bands = (a.Ho + R - 1) / R;
                const long long rounds = ((long long)a.N * bands + 255) / 256;
                // fixed part: launch, the prologue's memory round trip, barriers, the drain
                const double cost = (double)rounds * (12000.0 + work);
                if (best.nw == 0 || cost < best.cost) best = {nw, pad, R, G, g3, tpg3, cost};
            }
        }
    }
    if (best.nw == 0) return false;
    const int R = best.R, G = best.G, nw = best.nw;
    a.NW = nw;
    a.R = R;
    a.RI = (R - 1) * s + 3;
    a.bands = (a.Ho + R - 1) / R;
    a.NP = NP;
    a.COT = COT;
    a.KWe = (cin + 15) / 16;
    a.KWp = KWp;
    a.KS3 = KS3;
    a.cinp = cinp;
    a.G1 = a.G2 = G;
    a.G3 = best.G3;
    a.TPG3 = best.TPG3;
    const int np1 = a.RI * a.W, np2 = R * a.Wo;
    const int nt1 = (np1 + 15) / 16, nt2 = (np2 + 15) / 16;
    const int plane1 = (a.RI * W2 + 1) * 16, plane2 = nt2 * 256;
    int off = align16i(nt1 * 16 * cinp + 64 * kse + 64);
    a.off_o1 = off; off += align16i(nt1 * 32);
    a.off_o2 = off; off += align16i(nt2 * 32);
    a.off_pp = off; off += COT * 256;
    a.S3 = ((KWp + 3) & ~3) + best.pad;
    a.off_w3 = off; off += 16 * COT * a.S3 * 4;
    a.off_wd = off; off += align16i(9 * chid);
    if (G == 1) {
        const int slot = plane1 > plane2 ? plane1 : plane2;
        a.slot1 = a.slot2 = slot;
        a.off_t2 = off;
        a.off_t1 = off + nw * slot;
        off += (NP + nw) * slot;
    } else {
        a.slot1 = plane1;
        a.slot2 = plane2;
        a.off_t1 = off; off += NP * plane1;
        a.off_t2 = off; off += NP * plane2;
    }
    off += 2048;  // phase 3 reads up to 8 pixel tiles from a unit's first one, whatever the band holds
    lds = (size_t)off;
    const long long gsz = (long long)a.N * a.bands;
    if (gsz > (1LL << 30)) return false;
    grid = (int)gsz;
    return true;
}

template <int NW> static PlanesFn planes_fn_nw(int kse, bool prelu)
{
    switch (kse) {
    case 1: return prelu ? &block_planes_kernel<1, true, NW> : &block_planes_kernel<1, false, NW>;
    case 2: return prelu ? &block_planes_kernel<2, true, NW> : &block_planes_kernel<2, false, NW>;
    default: return prelu ? &block_planes_kernel<3, true, NW> : &block_planes_kernel<3, false, NW>;
    }
}
static PlanesFn planes_fn(int kse, bool prelu, int nw)
{
    return nw == 16 ? planes_fn_nw<16>(kse, prelu) : nw == 12 ? planes_fn_nw<12>(kse, prelu) : planes_fn_nw<8>(kse, prelu);
}

int launch_planes(const PlanesArgs &a, size_t lds, int grid, int kse, void *stream)
{
    const bool prelu = a.ne != nullptr || a.nd != nullptr;
    const PlanesFn fn = planes_fn(kse, prelu, a.NW);
    static std::mutex mu;
    static std::vector<PlanesFn> attr_done;
    {
        std::lock_guard<std::mutex> lock(mu);
        bool done = false;
        for (PlanesFn f : attr_done) done |= f == fn;
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
    PlanesArgs args = a;
    void *kargs[] = {&args};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(fn), dim3(grid), dim3(64 * a.NW), kargs, lds,
                                         static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        last_hip_error() = e;
        (void)hipGetLastError();
        return PROM_EHIP;
    }
    return check_launch();
}

}  // namespace prom

#ifdef PROM_TIMELINE
extern "C" int prom_debug_pl_stamps(unsigned long long *host)
{
    if (hipDeviceSynchronize() != hipSuccess) return PROM_EHIP;
    return hipMemcpyFromSymbol(host, HIP_SYMBOL(prom::g_pl_stamps), sizeof(unsigned long long) * 256 * 8) == hipSuccess ? PROM_OK : PROM_EHIP;
}
#endif
