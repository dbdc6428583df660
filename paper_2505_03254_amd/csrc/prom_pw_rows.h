// Row-cooperative variant of the streaming pointwise kernel, for layers whose output row is
// wider than one wavefront's chunk of channels.
//
// In the plain streaming kernel the chunks of a row belong to different workgroups: each writes
// row pieces of 16*NT bytes at a stride of the row and re-reads the activations.  Measured on
// gfx950 that costs about 40 % of the rate of a layer whose chunk is the whole row: the memory
// traffic is the same, but a store instruction then touches twice as many 128-byte lines on its
// way through the vector L1, and that path is what limits a write-heavy layer.
//
// Here the CW = 2, 3 or 4 chunks of one pixel group sit on the wavefronts of ONE workgroup
// (G = 4 / CW pixel groups per workgroup step: 2, 1, 1; the workgroup has 64*CW*G threads).  Every wavefront computes its 16 pixels x 16*NT
// channels as before and puts them into a shared LDS tile [16*G pixels][16*NT*CW bytes]; after a
// workgroup barrier all lanes of the workgroup write the tile as whole rows, in 16-byte pieces that follow each
// other in memory.  The tile is double buffered, so one barrier per step suffices: a wavefront
// can reach the writes of step s+2 only through the barrier of step s+1, which every wavefront
// passes after its reads of step s have returned.  The activations of a pixel group are loaded by
// each of its CW wavefronts (same lines at the same time: hits in the vector L1).
//
// A row wider than 16*NT*CW bytes is split into "super-chunks" of that width, handled by different
// workgroups as before (a.n_chunks counts super-chunks here).
#pragma once
#include "prom_pw_stream.h"

namespace prom {

// LDS bytes: fragments and parameters of the CW*NT tiles, two output tiles of
// 16*G pixels x 16*NT*CW bytes.
__host__ __device__ constexpr int rows_groups(int cw) { return 4 / cw; }
__host__ __device__ constexpr int rows_threads(int cw) { return 64 * cw * rows_groups(cw); }
__host__ __device__ constexpr size_t lds_bytes_rows(int nt, int cw, int ks)
{
    return (size_t)cw * nt * ks * 1024 + (size_t)cw * nt * 256 + (size_t)2 * 256 * nt * cw * rows_groups(cw);
}

// Fragments frag[CW*NT][KS][64] and parameters lpar[CW*NT][4 g][4 r] of a super-chunk; tile slot
// cw*NT + t holds the channels base + 16*NT*cw + chan_of<NT>(t, ., .).  Ends with the barrier.
template <int NT>
__device__ __forceinline__ void stage_weights_rows(const PwArgs &a, int cbase, int CW, int nthr, bool prelu, v4i *frag,
                                                   v4i *lpar)
{
    const int tid = threadIdx.x;
    const int KS = a.KS, Nc = a.Nc;
    const int NTT = CW * NT;
    const int nfrag = NTT * KS * 64;
    // The parameter loads and the first batch of weight loads are issued in straight-line code, so
    // that they leave together with the activation loads issued before this call: one memory
    // round trip for everything a workgroup needs before its first MFMA.
    constexpr int PU = 2;  // parameter slots per thread (NTT*16 <= 24*16 channels, >= 192 threads)
    int pb[PU], pm[PU], pn[PU], ps[PU];
#pragma unroll
    for (int q = 0; q < PU; ++q) {
        const int s = tid + q * nthr;
        const int tt = (s >> 4) < NTT ? (s >> 4) : 0;
        const int cw = tt / NT;
        const int t = tt - cw * NT;
        const int c = cbase + cw * NT * 16 + chan_of<NT>(t, (s >> 2) & 3, s & 3);
        const bool ok = s < NTT * 16 && c < Nc;
        const int ci = ok ? c : 0;
        pb[q] = a.bias[ci];
        pm[q] = a.mult[ci];
        ps[q] = a.shift[ci];
        pn[q] = prelu ? a.mult_neg[ci] : 0;
        if (!ok) {
            pb[q] = 0; pm[q] = 0; pn[q] = 0; ps[q] = 1;
        }
    }
    constexpr int U = 8;  // words in flight per thread
    const unsigned recip = (65536u + (unsigned)KS - 1u) / (unsigned)KS;  // tk / KS == (tk * recip) >> 16 for tk < 1024
    auto batch = [&](const int base) __attribute__((always_inline)) {
        uint32_t word[U];
#pragma unroll
        for (int q = 0; q < U; ++q) {
            const int idx = base + q * nthr + tid;
            const int tk = idx < nfrag ? idx >> 6 : 0;
            const int tt = (int)(((unsigned)tk * recip) >> 16);
            const int ks = tk - tt * KS;
            const int cw = tt / NT;
            const int t = tt - cw * NT;
            const int i = idx & 15;
            const int c = cbase + cw * NT * 16 + chan_of<NT>(t, i >> 2, i & 3);
            const int kw = 4 * ks + ((idx & 63) >> 4);
            const bool ok = idx < nfrag && c < Nc && kw < a.KW;
            const uint32_t v = a.wq[ok ? (long long)c * a.KW + kw : 0];
            word[q] = ok ? v : 0u;
        }
#pragma unroll
        for (int q = 0; q < U; ++q) {
            const int idx = base + q * nthr + tid;
            if (idx < nfrag) frag[idx] = decode_word(word[q]);
        }
    };
    batch(0);
    for (int base = nthr * U; base < nfrag; base += nthr * U) batch(base);
#pragma unroll
    for (int q = 0; q < PU; ++q) {
        const int s = tid + q * nthr;
        if (s < NTT * 16) lpar[s] = requant_params(pb[q], pm[q], pn[q], ps[q], prelu);
    }
    for (int s = tid + PU * nthr; s < NTT * 16; s += nthr) {  // (not reached with the compiled shapes)
        const int tt = s >> 4;
        const int cw = tt / NT;
        const int t = tt - cw * NT;
        const int c = cbase + cw * NT * 16 + chan_of<NT>(t, (s >> 2) & 3, s & 3);
        int qb = 0, qm = 0, qn = 0, qs = 1;
        if (c < Nc) {
            qb = a.bias[c];
            qm = a.mult[c];
            qs = a.shift[c];
            if (prelu) qn = a.mult_neg[c];
        }
        lpar[s] = requant_params(qb, qm, qn, qs, prelu);
    }
    __syncthreads();
}

// Requirements (checked by the host): cin % 16 == 0 (XMODE 16) or cin % 8 == 0 (XMODE 8, two
// 8-byte loads per fragment), cout % (16*NT*CW) == 0, 4-byte aligned tensors below 2^31 bytes,
// CW in {2, 3, 4} (a.cw), 64*CW*G threads per workgroup, a.units counts groups of 16 pixels.
template <int NT, bool KS1, int XMODE = 16, int D = 4, int EPI = kEpiPlain>
__device__ __forceinline__ void pw_rows_body(const PwArgs &a, const int lid, unsigned char *lds_raw)
{
    const bool prelu = EPI == kEpiPrelu || (EPI == kEpiBoth && a.mult_neg != nullptr);
    constexpr int NI = (NT + 3) / 4;  // 16-byte pieces per lane per step: 16*G*CW*NT pieces, 64*G*CW lanes
    const int KS = KS1 ? 1 : a.KS;
    const int CW = a.cw, G = 4 / CW, NTT = CW * NT;
    v4i *frag = reinterpret_cast<v4i *>(lds_raw);
    v4i *lpar = frag + NTT * KS * 64;
    unsigned char *tiles = reinterpret_cast<unsigned char *>(lpar + NTT * 16);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15;
    const int g = lane >> 4;

    const int sc = lid % a.n_chunks;
    const int wg = lid / a.n_chunks;
    if (wg >= a.wg_per_chunk) return;  // the whole workgroup leaves: no barrier is missed
    // a workgroup launched with more wavefronts than CW*G (a batch of layers shares one workgroup
    // size): the spare ones leave now; a finished wavefront no longer counts at the barriers
    if (wave >= CW * G) return;
    const int nthr = 64 * CW * G;
    const int cwi = wave % CW;         // this wavefront's chunk within the super-chunk
    const int gsub = wave / CW;        // and its pixel group within the workgroup step
    const int cbase = sc * NTT * 16;
    const int RWs = NTT * 16;          // bytes of a tile row
    const int K = a.K, Nc = a.Nc;

    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a.x), 0, a.M * K, kBufFlags);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, a.M * Nc, kBufFlags);
    const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.residual ? a.residual : a.y), 0, a.M * Nc, kBufFlags);

    // workgroup steps: step i of workgroup wg covers the pixel groups (wg + i*wg_per_chunk)*G + 0..G-1
    const int units_wg = (a.units + G - 1) / G;
    const int my_steps = wg < units_wg ? (units_wg - wg + a.wg_per_chunk - 1) / a.wg_per_chunk : 0;

    int lk = 0;
    unsigned xoff = min((unsigned)kOobOffset, (unsigned)((wg * G + gsub) * 16 + j) * (unsigned)K + 16u * g);
    const unsigned xstep = (unsigned)a.wg_per_chunk * (unsigned)(G * 16) * (unsigned)K;
    auto load_group = [&](v4i &b) {
        if constexpr (XMODE == 16) {
            b = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)xoff, 64 * lk, 0);
        } else {
            const v2i lo2 = __builtin_amdgcn_raw_buffer_load_b64(rx, (int)xoff, 64 * lk, 0);
            const v2i hi2 = __builtin_amdgcn_raw_buffer_load_b64(rx, (int)(xoff + 8), 64 * lk, 0);
            b = v4i{lo2[0], lo2[1], hi2[0], hi2[1]};
        }
        if (KS1 || ++lk == KS) {
            lk = 0;
            xoff = min(xoff + xstep, (unsigned)kOobOffset);
        }
    };
    PW_STAMP(0);
    v4i ring[D];
#pragma unroll
    for (int d = 0; d < D; ++d) load_group(ring[d]);
    PW_STAMP(1);
    stage_weights_rows<NT>(a, cbase, CW, nthr, prelu, frag, lpar);
    PW_STAMP(2);

    v4i par[NT][4];
    const v4i *lpg = lpar + cwi * NT * 16 + g * 4;
    bool sh0 = false;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            par[t][r] = lpg[t * 16 + r];
            sh0 |= par[t][r][3] == 0;
        }
    // per wavefront: the wavefronts of a workgroup may take different forms of the loop; they
    // still meet at the same number of barriers
    const bool general_shift = prelu || __builtin_amdgcn_ballot_w64(sh0) != 0;
    if (!general_shift) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) par[t][r][3] -= 1;
    }
    const int lo = in_vgpr(a.lo), hi = in_vgpr(a.hi);
    const int m128 = in_vgpr(-128), p127 = in_vgpr(127);

    // where this lane puts its outputs in the tile: row gsub*16 + j, this wavefront's columns
    const int wbase = (gsub * 16 + j) * RWs + cwi * NT * 16;
    // the pieces this lane writes to memory: piece q = nthr*i + tid of 16*G*NTT, row-major in the tile
    const int tile_bytes = 256 * G * NTT;
    int goff[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int q = i * nthr + tid;
        const int row = q / NTT;
        goff[i] = q < 16 * G * NTT ? row * Nc + 16 * (q - row * NTT) : kOobOffset;
    }
    // byte offset of (first pixel of the workgroup step, super-chunk base)
    unsigned ytile = min((unsigned)kOobOffset, (unsigned)(wg * G * 16) * (unsigned)Nc + (unsigned)cbase);
    const unsigned ystep = (unsigned)a.wg_per_chunk * (unsigned)(G * 16) * (unsigned)Nc;
    const unsigned rwave = (unsigned)(gsub * 16) * (unsigned)Nc + (unsigned)(cwi * NT * 16);  // for the residual

    const int total_steps = my_steps * KS;
    const int full_rounds = total_steps / D;
    const int tail_steps = total_steps - full_rounds * D;
    const v4i *fl = frag + cwi * NT * KS * 64 + lane;

    auto run = [&](auto has_res_tag, auto mode_tag) {
        constexpr bool HAS_RES = decltype(has_res_tag)::value;
        constexpr int MODE = decltype(mode_tag)::value;
        v4i acc[NT];
        const v4i zero4 = {0, 0, 0, 0};
        // PReLU: the parameters per tile as four vectors over the lane's 4 channels.  The biases
        // are the accumulators' start value (a register quad the first MFMA of a group reads
        // as its C operand), so that the sign of the accumulator is the sign that selects the
        // multiplier.
        v4i cinit[NT], pmul[NT], pneg[NT], pshift[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if constexpr (MODE == 2) {
                cinit[t] = v4i{par[t][0][0], par[t][1][0], par[t][2][0], par[t][3][0]};
                pmul[t] = v4i{par[t][0][1], par[t][1][1], par[t][2][1], par[t][3][1]};
                pneg[t] = v4i{par[t][0][2], par[t][1][2], par[t][2][2], par[t][3][2]};
                pshift[t] = v4i{par[t][0][3], par[t][1][3], par[t][2][3], par[t][3][3]};
            } else {
                cinit[t] = zero4;
            }
        }
        int ck = 0;
        int buf = 0;
        auto step = [&](v4i &slot, auto refill_tag) {
            constexpr bool REFILL = decltype(refill_tag)::value;
            // opaque offset: keeps the fragment reads inside the loop (see the streaming kernel)
            int fo = ck * 64;
            asm volatile("" : "+v"(fo));
            const v4i *fk = fl + fo;
            if (KS1 || ck == 0) {
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fk[t * KS * 64], slot, cinit[t], 0, 0, 0);
            } else {
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fk[t * KS * 64], slot, acc[t], 0, 0, 0);
            }
            if constexpr (REFILL) load_group(slot);
            if (KS1 || ++ck == KS) {
                ck = 0;
                unsigned char *tile = tiles + buf * tile_bytes;
#pragma unroll
                for (int t0 = 0; t0 < NT; t0 += grp_size<NT>(t0)) {
                    const int S = grp_size<NT>(t0);
                    const int cl = chan_of<NT>(t0, g, 0);
                    uint32_t res[4] = {0, 0, 0, 0};
                    if constexpr (HAS_RES) {
                        const int ro = (int)min(ytile + rwave, (unsigned)kOobOffset) + j * Nc + cl;
                        if (S == 4) {
                            const v4i v = __builtin_amdgcn_raw_buffer_load_b128(rr, ro, 0, 0);
                            res[0] = v[0]; res[1] = v[1]; res[2] = v[2]; res[3] = v[3];
                        } else if (S == 2) {
                            const v2i v = __builtin_amdgcn_raw_buffer_load_b64(rr, ro, 0, 0);
                            res[0] = v[0]; res[1] = v[1];
                        } else {
                            res[0] = __builtin_amdgcn_raw_buffer_load_b32(rr, ro, 0, 0);
                        }
                    }
                    uint32_t out[4] = {0, 0, 0, 0};
#pragma unroll
                    for (int tt = 0; tt < 4; ++tt) {
                        if (tt < S) {
                            int v[4];
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                {
                                    if constexpr (MODE == 2)
                                        v[r] = requant_prelu_s(acc[t0 + tt][r], pmul[t0 + tt][r], pneg[t0 + tt][r],
                                                               pshift[t0 + tt][r], lo, hi);
                                    else
                                        v[r] = requant_mode<MODE>(acc[t0 + tt][r], par[t0 + tt][r], lo, hi);
                                }
                            if constexpr (HAS_RES) {
#pragma unroll
                                for (int r = 0; r < 4; ++r) v[r] = med3_i32(v[r] + sbyte(res[tt], r), m128, p127);
                            }
                            out[tt] = pack4_low_bytes(v[0], v[1], v[2], v[3]);
                        }
                    }
                    unsigned char *sp = tile + wbase + cl;
                    if (S == 4)
                        *reinterpret_cast<v4i *>(sp) = v4i{(int)out[0], (int)out[1], (int)out[2], (int)out[3]};
                    else if (S == 2)
                        *reinterpret_cast<v2i *>(sp) = v2i{(int)out[0], (int)out[1]};
                    else
                        *reinterpret_cast<uint32_t *>(sp) = out[0];
                }
                __syncthreads();
#pragma unroll
                for (int i = 0; i < NI; ++i) {
                    const v4i v = *reinterpret_cast<const v4i *>(tile + (i * nthr + tid) * 16);
                    // tile offset in the vector offset: see the store of the streaming kernel
                    store_b128_guarded(v, ry, (int)min((unsigned)goff[i] + ytile, (unsigned)kOobOffset));
                }
                buf ^= 1;
                ytile = min(ytile + ystep, (unsigned)kOobOffset);
            }
        };
        PW_STAMP(3);
        for (int it = 0; it < full_rounds; ++it) {
#pragma unroll
            for (int d = 0; d < D; ++d) step(ring[d], std::true_type{});
            if (it == 0) PW_STAMP(4);
        }
#pragma nounroll
        for (int r = 0; r < tail_steps; ++r) {
            step(ring[0], std::false_type{});
#pragma unroll
            for (int d = 0; d + 1 < D; ++d) ring[d] = ring[d + 1];
        }
        PW_STAMP(5);
#ifdef PROM_TIMELINE
        __builtin_amdgcn_s_waitcnt(0);
        PW_STAMP(6);
#endif
    };

    using Fast = std::integral_constant<int, 0>;
    using General = std::integral_constant<int, 1>;
    using Prelu = std::integral_constant<int, 2>;
    if constexpr (EPI != kEpiPlain) {
        if (prelu) {
            if (a.residual)
                run(std::true_type{}, Prelu{});
            else
                run(std::false_type{}, Prelu{});
            return;
        }
    }
    if constexpr (EPI != kEpiPrelu) {
        if (a.residual) {
            if (general_shift)
                run(std::true_type{}, General{});
            else
                run(std::true_type{}, Fast{});
        } else {
            if (general_shift)
                run(std::false_type{}, General{});
            else
                run(std::false_type{}, Fast{});
        }
    }
}

template <int NT, bool KS1, int XMODE, int EPI>
__global__ __launch_bounds__(256, (NT <= 7 ? 2 : 1)) void pw_rows_kernel(const PwArgs a)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    pw_rows_body<NT, KS1, XMODE, 4, EPI>(a, logical_block_id(), lds_raw);
}

// ---- several independent layers in one launch -------------------------------------------------
// Workgroups [start[i], start[i+1]) (both multiples of 8) run layer i; body[i] selects the kernel
// body (pw_bigbatch_kernel only).
constexpr int kMaxBatch = 32;
struct PwBatchArgs {
    int count;
    int start[kMaxBatch + 1];
    unsigned char body[kMaxBatch];
    PwArgs layer[kMaxBatch];
};
using PwBatchFn = void (*)(PwBatchArgs);

// Bodies pw_bigbatch_kernel carries (the plans the library picks for the large layers at the head
// of MobileNetV2); -1 if this plan is not among them.  Defined in prom_pw_big.hip.
int pw_big_body_id(int nt, int pt, int xmode, bool ks1, bool fullw, int row_waves);
PwBatchFn pw_bigbatch_fn(bool any_prelu);
size_t pw_big_body_lds(int body, const PwArgs &a);
double pw_big_body_ns_per_pixel(int body);
int pw_big_replan(int body, PwArgs &a, int *units_per_wg_round);

// Defined in prom_pw_rows.hip: the instantiation for NT in 1..6 and load width 16 or 8, or nullptr.
PwKernelFn pw_rows_select(int nt, bool ks1, int xmode, bool prelu);
constexpr int kRowsMaxNT = 6;

}  // namespace prom
