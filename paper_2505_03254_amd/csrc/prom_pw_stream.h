// Ternary pointwise 1x1 convolution on gfx950: int8 MFMA over weights decoded from 2-bit
// codes into LDS, activations streamed from HBM straight into the MFMA operand registers,
// exact integer requantisation in the epilogue, outputs staged through LDS so that every
// global store instruction writes one contiguous run.
//
// Formulation.  The layer is Y[m][co] = sum_k X[m][k] * W[co][k]  (paper Section 2: a sum of
// input channels; Section 3.1: convolve with the ternary weights, rescale afterwards).  The
// kernel computes the transpose, D = W_tile (16 channels x 64 k) * X_tile^T (64 k x 16 pixels)
// with v_mfma_i32_16x16x64_i8, because then
//   - the B operand of lane l is 16 consecutive k-bytes of pixel (l & 15): one 16-byte
//     load from the NHWC row, no LDS staging of activations;
//   - the D registers of lane l are 4 consecutive output channels of pixel (l & 15): one
//     packed dword of int8 outputs, and per-lane requantisation parameters.
// A wavefront owns NT 16-channel tiles (a "chunk" of 16*NT output channels) and walks over
// groups of 16*PT pixels; the 4 wavefronts of a workgroup share the decoded weights.
//
// Requantisation.  With acc the raw accumulator, the epilogue needs
//     q = floor(((acc + bias) * mult + 2^(30+shift)) / 2^(31+shift)).
// Per channel the prologue forms the 64-bit constant C = bias*mult + 2^(30+shift); then
//     t = acc*mult + C            one v_mad_i64_i32 (full rate on gfx950)
//     q = hi32(t) >> (shift-1)    when shift >= 1 (arithmetic shifts are floor divisions)
//     q = (t >> 31) >> shift      in general (taken by a workgroup whose chunk has a shift of 0)
// which is exact integer arithmetic for |acc + bias| < 2^30.
//
// Memory pipeline.  The streaming kernel addresses x, y and the residual through buffer
// resources: an access whose byte offset is beyond the tensor reads zero or is dropped by the
// hardware, so ragged pixel counts need no branches, the loop body is straight-line code, and
// the activation loads of a ring of D future steps stay in flight across the epilogue.
#pragma once
#include "prom.h"
#include "prom_device.h"

#include <type_traits>

namespace prom {

// Which epilogues a kernel body carries: the plain forms, the PReLU form, or both.  A body is
// compiled per kind because the registers of a kernel are those of its hungriest path; the
// shared-launch kernels take kEpiBoth to mean "members of either kind" and run each member through
// a body of its own kind, so no body is instantiated with both at present.
constexpr int kEpiPlain = 0, kEpiPrelu = 1, kEpiBoth = 2;

struct PwArgs {
    const int8_t *x;
    const uint32_t *wq;
    const int32_t *bias;
    const int32_t *mult;
    const int32_t *mult_neg;  // PReLU: multiplier for acc + bias < 0, or nullptr
    const int32_t *shift;
    const int8_t *residual;
    int8_t *y;
    int32_t *acc_out;
    int M;       // pixels
    int units;   // pixel groups of 16*PT pixels, one per wavefront iteration
    int K, Nc;
    int KW;      // packed 32-bit words per weight row = ceil(K/16)
    int KS;      // 64-wide k steps = ceil(K/64)
    int n_chunks;      // output-channel chunks of 16*NT channels
    int wg_per_chunk;  // workgroups per chunk; 4*wg_per_chunk wavefronts share the units
    int lo, hi;        // activation window
    int cw;            // row-cooperative kernel only: chunks of a pixel group per workgroup (2 or 4), else 0
};

// Tiles of a chunk are stored in groups of 4, then 2, then 1 so that a lane's outputs of a
// group are 16, 8 or 4 contiguous bytes.
template <int NT> __host__ __device__ constexpr int grp_size(int t)
{
    return t < 4 * (NT / 4) ? 4 : (((NT % 4) >= 2 && t < 4 * (NT / 4) + 2) ? 2 : 1);
}
template <int NT> __host__ __device__ constexpr int grp_first(int t)
{
    return t < 4 * (NT / 4) ? (t & ~3)
           : (((NT % 4) >= 2 && t < 4 * (NT / 4) + 2) ? 4 * (NT / 4)
                                                       : 4 * (NT / 4) + ((NT % 4) >= 2 ? 2 : 0));
}
// Channel (relative to the chunk base) held in D row 4*gr + r of tile slot t.
template <int NT> __host__ __device__ constexpr int chan_of(int t, int gr, int r)
{
    return 16 * grp_first<NT>(t) + 4 * grp_size<NT>(t) * gr + 4 * (t - grp_first<NT>(t)) + r;
}

// 16 two-bit codes (layout of prom_pack_ternary) -> 16 int8 weights in MFMA operand order.
__device__ __forceinline__ v4i decode_word(uint32_t word)
{
    v4i f;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        // code c in {0,1,3} -> byte selector 2c in {0,2,6} of the 8-byte table below
        const uint32_t sel = ((word >> (2 * d)) & 0x03030303u) << 1;
        // table bytes: [0]=0x00 (zero), [2]=0x01 (+1), [6]=0xFF (-1)
        f[d] = (int)__builtin_amdgcn_perm(0x00FF0000u, 0x00010000u, sel);
    }
    return f;
}

// Decode the chunk's weights into LDS fragments frag[NT][KS][64 lanes] and the chunk's
// requantisation parameters into lpar[NT][4 g][4 r] = (C lo, C hi, mult, shift), or
// (bias, mult, mult_neg, shift) for a PReLU layer.  Ends with the workgroup barrier that
// publishes both.
template <int NT, bool WITH_PARAMS>
__device__ __forceinline__ void stage_weights(const PwArgs &a, int cbase, v4i *frag, v4i *lpar, bool prelu)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int KS = a.KS, Nc = a.Nc;
    int pb = 0, pm = 0, pn = 0, ps = 1;
    const bool ptid = WITH_PARAMS && tid < NT * 16;
    if (ptid) {
        const int c = cbase + chan_of<NT>(tid >> 4, (tid >> 2) & 3, tid & 3);
        if (c < Nc) {
            pb = a.bias[c];
            pm = a.mult[c];
            ps = a.shift[c];
            if (prelu) pn = a.mult_neg[c];
        }
    }
    // A fragment entry e = t*KS + ks is 64 lanes x 16 bytes: lane (i, kg) holds the decoded word
    // 4*ks + kg of the row of channel chan_of(t, i).  The loads of a batch are issued back to back
    // -- the first batch in straight-line code, so that it leaves together with the activation
    // loads issued before this call instead of behind a wait at a loop header -- and decoded as
    // they arrive.
    const int total = NT * KS;
    if ((a.KW & 3) == 0 && (reinterpret_cast<uintptr_t>(a.wq) & 15) == 0) {
        // Rows of whole 16-byte pieces: a thread fetches the four words of (entry, i) with one
        // load and decodes them for the lanes kg = 0..3 of the entry; 16 threads per entry.
        constexpr int U = 4;
        const unsigned recip = (65536u + (unsigned)KS - 1u) / (unsigned)KS;  // e / KS == (e * recip) >> 16 for e < 1024
        const int i = tid & 15;
        auto batch = [&](const int v0) __attribute__((always_inline)) {
            v4i w4[U];
#pragma unroll
            for (int q = 0; q < U; ++q) {
                const int e = (v0 + 256 * q + tid) >> 4;
                const int t = (int)(((unsigned)e * recip) >> 16), ks = e - t * KS;
                const bool valid = e < total;
                const int c = cbase + chan_of<NT>(valid ? t : 0, i >> 2, i & 3);
                const bool ok = valid && c < Nc;
                const v4i v = *reinterpret_cast<const v4i *>(a.wq + (ok ? (long long)c * a.KW + 4 * ks : 0));
                w4[q] = ok ? v : v4i{0, 0, 0, 0};
            }
#pragma unroll
            for (int q = 0; q < U; ++q) {
                const int e = (v0 + 256 * q + tid) >> 4;
                if (e < total) {
#pragma unroll
                    for (int kg = 0; kg < 4; ++kg) frag[e * 64 + 16 * kg + i] = decode_word((uint32_t)w4[q][kg]);
                }
            }
        };
        batch(0);
        for (int v0 = 256 * U; v0 < total * 16; v0 += 256 * U) batch(v0);
    } else {
        // Any row length: one word per lane; wavefront w decodes entries w, w + 4, ... (tile and k
        // step of an entry are wave-uniform and advance without a division).
        constexpr int U = 16;
        const int i = lane & 15, kg = lane >> 4;
        int t = 0, ks = wave;
        while (ks >= KS) {
            ks -= KS;
            ++t;
        }
        auto batch = [&](const int e0) __attribute__((always_inline)) {
            uint32_t word[U];
#pragma unroll
            for (int q = 0; q < U; ++q) {
                const bool valid = e0 + 4 * q < total;
                const int c = cbase + chan_of<NT>(valid ? t : 0, i >> 2, i & 3);
                const int kw = 4 * ks + kg;
                // clamp instead of branching so that the loads of a batch are issued back to back
                const bool ok = valid && c < Nc && kw < a.KW;
                const uint32_t v = a.wq[ok ? (long long)c * a.KW + kw : 0];
                word[q] = ok ? v : 0u;
                ks += 4;
                while (ks >= KS) {
                    ks -= KS;
                    ++t;
                }
            }
#pragma unroll
            for (int q = 0; q < U; ++q)
                if (e0 + 4 * q < total) frag[(e0 + 4 * q) * 64 + lane] = decode_word(word[q]);
        };
        batch(wave);
        for (int e0 = wave + 4 * U; e0 < total; e0 += 4 * U) batch(e0);
    }
    if (ptid) lpar[tid] = requant_params(pb, pm, pn, ps, prelu);
    __syncthreads();
}

// XCD-aware logical workgroup id: consecutive hardware ids go round-robin over the 8 XCDs;
// make logical neighbours (the chunks of one pixel range) land on the same XCD and L2.
__device__ __forceinline__ int logical_block_id(int bid, int nblk /* multiple of 8 */)
{
    return (bid & 7) * (nblk >> 3) + (bid >> 3);
}
__device__ __forceinline__ int logical_block_id() { return logical_block_id(blockIdx.x, gridDim.x); }
// The same for member `m` of a shared launch.  A member's grid is padded to a multiple of 8 and the
// padding is its last logical ids, i.e. all in one XCD's eighth; the eighths are handed to the XCDs
// rotated by the member's index, so that it is not the same XCD that comes short in every member.
__device__ __forceinline__ int logical_block_id(int bid, int nblk, int m)
{
    return ((bid + m) & 7) * (nblk >> 3) + (bid >> 3);
}

// Depth of the activation prefetch ring (load groups in flight per wavefront).
template <int PT> __host__ __device__ constexpr int ring_depth() { return PT == 1 ? 4 : 3; }

// LDS bytes of the streaming kernel: decoded weight fragments, one int4 of parameters per
// channel, one output staging tile (16 pixels x 16*NT bytes) per wavefront.
__host__ __device__ constexpr size_t lds_bytes_fast(int nt, int ks)
{
    return (size_t)nt * ks * 1024 + (size_t)nt * 16 * 16 + (size_t)4 * 256 * nt;
}
__host__ __device__ constexpr size_t lds_bytes_generic(int nt, int ks)
{
    return (size_t)nt * ks * 1024 + (size_t)nt * 16 * 16;
}

constexpr int kBufFlags = 0x00020000;   // raw buffer of dwords, gfx9 family
constexpr int kOobOffset = 0x7ffff000;  // byte offset beyond any tensor handled here

// ============================================================================================
// Streaming kernel: cin % 8 == 0, cout % 4 == 0, 4-byte aligned tensors below 2^30 bytes, and
// either one chunk (its tile is one contiguous run) or cout % 16 == 0.
//   XMODE 16: cin % 16 == 0, one 16-byte load per fragment; XMODE 8: two 8-byte loads.
//   KS1: cin <= 64 (one k step per group, no branch around the epilogue).
//   FULLW: cout % (16*NT) == 0, every chunk is 16*NT valid channels wide (no per-lane channel
//          conditions, compile-time staging geometry).
// ============================================================================================
// `lid` is the workgroup's logical id within this layer's grid (see logical_block_id).
#ifdef PROM_TIMELINE
// Developer build: the first 64 logical workgroups of a single-layer launch record the 100 MHz
// clock at 8 points of their life into the buffer the host passed in a.acc_out (unused otherwise).
#define PW_STAMP(i)                                                                                  \
    do {                                                                                             \
        if (a.acc_out && threadIdx.x == 0 && lid < 64)                                               \
            reinterpret_cast<unsigned long long *>(a.acc_out)[lid * 8 + (i)] = wall_clock64();       \
    } while (0)
#else
#define PW_STAMP(i) do { } while (0)
#endif

template <int NT, int PT, int XMODE, bool KS1, bool FULLW, int D = ring_depth<PT>(), int EPI = kEpiPlain>
__device__ __forceinline__ void pw_stream_body(const PwArgs &a, const int lid, unsigned char *lds_raw)
{
    PW_STAMP(0);
    // PReLU layer?  Known at compile time unless the body carries both kinds of epilogue.
    const bool prelu = EPI == kEpiPrelu || (EPI == kEpiBoth && a.mult_neg != nullptr);
    constexpr int NI = (NT + 3) / 4;  // 16-byte store instructions per staged tile
    const int KS = KS1 ? 1 : a.KS;
    v4i *frag = reinterpret_cast<v4i *>(lds_raw);  // [NT][KS][64 lanes] decoded A operands
    v4i *lpar = frag + NT * KS * 64;               // [NT][4 g][4 r] requantisation parameters
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keep it in a scalar register
    const int j = lane & 15;  // pixel within a 16-pixel tile
    const int g = lane >> 4;  // k group on the input side, channel group on the output side

    const int chunk = lid % a.n_chunks;
    const int wg = lid / a.n_chunks;
    if (wg >= a.wg_per_chunk) return;
    const int cbase = chunk * NT * 16;
    const int Wv = a.wg_per_chunk * 4;  // wavefronts sharing the pixel groups of this chunk
    const int w0 = wg * 4 + wave;       // this wavefront's first group
    const int K = a.K, Nc = a.Nc;
    unsigned char *stage = reinterpret_cast<unsigned char *>(lpar + NT * 16) + wave * (256 * NT);

    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a.x), 0, a.M * K, kBufFlags);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, a.M * Nc, kBufFlags);
    const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.residual ? a.residual : a.y), 0, a.M * Nc, kBufFlags);

    // ---- load cursor: next (group, k step) to fetch.  Offsets beyond the tensor read zero. ----
    // Offsets are unsigned 32-bit and saturate at kOobOffset, so running past the end of this
    // wavefront's work can never wrap around into the tensor.
    int lk = 0;
    unsigned xoff = min((unsigned)kOobOffset,
                        (unsigned)(w0 * (16 * PT) + j) * (unsigned)K + 16u * g);  // pixel tile 0, k step 0
    const unsigned xstep = (unsigned)Wv * (16 * PT) * (unsigned)K;
    auto load_group = [&](v4i(&b)[PT]) {
#pragma unroll
        for (int p = 0; p < PT; ++p) {
            const int so = (16 * p) * K + 64 * lk;
            if constexpr (XMODE == 16) {
                b[p] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)xoff, so, 0);
            } else {
                const v2i lo2 = __builtin_amdgcn_raw_buffer_load_b64(rx, (int)xoff, so, 0);
                const v2i hi2 = __builtin_amdgcn_raw_buffer_load_b64(rx, (int)(xoff + 8), so, 0);
                b[p] = v4i{lo2[0], lo2[1], hi2[0], hi2[1]};
            }
        }
        if (KS1 || ++lk == KS) {
            lk = 0;
            xoff = min(xoff + xstep, (unsigned)kOobOffset);
        }
    };

    // ---- start the activation prefetch ring before anything else ----------------------------
    v4i ring[D][PT];
#pragma unroll
    for (int d = 0; d < D; ++d) load_group(ring[d]);
    PW_STAMP(1);
    stage_weights<NT, true>(a, cbase, frag, lpar, prelu);
    PW_STAMP(2);

    // per-lane parameters: 4 channels per tile slot.  The lanes of a wavefront hold every channel
    // of the chunk between them, so a wavefront can see by itself whether any shift is 0 and
    // then takes the general form of the requantisation; otherwise .w holds shift-1.
    v4i par[NT][4];
    const v4i *lpg = lpar + g * 4;
    bool sh0 = false;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            par[t][r] = lpg[t * 16 + r];
            sh0 |= par[t][r][3] == 0;
        }
    const bool general_shift = prelu || __builtin_amdgcn_ballot_w64(sh0) != 0;
    if (!general_shift) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) par[t][r][3] -= 1;
    }
    const int lo = in_vgpr(a.lo), hi = in_vgpr(a.hi);
    const int m128 = in_vgpr(-128), p127 = in_vgpr(127);

    // ---- output staging geometry (uniform per workgroup) -----------------------------------------
    // RW: valid bytes per pixel row of this chunk.  The staged tile is 16 rows of RW bytes,
    // written to y in 16-byte pieces; piece q = 64*i + lane sits at staged offset 16*q.  When the
    // chunk is the whole row (RW == Nc) the tile is one contiguous run of 16*Nc bytes; otherwise
    // RW % 16 == 0 and a piece never crosses a row.
    const int RW = FULLW ? 16 * NT : min(16 * NT, Nc - cbase);
    const bool rw16 = (RW & 15) == 0, rw8 = (RW & 7) == 0;
    const bool contig = RW == Nc;
    int goff[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int q = i * 64 + lane;
        int o;
        if (contig) {
            o = 16 * q;
        } else {
            const int per_row = RW >> 4;
            const int row = q / per_row;
            o = row * Nc + 16 * (q - row * per_row);
        }
        goff[i] = q < RW ? o : kOobOffset;
    }

    // byte offset of (first pixel of the group, chunk base); uniform per wavefront
    unsigned ytile = min((unsigned)kOobOffset, (unsigned)(w0 * (16 * PT)) * (unsigned)Nc + (unsigned)cbase);
    const unsigned ystep = (unsigned)Wv * (16 * PT) * (unsigned)Nc;

    const int my_groups = w0 < a.units ? (a.units - w0 + Wv - 1) / Wv : 0;
    const int total_steps = my_groups * KS;
    const int full_rounds = total_steps / D;
    const int tail_steps = total_steps - full_rounds * D;
    const v4i *fl = frag + lane;

    // ---- main loop: D ring slots per round, straight-line.  Refills past the end of this
    // wavefront's work read zeros (their offsets are beyond the tensor) and are never used.
    // The last total_steps % D steps run one at a time on slot 0 with the ring rotated down.
    // The loop is instantiated per (residual, epilogue form) so that its body has no branch on
    // either. ------------------------------------------------------------------------------------
    auto run = [&](auto has_res_tag, auto mode_tag) {
        constexpr bool HAS_RES = decltype(has_res_tag)::value;
        constexpr int MODE = decltype(mode_tag)::value;
        v4i acc[PT][NT];
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
        auto step = [&](v4i(&slot)[PT], auto refill_tag) {
            constexpr bool REFILL = decltype(refill_tag)::value;
            // opaque offset: the fragment reads stay inside the loop (4 registers in flight per
            // tile) instead of being hoisted into 4*NT*KS registers when the weights are loop-invariant
            int fo = ck * 64;
            asm volatile("" : "+v"(fo));
            const v4i *fk = fl + fo;
            if (KS1 || ck == 0) {
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const v4i wfrag = fk[t * KS * 64];
#pragma unroll
                    for (int p = 0; p < PT; ++p)
                        acc[p][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wfrag, slot[p], cinit[t], 0, 0, 0);
                }
            } else {
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const v4i wfrag = fk[t * KS * 64];
#pragma unroll
                    for (int p = 0; p < PT; ++p)
                        acc[p][t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wfrag, slot[p], acc[p][t], 0, 0, 0);
                }
            }
            if constexpr (REFILL) load_group(slot);  // refill this slot with the group D steps ahead
            if (KS1 || ++ck == KS) {
                ck = 0;
#pragma unroll
                for (int p = 0; p < PT; ++p) {
                    const int tile_off = (int)(ytile + (unsigned)((16 * p) * Nc));
#pragma unroll
                    for (int t0 = 0; t0 < NT; t0 += grp_size<NT>(t0)) {
                        const int S = grp_size<NT>(t0);
                        const int cl = chan_of<NT>(t0, g, 0);  // lane's first channel of the group
                        uint32_t res[4] = {0, 0, 0, 0};
                        if constexpr (HAS_RES) {
                            const int ro = j * Nc + cl;
                            if (S == 4) {
                                const v4i v = __builtin_amdgcn_raw_buffer_load_b128(rr, ro, tile_off, 0);
                                res[0] = v[0]; res[1] = v[1]; res[2] = v[2]; res[3] = v[3];
                            } else if (S == 2) {
                                const v2i v = __builtin_amdgcn_raw_buffer_load_b64(rr, ro, tile_off, 0);
                                res[0] = v[0]; res[1] = v[1];
                            } else {
                                res[0] = __builtin_amdgcn_raw_buffer_load_b32(rr, ro, tile_off, 0);
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
                                        v[r] = requant_prelu_s(acc[p][t0 + tt][r], pmul[t0 + tt][r], pneg[t0 + tt][r],
                                                               pshift[t0 + tt][r], lo, hi);
                                    else
                                        v[r] = requant_mode<MODE>(acc[p][t0 + tt][r], par[t0 + tt][r], lo, hi);
                                }
                                if constexpr (HAS_RES) {
#pragma unroll
                                    for (int r = 0; r < 4; ++r)
                                        v[r] = med3_i32(v[r] + sbyte(res[tt], r), m128, p127);
                                }
                                out[tt] = pack4_low_bytes(v[0], v[1], v[2], v[3]);
                            }
                        }
                        // stage the lane's dwords at [pixel j][channel cl..] of the wavefront's tile
                        unsigned char *sp = stage + j * RW + cl;
                        const bool full = FULLW || cl + 4 * S <= RW;
                        if (full && S == 4 && (FULLW || rw16)) {
                            *reinterpret_cast<v4i *>(sp) = v4i{(int)out[0], (int)out[1], (int)out[2], (int)out[3]};
                        } else if (full && S == 2 && (FULLW || rw8)) {
                            *reinterpret_cast<v2i *>(sp) = v2i{(int)out[0], (int)out[1]};
                        } else {
#pragma unroll
                            for (int tt = 0; tt < 4; ++tt)
                                if (tt < S && (FULLW || cl + 4 * tt + 4 <= RW))
                                    *reinterpret_cast<uint32_t *>(sp + 4 * tt) = out[tt];
                        }
                    }
                    // write the staged tile; pieces outside the tile or the tensor are dropped
#pragma unroll
                    for (int i = 0; i < NI; ++i) {
                        const v4i v = *reinterpret_cast<const v4i *>(stage + (i * 64 + lane) * 16);
                        // The tile offset goes into the vector offset (goff is unsigned-saturated, so
                        // the sum cannot wrap into the tensor); see store_b128_guarded for the hazard
                        // this store form once ran into with a scalar offset.
                        store_b128_guarded(v, ry, (int)min((unsigned)goff[i] + (unsigned)tile_off, (unsigned)kOobOffset));
                    }
                }
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
            for (int d = 0; d + 1 < D; ++d)
#pragma unroll
                for (int p = 0; p < PT; ++p) ring[d][p] = ring[d + 1][p];
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

template <int NT, int PT, int XMODE, bool KS1, bool FULLW, int EPI>
__global__ __launch_bounds__(256, (NT * PT <= (EPI == kEpiPlain ? 7 : 6) ? 2 : 1)) void pw_stream_kernel(const PwArgs a)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    pw_stream_body<NT, PT, XMODE, KS1, FULLW, ring_depth<PT>(), EPI>(a, logical_block_id(), lds_raw);
}

using PwKernelFn = void (*)(const PwArgs);

// One translation unit per NT instantiates the streaming kernel (prom_pw_inst.hip) and exports
// its selector; returns nullptr for a combination that is not compiled.
template <int NT> PwKernelFn pw_stream_select(int pt, int xmode, bool ks1, bool fullw, bool prelu);

constexpr int kMaxNT = 10;

}  // namespace prom
