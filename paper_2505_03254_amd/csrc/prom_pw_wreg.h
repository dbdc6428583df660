// Pointwise layer with many input channels (the projection layers of the deep inverted-residual
// blocks, Section 2: 384 -> 64/96, 576 -> 96/160, 960 -> 160/320): the decoded weights of such a
// layer (cout x cin bytes: 37 to 307 KB) do not fit LDS beside three resident workgroups, so the
// streaming body cuts the output channels into chunks and reads the activations once per chunk.
// Here the weights live in REGISTERS instead -- the register file is the largest memory of a CU --
// and the activations pass through LDS:
//   - wavefront w of a workgroup owns NTW 16-channel tiles of a group of 4*NTW tiles (64*NTW
//     channels) and keeps their A operands for all KS k steps in registers: decoded once from the
//     2-bit codes (DEC: 4*NTW*KS registers), or, for the deepest layers, as the 2-bit codes
//     themselves (NTW*KS registers) that are decoded right before each MFMA -- 11 vector-ALU
//     instructions per MFMA, which a layer with 9 or 15 k steps per output tile has to spare;
//   - the workgroup walks over 16-pixel tiles.  A tile's 16*cin activation bytes are one contiguous
//     run of the NHWC tensor: the 256 threads fetch it with fully coalesced 16-byte loads (LA tiles
//     ahead, held in registers), put it into a double-buffered LDS slab, and every wavefront reads
//     its B operands from there (rows padded so that the 16-byte reads of 16 pixels fall into
//     different banks).  The activations thus pass the memory pipeline once per group, not once
//     per 48 or 64 output channels;
//   - every wavefront requantises its 16 pixels x 16*NTW channels (parameters read from LDS: with
//     many k steps the epilogue is rare) into a shared, double-buffered output tile, and after the
//     one workgroup barrier of the step all threads write the tile as whole row pieces.
// One barrier per pixel tile: the slab half written in step s was last read in step s-1, the
// output tile half written in step s was last stored in step s-2, both behind a barrier.
//
// Limits (checked on the host): cin % 16 == 0, 64*(KS-1) < cin <= 64*KS, cout % 16 == 0, tensors
// below 2^30 bytes.  Residual and PReLU as in the streaming kernel.
#pragma once
#include "prom_pw_stream.h"

namespace prom {

// Slab row stride: cin bytes, plus 16 when cin/16 is even, so that pixel rows start at 16-byte
// slots j * (odd number): a permutation of the 16 slots of a 256-byte bank row.
__host__ __device__ constexpr int wreg_row_stride(int K) { return ((K >> 4) & 1) ? K : K + 16; }
// 16-byte pieces per thread and pixel tile
__host__ __device__ constexpr int wreg_load_rounds(int ks) { return (64 * ks + 255) / 256; }
// LDS bytes: slab [2][16][stride] (+64: the 16-byte slot idle lanes write, and the over-read of the
// last row when cin % 64 != 0), output tile [2][16][64*NTW], parameters [64*NTW][16].
__host__ __device__ constexpr size_t lds_bytes_wreg(int K, int ntw)
{
    return (size_t)2 * 16 * wreg_row_stride(K) + 64 + (size_t)2 * 16 * 64 * ntw + (size_t)64 * ntw * 16;
}

template <int KS, int NTW, int LA, bool DEC, int EPI>
__device__ __forceinline__ void pw_wreg_body(const PwArgs &a, const int lid, unsigned char *lds_raw)
{
    constexpr bool PRELU = EPI == kEpiPrelu;
    constexpr int GW = 64 * NTW;  // channels of a group
    constexpr int RL = wreg_load_rounds(KS);
    constexpr int SR = (GW + 255) / 256;  // store rounds: one 16-byte piece of the output tile per thread and round
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15;
    const int g = lane >> 4;

    const int ngroups = a.n_chunks;
    const int grp = lid % ngroups;
    const int wg = lid / ngroups;
    if (wg >= a.wg_per_chunk) return;  // the whole workgroup leaves: no barrier is missed
    const int K = a.K, Nc = a.Nc, KW = a.KW;
    const int RS = wreg_row_stride(K);
    const int P = K >> 4;  // 16-byte pieces per pixel row
    const int gbase = grp * GW;
    const int gwv = min(GW, Nc - gbase);  // valid channels of the group, a multiple of 16

    unsigned char *slab = lds_raw;                                  // [2][16][RS]
    unsigned char *idle = slab + 2 * 16 * RS;                       // 64 spare bytes
    unsigned char *outt = idle + 64;                                // [2][16][GW]
    v4i *lpar = reinterpret_cast<v4i *>(outt + 2 * 16 * GW);        // [GW]

    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a.x), 0, a.M * K, kBufFlags);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, a.M * Nc, kBufFlags);
    const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.residual ? a.residual : a.y), 0, a.M * Nc, kBufFlags);

    // ---- this thread's pieces of a pixel tile: piece q = tid + 256*r is bytes [16q, 16q+16) of
    // the tile's 16*K contiguous bytes, i.e. piece q % P of pixel row q / P --------------------
    int lds_x[RL];
    unsigned gx[RL];
#pragma unroll
    for (int r = 0; r < RL; ++r) {
        const int q = tid + 256 * r;
        const bool ok = q < K;  // 16 rows * P pieces = K pieces
        const int px = q / P;
        lds_x[r] = ok ? px * RS + (q - px * P) * 16 : -1;
        gx[r] = ok ? 16u * (unsigned)q : (unsigned)kOobOffset;
    }
    // Tiles wg, wg + WG, ... of this group's pixel tiles; offsets are unsigned and saturate beyond
    // the tensor, where loads read zero and stores are dropped.
    const int WG = a.wg_per_chunk;
    const int count = wg < a.units ? (a.units - wg + WG - 1) / WG : 0;
    const unsigned xstep = (unsigned)WG * 16u * (unsigned)K;
    unsigned xl = min((unsigned)kOobOffset, (unsigned)wg * 16u * (unsigned)K);  // next tile to fetch
    v4i xr[LA][RL];
    auto load_tile = [&](v4i(&slot)[RL]) __attribute__((always_inline)) {
#pragma unroll
        for (int r = 0; r < RL; ++r)
            slot[r] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)min(xl + gx[r], (unsigned)kOobOffset), 0, 0);
        xl = min(xl + xstep, (unsigned)kOobOffset);
    };
    auto put_tile = [&](const v4i(&slot)[RL], int buf) __attribute__((always_inline)) {
        unsigned char *sb = slab + buf * (16 * RS);
#pragma unroll
        for (int r = 0; r < RL; ++r) {
            unsigned char *dst = lds_x[r] >= 0 ? sb + lds_x[r] : idle + 16 * (lane & 3);
            *reinterpret_cast<v4i *>(dst) = slot[r];
        }
    };
    load_tile(xr[0]);

    // ---- weights of this wavefront's tiles into registers; parameters of the group into LDS ----
    uint32_t Aw[NTW][KS];            // the 2-bit codes of this lane's 16 weights per tile and k step
    v4i A[DEC ? NTW : 1][DEC ? KS : 1];  // DEC: the same decoded
    {
#pragma unroll
        for (int t = 0; t < NTW; ++t) {
            const int c = gbase + 16 * (wave * NTW + t) + j;  // A row = D row = channel within the tile
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int kw = 4 * ks + g;
                const bool ok = c < Nc && kw < KW;
                const uint32_t v = a.wq[ok ? (long long)c * KW + kw : 0];
                Aw[t][ks] = ok ? v : 0u;
            }
        }
        for (int p = tid; p < GW; p += 256) {
            const int c = gbase + p;
            v4i pr = {0, 0, 0, 1};
            if (c < Nc) pr = requant_params(a.bias[c], a.mult[c], PRELU ? a.mult_neg[c] : 0, a.shift[c], PRELU);
            lpar[p] = pr;
        }
        if constexpr (DEC) {
#pragma unroll
            for (int t = 0; t < NTW; ++t)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) A[t][ks] = decode_word(Aw[t][ks]);
        }
    }
    put_tile(xr[0], 0);
#pragma unroll
    for (int u = 1; u <= LA; ++u) load_tile(xr[u % LA]);
    __syncthreads();

    // any shift of the group equal to 0 -> the general form of the requantisation (every wavefront
    // scans the whole group, so the decision is uniform over the workgroup)
    bool sh0 = false;
    if constexpr (!PRELU)
        for (int c = lane; c < GW; c += 64) sh0 |= lpar[c][3] == 0;
    const bool general_shift = __builtin_amdgcn_ballot_w64(sh0) != 0;

    const int lo = in_vgpr(a.lo), hi = in_vgpr(a.hi);
    const int m128 = in_vgpr(-128), p127 = in_vgpr(127);
    // output tile -> global: piece p = tid + 256*r (p < gwv) is piece p % (gwv/16) of pixel row
    // p / (gwv/16)
    const int ppr = gwv >> 4;
    int so_lds[SR];
    unsigned so_g[SR];
#pragma unroll
    for (int r = 0; r < SR; ++r) {
        const int p = tid + 256 * r;
        const int srow = p / ppr, scol = p - srow * ppr;
        so_lds[r] = p < gwv ? srow * GW + 16 * scol : 0;
        so_g[r] = p < gwv ? (unsigned)(srow * Nc + gbase + 16 * scol) : (unsigned)kOobOffset;
    }
    const unsigned ystep = (unsigned)WG * 16u * (unsigned)Nc;
    unsigned ytile = min((unsigned)kOobOffset, (unsigned)wg * 16u * (unsigned)Nc);
    // this lane's dwords: tile tl of the group, pixel j, channels 16*tl + 4g .. +3
    const int tl0 = wave * NTW;
    const v4i zero4 = {0, 0, 0, 0};

    auto run = [&](auto has_res_tag, auto mode_tag) __attribute__((always_inline)) {
        constexpr bool HAS_RES = decltype(has_res_tag)::value;
        constexpr int MODE = decltype(mode_tag)::value;
        int s = 0;
        auto step = [&](v4i(&slot)[RL]) __attribute__((always_inline)) {
            const int buf = s & 1;
            uint32_t res[NTW];
            if constexpr (HAS_RES) {
#pragma unroll
                for (int t = 0; t < NTW; ++t)
                    res[t] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(
                        rr, (int)min(ytile + (unsigned)(j * Nc + gbase + 16 * (tl0 + t) + 4 * g), (unsigned)kOobOffset), 0, 0);
            }
            // ---- accumulate: B operands from the slab, A operands from registers.  The LDS reads run
            // two k steps ahead of the MFMAs and no further (scheduling barriers): left alone the
            // compiler issues all KS reads first and holds 4*KS registers for them -------------
            v4i acc[NTW];
            const unsigned char *sb = slab + buf * (16 * RS) + j * RS + 16 * g;
            v4i Bq[KS];
            Bq[0] = *reinterpret_cast<const v4i *>(sb);
            if constexpr (KS > 1) Bq[1] = *reinterpret_cast<const v4i *>(sb + 64);
#pragma unroll
            for (int ks = 0; ks < KS; ks += 2) {
                __builtin_amdgcn_sched_barrier(0);
                if (ks + 2 < KS) Bq[ks + 2] = *reinterpret_cast<const v4i *>(sb + 64 * (ks + 2));
                if (ks + 3 < KS) Bq[ks + 3] = *reinterpret_cast<const v4i *>(sb + 64 * (ks + 3));
#pragma unroll
                for (int kk = ks; kk < ks + 2 && kk < KS; ++kk)
#pragma unroll
                    for (int t = 0; t < NTW; ++t) {
                        v4i Af;
                        if constexpr (DEC)
                            Af = A[t][kk];
                        else {
                            // opaque copy: the codes are loop invariants, and the compiler would
                            // otherwise decode them all once and keep 4 registers per operand
                            uint32_t w = Aw[t][kk];
                            asm volatile("" : "+v"(w));
                            Af = decode_word(w);
                        }
                        acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(Af, Bq[kk], kk == 0 ? zero4 : acc[t], 0, 0, 0);
                    }
            }
            __builtin_amdgcn_sched_barrier(0);
            // ---- the tile after this one into the other half of the slab, a new tile on its way -
            put_tile(slot, buf ^ 1);
            load_tile(slot);
            // ---- requantise into the shared output tile, tile by tile (the parameters of one
            // tile at a time in registers) ---------------------------------------------------------
            unsigned char *ob = outt + buf * (16 * GW) + j * GW + 4 * g;
#pragma unroll
            for (int t = 0; t < NTW; ++t) {
                v4i pt[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    pt[r] = lpar[16 * (tl0 + t) + 4 * g + r];
                    if constexpr (MODE == 0) pt[r][3] -= 1;
                }
                int v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    v[r] = requant_mode<MODE>(acc[t][r], pt[r], lo, hi);  // (the PReLU form adds the bias itself)
                    if constexpr (HAS_RES) v[r] = med3_i32(v[r] + sbyte(res[t], r), m128, p127);
                }
                *reinterpret_cast<uint32_t *>(ob + 16 * (tl0 + t)) = pack4_low_bytes(v[0], v[1], v[2], v[3]);
                if (t + 1 < NTW) __builtin_amdgcn_sched_barrier(0);
            }
            __syncthreads();
            // ---- the tile leaves as row pieces of gwv bytes (whole rows when there is one group) --
#pragma unroll
            for (int r = 0; r < SR; ++r) {
                const v4i v = *reinterpret_cast<const v4i *>(outt + buf * (16 * GW) + so_lds[r]);
                // offset in the vector operand (see the streaming kernel's store)
                store_b128_guarded(v, ry, (int)min(so_g[r] + ytile, (unsigned)kOobOffset));
            }
            ytile = min(ytile + ystep, (unsigned)kOobOffset);
            ++s;
        };
        // Steps run in rounds of LA ring slots, straight-line; steps past the end of this
        // workgroup's tiles work on zeros (their offsets are beyond the tensor) and store nothing.
        const int rounds = (count + LA - 1) / LA;
        for (int it = 0; it < rounds; ++it) {
#pragma unroll
            for (int d = 0; d < LA; ++d) step(xr[(d + 1) % LA]);
        }
    };
    using Fast = std::integral_constant<int, 0>;
    using General = std::integral_constant<int, 1>;
    using Prelu = std::integral_constant<int, 2>;
    if constexpr (PRELU) {
        if (a.residual)
            run(std::true_type{}, Prelu{});
        else
            run(std::false_type{}, Prelu{});
    } else {
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

}  // namespace prom
