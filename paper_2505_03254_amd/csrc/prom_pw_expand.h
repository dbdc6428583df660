// Pointwise layer with few input and many output channels (the expansion layers of the
// inverted-residual blocks, Section 2): the activations of a pixel group stay in registers while
// the wavefront walks over the output channels, so that they pass through the memory pipeline
// once per part of the output channels instead of once per 64 of them.
//
// Work division.  The output channels are cut into sub-chunks of 64 (4 MFMA tiles) and the
// sub-chunks into parts of up to a.cw consecutive ones; a workgroup belongs to one part (decoded
// fragments and parameters of all its sub-chunks in LDS) and its 4 wavefronts take pixel units of
// 16*G pixels round robin with the other workgroups of the part.  Per unit a wavefront holds
// G x KSC B operands (16 bytes per lane each), and for every sub-chunk and pixel tile runs
// 4 x KSC MFMAs, requantises and stores 16 pixels x 64 channels.  The B operands of the next unit
// are fetched tile by tile during the last sub-chunk, right after a tile's last MFMA.
//
// Limits (checked on the host): K % 16 == 0, K <= 64*KSC, Nc % 64 == 0, no residual, tensors
// below 2^30 bytes.  PRELU: the layer has PReLU multipliers (a.mult_neg).
#pragma once
#include "prom_pw_stream.h"

namespace prom {

// LDS bytes: fragments and parameters of a part, one 16 x 64-byte staging tile per wavefront.
__host__ __device__ constexpr size_t lds_bytes_expand(int nsc, int ks)
{
    return (size_t)nsc * (4 * ks * 1024 + 1024) + 4 * 1024;
}

// Decode the weights of sub-chunks [sc0, sc0 + nsc) into frag[nsc][4][KSC][64 lanes] and their
// requantisation parameters into lpar[nsc][4][4 g][4 r] = (C lo, C hi, mult, shift), or (bias, mult,
// mult_neg, shift) for a PReLU layer; all global loads of a thread are issued before the first
// decode.  Ends with the workgroup barrier.
template <int KSC, bool PRELU>
__device__ __forceinline__ void stage_part(const PwArgs &a, int sc0, int nsc, v4i *frag, v4i *lpar)
{
    const int tid = threadIdx.x;
    const int nfrag = nsc * 4 * KSC * 64;
    constexpr int U = 12;  // words in flight per thread
    for (int base = 0; base < nfrag; base += 256 * U) {
        uint32_t word[U];
#pragma unroll
        for (int q = 0; q < U; ++q) {
            const int idx = base + q * 256 + tid;
            const int tk = idx >> 6;  // (sub-chunk, tile, k step)
            const int ks = tk % KSC;
            const int t = (tk / KSC) & 3;
            const int s = tk / (4 * KSC);
            const int i = idx & 15;
            const int c = (sc0 + s) * 64 + chan_of<4>(t, i >> 2, i & 3);
            const int kw = 4 * ks + ((idx & 63) >> 4);
            const bool ok = idx < nfrag && kw < a.KW;
            const uint32_t v = a.wq[ok ? (long long)c * a.KW + kw : 0];
            word[q] = ok ? v : 0u;
        }
#pragma unroll
        for (int q = 0; q < U; ++q) {
            const int idx = base + q * 256 + tid;
            if (idx < nfrag) frag[idx] = decode_word(word[q]);
        }
    }
    for (int p = tid; p < nsc * 64; p += 256) {
        const int c = (sc0 + (p >> 6)) * 64 + chan_of<4>((p >> 4) & 3, (p >> 2) & 3, p & 3);
        lpar[p] = requant_params(a.bias[c], a.mult[c], PRELU ? a.mult_neg[c] : 0, a.shift[c], PRELU);
    }
    __syncthreads();
}

template <int KSC, int G, bool PRELU = false>
__device__ __forceinline__ void pw_expand_body(const PwArgs &a, const int lid, unsigned char *lds_raw)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15;
    const int g = lane >> 4;

    const int nparts = a.n_chunks;
    const int part = lid % nparts;
    const int wg = lid / nparts;
    if (wg >= a.wg_per_chunk) return;
    const int nsc_max = a.cw;
    const int sc0 = part * nsc_max;
    const int nsc = min(nsc_max, (a.Nc >> 6) - sc0);  // sub-chunks of this part (>= 1)
    const int K = a.K, Nc = a.Nc;

    v4i *frag = reinterpret_cast<v4i *>(lds_raw);  // [nsc][4 tiles][KSC][64 lanes]
    v4i *lpar = frag + nsc_max * 4 * KSC * 64;     // [nsc][4 tiles][4 g][4 r]
    unsigned char *stage = reinterpret_cast<unsigned char *>(lpar + nsc_max * 64) + wave * 1024;

    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a.x), 0, a.M * K, kBufFlags);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, a.M * Nc, kBufFlags);

    const int Wv = a.wg_per_chunk * 4;
    const int w0 = wg * 4 + wave;
    // Offsets are unsigned and saturate beyond the tensor, where loads read zero and stores are
    // dropped, so a unit past the end of the layer (or its ragged last tiles) needs no branch.
    unsigned xoff = min((unsigned)kOobOffset, (unsigned)(w0 * (16 * G) + j) * (unsigned)K + 16u * g);
    const unsigned xstep = (unsigned)Wv * (16 * G) * (unsigned)K;
    v4i B[G][KSC];
    // The whole offset sits in the vector operand (plus an immediate), which is what the range
    // check of a raw buffer covers.
    auto load_tile = [&](int gi) {
        const unsigned xo = min(xoff + (unsigned)((16 * gi) * K), (unsigned)kOobOffset);
#pragma unroll
        for (int k = 0; k < KSC; ++k)
            B[gi][k] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)(xo + 64u * k), 0, 0);
    };
#pragma unroll
    for (int gi = 0; gi < G; ++gi) load_tile(gi);
    xoff = min(xoff + xstep, (unsigned)kOobOffset);

    stage_part<KSC, PRELU>(a, sc0, nsc, frag, lpar);

    // any shift of the part equal to 0 -> the general form of the requantisation
    bool sh0 = false;
    if constexpr (!PRELU)
        for (int c = lane; c < nsc * 64; c += 64) sh0 |= lpar[c][3] == 0;
    const bool general_shift = __builtin_amdgcn_ballot_w64(sh0) != 0;

    const int lo = in_vgpr(a.lo), hi = in_vgpr(a.hi);
    // staged tile -> global: piece `lane` is bytes [16*(lane&3), +16) of pixel row lane>>2
    const unsigned goff = (unsigned)(lane >> 2) * (unsigned)Nc + 16u * (lane & 3);
    unsigned ytile = min((unsigned)kOobOffset, (unsigned)(w0 * (16 * G)) * (unsigned)Nc + (unsigned)(sc0 * 64));
    const unsigned ystep = (unsigned)Wv * (16 * G) * (unsigned)Nc;
    const int my_units = w0 < a.units ? (a.units - w0 + Wv - 1) / Wv : 0;
    const v4i zero4 = {0, 0, 0, 0};

    auto run = [&](auto mode_tag) {
        constexpr int MODE = decltype(mode_tag)::value;
        auto sub_chunk = [&](const int sc, auto last_tag) {
            constexpr bool LAST = decltype(last_tag)::value;
            v4i par[4][4];
            const v4i *lpg = lpar + sc * 64 + g * 4;
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    par[t][r] = lpg[t * 16 + r];
                    if constexpr (MODE == 0) par[t][r][3] -= 1;
                }
            const v4i *fk = frag + sc * 4 * KSC * 64 + lane;
#pragma unroll
            for (int gi = 0; gi < G; ++gi) {
                v4i acc[4];
#pragma unroll
                for (int k = 0; k < KSC; ++k) {
                    // opaque offset: with several k steps the fragment reads stay next to their
                    // MFMAs instead of being kept in 16*KSC registers across the pixel tiles
                    int fo = k * 64;
                    if constexpr (KSC > 1) asm volatile("" : "+v"(fo));
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        // PReLU: the biases are the accumulators' start value, so that the sign of
                        // an accumulator is the sign that selects the multiplier
                        v4i c0 = zero4;
                        if constexpr (MODE == 2) c0 = v4i{par[t][0][0], par[t][1][0], par[t][2][0], par[t][3][0]};
                        acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fk[t * KSC * 64 + fo], B[gi][k],
                                                                       k == 0 ? c0 : acc[t], 0, 0, 0);
                    }
                }
                if constexpr (LAST) load_tile(gi);  // this tile of the next unit
                uint32_t out[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    int v[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if constexpr (MODE == 2)
                            v[r] = requant_prelu_s(acc[t][r], par[t][r][1], par[t][r][2], par[t][r][3], lo, hi);
                        else
                            v[r] = requant_mode<MODE>(acc[t][r], par[t][r], lo, hi);
                    }
                    out[t] = pack4_low_bytes(v[0], v[1], v[2], v[3]);
                }
                // the lane's 16 channels of pixel j: tile t holds channels 16*g + 4*t + r
                // (16-byte columns swizzled by the row so that neither side has bank conflicts)
                *reinterpret_cast<v4i *>(stage + j * 64 + 16 * (g ^ (j >> 2))) =
                    v4i{(int)out[0], (int)out[1], (int)out[2], (int)out[3]};
                const v4i v = *reinterpret_cast<const v4i *>(stage + (lane >> 2) * 64 + 16 * ((lane & 3) ^ (lane >> 4)));
                const unsigned tile_off = ytile + (unsigned)((16 * gi) * Nc + sc * 64);
                // offset in the vector operand (see the streaming kernel's store)
                store_b128_guarded(v, ry, (int)min(goff + tile_off, (unsigned)kOobOffset));
            }
        };
        for (int u = 0; u < my_units; ++u) {
#pragma nounroll
            for (int sc = 0; sc + 1 < nsc; ++sc) sub_chunk(sc, std::false_type{});
            sub_chunk(nsc - 1, std::true_type{});
            xoff = min(xoff + xstep, (unsigned)kOobOffset);
            ytile = min(ytile + ystep, (unsigned)kOobOffset);
        }
    };
    if constexpr (PRELU)
        run(std::integral_constant<int, 2>{});
    else if (general_shift)
        run(std::integral_constant<int, 1>{});
    else
        run(std::integral_constant<int, 0>{});
}

// ============================================================================================
// The same walk over the output channels for wide rows of few input channels at high resolution
// (one k step, cout = nsc sub-chunks of 16*NTS channels, all of them in every workgroup): the
// outputs of a whole pixel unit (16*G pixels x Nc bytes, contiguous in NHWC) are assembled in the
// wavefront's own LDS area and leave as one contiguous run of 16-byte stores.  One wavefront does
// what the row-cooperative kernel spreads over the wavefronts of a workgroup, without its barriers.
//   XMODE 16: K % 16 == 0, one 16-byte load per lane; XMODE 8: K % 8 == 0, two 8-byte loads.
//   (16*G*Nc) % 16 == 0 always; no residual.
__host__ __device__ constexpr size_t lds_bytes_expand_rows(int nsc, int nts, int g, int nc)
{
    return (size_t)nsc * nts * (1024 + 256) + (size_t)4 * 16 * g * nc;
}

template <int G, int NTS, int XMODE, bool PRELU>
__device__ __forceinline__ void pw_expand_rows_body(const PwArgs &a, const int lid, unsigned char *lds_raw)
{
    static_assert(NTS == 3 || NTS == 4, "sub-chunks of 48 or 64 channels");
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15;
    const int g = lane >> 4;
    if (lid >= a.wg_per_chunk) return;
    const int K = a.K, Nc = a.Nc;
    const int nsc = Nc / (16 * NTS);

    v4i *frag = reinterpret_cast<v4i *>(lds_raw);  // [nsc][NTS][64 lanes]
    v4i *lpar = frag + nsc * NTS * 64;             // [nsc][NTS][4 g][4 r]
    unsigned char *stage = reinterpret_cast<unsigned char *>(lpar + nsc * NTS * 16) + wave * (16 * G * Nc);

    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a.x), 0, a.M * K, kBufFlags);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, a.M * Nc, kBufFlags);

    const int Wv = a.wg_per_chunk * 4;
    const int w0 = lid * 4 + wave;
    unsigned xoff = min((unsigned)kOobOffset, (unsigned)(w0 * (16 * G) + j) * (unsigned)K + 16u * g);
    const unsigned xstep = (unsigned)Wv * (16 * G) * (unsigned)K;
    v4i B[G];
    auto load_tile = [&](int gi) {
        const unsigned xo = min(xoff + (unsigned)((16 * gi) * K), (unsigned)kOobOffset);
        if constexpr (XMODE == 16) {
            B[gi] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)xo, 0, 0);
        } else {
            const v2i lo2 = __builtin_amdgcn_raw_buffer_load_b64(rx, (int)xo, 0, 0);
            const v2i hi2 = __builtin_amdgcn_raw_buffer_load_b64(rx, (int)(xo + 8u), 0, 0);
            B[gi] = v4i{lo2[0], lo2[1], hi2[0], hi2[1]};
        }
    };
#pragma unroll
    for (int gi = 0; gi < G; ++gi) load_tile(gi);
    xoff = min(xoff + xstep, (unsigned)kOobOffset);

    // ---- weights and parameters of all sub-chunks ------------------------------------------------
    {
        const int nfrag = nsc * NTS * 64;
        for (int idx = tid; idx < nfrag; idx += 256) {
            const int tk = idx >> 6;
            const int t = tk % NTS, sc = tk / NTS;
            const int i = idx & 15;
            const int c = sc * (16 * NTS) + chan_of<NTS>(t, i >> 2, i & 3);
            const int kw = (idx & 63) >> 4;
            frag[idx] = decode_word(kw < a.KW ? a.wq[(long long)c * a.KW + kw] : 0u);
        }
        for (int p = tid; p < nsc * NTS * 16; p += 256) {
            const int q = p % (NTS * 16);
            const int c = (p / (NTS * 16)) * (16 * NTS) + chan_of<NTS>(q >> 4, (q >> 2) & 3, q & 3);
            lpar[p] = requant_params(a.bias[c], a.mult[c], PRELU ? a.mult_neg[c] : 0, a.shift[c], PRELU);
        }
        __syncthreads();
    }
    bool sh0 = false;
    if constexpr (!PRELU)
        for (int c = lane; c < nsc * NTS * 16; c += 64) sh0 |= lpar[c][3] == 0;
    const bool general_shift = __builtin_amdgcn_ballot_w64(sh0) != 0;

    const int lo = in_vgpr(a.lo), hi = in_vgpr(a.hi);
    const int unit_bytes = 16 * G * Nc;
    unsigned yunit = min((unsigned)kOobOffset, (unsigned)w0 * (unsigned)unit_bytes);
    const unsigned ystep = (unsigned)Wv * (unsigned)unit_bytes;
    const int my_units = w0 < a.units ? (a.units - w0 + Wv - 1) / Wv : 0;
    const v4i zero4 = {0, 0, 0, 0};

    auto run = [&](auto mode_tag) {
        constexpr int MODE = decltype(mode_tag)::value;
        auto sub_chunk = [&](const int sc, auto last_tag) {
            constexpr bool LAST = decltype(last_tag)::value;
            v4i par[NTS][4];
            const v4i *lpg = lpar + sc * (NTS * 16) + g * 4;
#pragma unroll
            for (int t = 0; t < NTS; ++t)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    par[t][r] = lpg[t * 16 + r];
                    if constexpr (MODE == 0) par[t][r][3] -= 1;
                }
            v4i wf[NTS];
#pragma unroll
            for (int t = 0; t < NTS; ++t) wf[t] = frag[(sc * NTS + t) * 64 + lane];
#pragma unroll
            for (int gi = 0; gi < G; ++gi) {
                v4i acc[NTS];
#pragma unroll
                for (int t = 0; t < NTS; ++t) {
                    v4i c0 = zero4;
                    if constexpr (MODE == 2) c0 = v4i{par[t][0][0], par[t][1][0], par[t][2][0], par[t][3][0]};
                    acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[t], B[gi], c0, 0, 0, 0);
                }
                if constexpr (LAST) load_tile(gi);  // this tile of the next unit
                uint32_t out[NTS];
#pragma unroll
                for (int t = 0; t < NTS; ++t) {
                    int v[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if constexpr (MODE == 2)
                            v[r] = requant_prelu_s(acc[t][r], par[t][r][1], par[t][r][2], par[t][r][3], lo, hi);
                        else
                            v[r] = requant_mode<MODE>(acc[t][r], par[t][r], lo, hi);
                    }
                    out[t] = pack4_low_bytes(v[0], v[1], v[2], v[3]);
                }
                // pixel row (16*gi + j) of the unit, channels of this sub-chunk: the lane's tiles
                // are stored in groups of 4, 2, 1 (chan_of), each group contiguous
                unsigned char *sp = stage + (16 * gi + j) * Nc + sc * (16 * NTS);
                if constexpr (NTS == 4) {
                    *reinterpret_cast<v4i *>(sp + 16 * g) = v4i{(int)out[0], (int)out[1], (int)out[2], (int)out[3]};
                } else {
                    *reinterpret_cast<v2i *>(sp + 8 * g) = v2i{(int)out[0], (int)out[1]};
                    *reinterpret_cast<uint32_t *>(sp + 32 + 4 * g) = out[2];
                }
            }
        };
        for (int u = 0; u < my_units; ++u) {
#pragma nounroll
            for (int sc = 0; sc + 1 < nsc; ++sc) sub_chunk(sc, std::false_type{});
            sub_chunk(nsc - 1, std::true_type{});
            // the unit's 16*G*Nc bytes, in 16-byte pieces in memory order
            for (int p = lane; p < unit_bytes / 16; p += 64) {
                const v4i v = *reinterpret_cast<const v4i *>(stage + 16 * p);
                store_b128_guarded(v, ry, (int)min(yunit + 16u * p, (unsigned)kOobOffset));
            }
            xoff = min(xoff + xstep, (unsigned)kOobOffset);
            yunit = min(yunit + ystep, (unsigned)kOobOffset);
        }
    };
    if constexpr (PRELU)
        run(std::integral_constant<int, 2>{});
    else if (general_shift)
        run(std::integral_constant<int, 1>{});
    else
        run(std::integral_constant<int, 0>{});
}

}  // namespace prom
