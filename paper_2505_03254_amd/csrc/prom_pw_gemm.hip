// Ternary pointwise convolution for wide layers (hundreds to thousands of input AND output
// channels: the 1x1 layers of the deeper stages of ResNeXt / RegNet, paper Section 5): the k loop is
// outermost over a workgroup tile of 128 output channels x 256 pixels.
//
// The streaming kernel (prom_pw_stream.h) keeps the decoded weights of a chunk of output channels
// for ALL input channels in LDS and streams the pixels past them once per chunk; with 16 to 32 k
// steps a chunk is two to four 16-channel tiles, so a layer with 2048 output channels reads its
// activations 32 to 64 times and a wavefront issues two to four MFMAs per 16-byte activation load.
// Such layers are bound by the matrix cores (arithmetic intensity above 625 op/B), and this kernel is
// shaped for that:
//   - a wavefront owns 8 channel tiles x 4 pixel tiles (32 accumulator tiles, 128 registers): 32
//     MFMAs per k step against 8 LDS reads of 16 bytes (the decoded weights, shared by the four
//     wavefronts) and 4 global loads of 16 bytes (its own pixels, straight into the B operand);
//   - the 128 x 64 ternary codes of the next k step (2 KB packed) are fetched one step ahead, decoded
//     by all 256 threads into the other of two 8 KB LDS slabs while the matrix cores work on this
//     step; one barrier per k step;
//   - the pixels of the next k step are fetched one step ahead into the other of two register sets;
//   - workgroups that share a pixel tile (the layer's 128-channel column tiles) are neighbours in
//     the XCD-aware order, so the activations are fetched from HBM once and from that XCD's L2 by the
//     others;
//   - epilogue as in the streaming kernel: 64-bit multiply-add requantisation per output, the
//     wavefront's 64 pixels x 128 channels staged through LDS and written as whole 128-byte rows.
#include "prom_pw_stream.h"
#include "prom_pw_gemm.h"

namespace prom {

constexpr int kGemmTN = 128;  // output channels per workgroup
constexpr int kGemmTM = 256;  // pixels per workgroup
constexpr int kGemmStageStride = 144;  // bytes between pixels of the output staging tile (128 + 16)

// Workgroup barrier that orders LDS traffic only.  __syncthreads() carries a release fence over
// every address space, which makes the compiler wait for ALL outstanding global loads -- here the
// pixels and codes requested for three k steps ahead.  The wavefront's LDS writes are complete when
// lgkmcnt reaches 0 (LDS operations of a wavefront finish in order).
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

#ifdef PROM_TIMELINE
__device__ unsigned long long g_gemm_stamps[1024 * 4];
#define GEMM_STAMP(i) do { if (threadIdx.x == 0 && blockIdx.x < 1024) g_gemm_stamps[blockIdx.x * 4 + (i)] = wall_clock64(); } while (0)
#else
#define GEMM_STAMP(i) do { } while (0)
#endif

size_t pw_gemm_lds_bytes()
{
    // two slabs of decoded weights, parameters of 128 channels, staging of 4 x 64 pixels
    return 2 * 8192 + 128 * 16 + 4 * 64 * kGemmStageStride;
}

// a.n_chunks = column tiles of 128 channels, a.wg_per_chunk = row tiles of 256 pixels; requires
// K % 64 == 0, Nc % 16 == 0, 16-byte aligned x, y, residual and 8-byte aligned packed weights.
template <bool PRELU>
__global__ __launch_bounds__(256, 1) void pw_gemm_kernel(const PwArgs a)
{
    extern __shared__ __align__(16) unsigned char lds[];
    v4i *frag = reinterpret_cast<v4i *>(lds);                     // [2][8 tiles][64 lanes]
    v4i *lpar = reinterpret_cast<v4i *>(lds + 2 * 8192);          // [128]
    unsigned char *stage_all = lds + 2 * 8192 + 128 * 16;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 15, g = lane >> 4;

    GEMM_STAMP(0);
    const int lid = logical_block_id();
    const int ntile = lid % a.n_chunks;
    const int mtile = lid / a.n_chunks;
    if (mtile >= a.wg_per_chunk) return;
    const int n0 = ntile * kGemmTN;
    const int m0 = mtile * kGemmTM + wave * 64;  // this wavefront's first pixel
    const int K = a.K, Nc = a.Nc, KW = a.KW, KS = a.KS;

    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a.x), 0, a.M * K, kBufFlags);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, a.M * Nc, kBufFlags);
    const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int8_t *>(a.residual ? a.residual : a.y), 0, a.M * Nc, kBufFlags);

    // activation offsets of the lane's pixel in each of the 4 pixel tiles (saturated beyond the tensor)
    unsigned xoff[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const long long o = (long long)(m0 + 16 * i + j) * K + 16 * g;
        xoff[i] = o < (long long)kOobOffset ? (unsigned)o : (unsigned)kOobOffset;
    }
    // weight staging: thread -> row tid >> 1 of the tile, words 4ks + 2*(tid & 1) + {0, 1}
    const int wr = tid >> 1, wh = tid & 1;
    const bool wrow_ok = n0 + wr < Nc;
    const uint32_t *wsrc = a.wq + (long long)(wrow_ok ? n0 + wr : 0) * KW + 2 * wh;
    v4i *wdst = frag + (wr >> 4) * 64 + (2 * wh) * 16 + (wr & 15);  // + slab * 512, and + 16 for the second word

    auto load_x = [&](int ks, v4i(&b)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            b[i] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)min(xoff[i] + (unsigned)(64 * ks), (unsigned)kOobOffset), 0, 0);
    };
    auto load_w = [&](int ks) __attribute__((always_inline)) {
        return *reinterpret_cast<const v2i *>(wsrc + 4 * ks);
    };
    // (rows beyond the layer are zeroed here, at the use, not at the load: a select right behind the
    // load would wait for it, and with it for every load issued before)
    auto put_w = [&](int slab, v2i w, bool real) __attribute__((always_inline)) {
        const bool ok = wrow_ok && real;
        wdst[slab * 512] = decode_word(ok ? (uint32_t)w[0] : 0u);
        wdst[slab * 512 + 16] = decode_word(ok ? (uint32_t)w[1] : 0u);
    };

    v4i acc[8][4];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[t][i] = v4i{0, 0, 0, 0};

    // Rings of three k steps: the pixels and the packed codes of step ks + 2 are requested when step
    // ks starts (a k step is about 0.25 us; a request that misses the L2 takes longer, one that hits
    // it less).
    v4i bx[3][4];
    v2i wq[3];
#pragma unroll
    for (int d = 0; d < 2; ++d) {
        const int kd = min(d, KS - 1);
        load_x(kd, bx[d]);
        wq[d] = load_w(kd);
    }
    if (tid < kGemmTN) {
        const int c = n0 + tid;
        v4i p = {0, 0, 0, 1};
        if (c < Nc) p = requant_params(a.bias[c], a.mult[c], PRELU ? a.mult_neg[c] : 0, a.shift[c], PRELU);
        lpar[tid] = p;
    }
    put_w(0, wq[0], true);
    __syncthreads();
    GEMM_STAMP(1);

    // one k step: the matrix cores on slab ks & 1 and the pixels of ring slot ks % 3; the codes of
    // the next step are decoded into the other slab behind the MFMAs; one barrier.  All eight weight
    // fragments of the step are read from LDS before the first MFMA: with one wavefront per SIMD
    // nothing else hides an LDS latency, and read pair by pair they cost four of them per step.  Six
    // steps per iteration in straight-line code (a step beyond the last one runs on zero weights:
    // branches inside the body make the compiler wait for the newest load instead of the one it needs).
    for (int ks0 = 0; ks0 < KS; ks0 += 6) {
#pragma unroll
        for (int d = 0; d < 6; ++d) {
            const int ks = ks0 + d;
            const int kf = min(ks + 2, KS - 1);
            load_x(kf, bx[(d + 2) % 3]);
            wq[(d + 2) % 3] = load_w(kf);
            const v4i *fr = frag + (d & 1) * 512 + lane;
            v4i A[8];
            __builtin_amdgcn_sched_barrier(0);  // (the scheduler would sink the reads to their uses)
#pragma unroll
            for (int t = 0; t < 8; ++t) A[t] = fr[t * 64];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    acc[t][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[t], bx[d % 3][i], acc[t][i], 0, 0, 0);
            }
            put_w((d + 1) & 1, wq[(d + 1) % 3], ks + 1 < KS);
            lds_barrier();
        }
    }

    GEMM_STAMP(2);
    // ---- epilogue: requantise, skip, stage the wavefront's 64 x 128 tile, write whole rows ------------
    const int lo = in_vgpr(a.lo), hi = in_vgpr(a.hi);
    const int m128 = in_vgpr(-128), p127 = in_vgpr(127);
    const bool has_res = a.residual != nullptr;
    unsigned char *stage = stage_all + wave * (64 * kGemmStageStride);
    // residual dwords of the lane's (pixel, 4 channels) of tile t, one tile ahead
    auto load_res = [&](int t, uint32_t(&r)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const long long o = (long long)(m0 + 16 * i + j) * Nc + n0 + 16 * t + 4 * g;
            const bool ok = n0 + 16 * t + 4 * g < Nc && o < (long long)kOobOffset;
            r[i] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(rr, ok ? (int)o : kOobOffset, 0, 0);
        }
    };
    uint32_t res[4] = {0, 0, 0, 0}, resn[4] = {0, 0, 0, 0};
    if (has_res) load_res(0, res);
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        if (has_res && t + 1 < 8) load_res(t + 1, resn);
        v4i par[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) par[r] = lpar[16 * t + 4 * g + r];
        auto tile = [&](auto mode) __attribute__((always_inline)) {
            constexpr int MODE = decltype(mode)::value;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = requant_mode<MODE>(acc[t][i][r], par[r], lo, hi);
                if (has_res) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = med3_i32(v[r] + sbyte(res[i], r), m128, p127);
                }
                *reinterpret_cast<uint32_t *>(stage + (16 * i + j) * kGemmStageStride + 16 * t + 4 * g) =
                    pack4_low_bytes(v[0], v[1], v[2], v[3]);
            }
        };
        if constexpr (PRELU) {
            tile(std::integral_constant<int, 2>{});
        } else {
            const bool shift0 = par[0][3] == 0 || par[1][3] == 0 || par[2][3] == 0 || par[3][3] == 0;
            if (__builtin_amdgcn_ballot_w64(shift0) == 0) {
#pragma unroll
                for (int r = 0; r < 4; ++r) par[r][3] -= 1;
                tile(std::integral_constant<int, 0>{});
            } else {
                tile(std::integral_constant<int, 1>{});
            }
        }
        if (has_res) {
#pragma unroll
            for (int i = 0; i < 4; ++i) res[i] = resn[i];
        }
    }
    // (a wavefront reads back only what it wrote itself: no barrier)
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int piece = lane + 64 * q;
        const int px = piece >> 3, c16 = piece & 7;
        const v4i v = *reinterpret_cast<const v4i *>(stage + px * kGemmStageStride + 16 * c16);
        const long long o = (long long)(m0 + px) * Nc + n0 + 16 * c16;
        const bool ok = n0 + 16 * c16 < Nc && o < (long long)kOobOffset;
        store_b128_guarded(v, ry, ok ? (int)o : kOobOffset);
    }
    GEMM_STAMP(3);
}

PwKernelFn pw_gemm_select(bool prelu)
{
    return prelu ? &pw_gemm_kernel<true> : &pw_gemm_kernel<false>;
}

}  // namespace prom

#ifdef PROM_TIMELINE
extern "C" int prom_debug_gemm_stamps(unsigned long long *host)
{
    if (hipDeviceSynchronize() != hipSuccess) return PROM_EHIP;
    return hipMemcpyFromSymbol(host, HIP_SYMBOL(prom::g_gemm_stamps), sizeof(unsigned long long) * 1024 * 4) == hipSuccess ? PROM_OK : PROM_EHIP;
}
#endif
