// Ternary pointwise layer whose int8 output takes the paper's dynamic activation scale (Section 3.1,
// Eq. 6-7: one absmax scale per batch element over all its channels and pixels), fused: the
// real-valued output is never written.  The scale of an image is known only when all of its outputs
// are, and an image's outputs (hundreds of kilobytes) fit in no on-chip memory, so the layer is
// computed twice from its int8 input:
//   pass 1   accumulators -> real values -> per-image maximum of |z| (registers, one atomic
//            maximum per wavefront and image), nothing else is written;
//   pass 2   the same accumulators and real values again -> codes with the final scale -> int8.
// Against the unfused form (layer -> float32 tensor -> maximum -> codes: 13 bytes per output) this
// moves 2 K / N + 1 bytes per output (K, N input and output channels).
//
// The matrix part is the transposed MFMA formulation of the other pointwise kernels: decoded
// weights of a chunk of 16*NT output channels in LDS as A operands, activations of 16 pixels as B
// operands straight from their NHWC rows, v_mfma_i32_16x16x64_i8.  A wavefront owns a contiguous
// range of 16-pixel tiles, so that it changes image rarely.
#include "prom_pw_stream.h"
#include "prom_launch.h"

namespace prom {

struct DynqArgs {
    const int8_t *x;
    const uint32_t *wq;
    const float *x_step;   // [n]
    const float *w_scale;  // [Nc]
    const float *bias;     // [Nc] or nullptr
    int8_t *q;
    uint32_t *amax_bits;   // [n] float bits of the per-image maximum (non-negative floats order as integers)
    float *scale;          // [n]
    float eps;
    int M, HW, n_img;
    int K, Nc, KW, KS;
    int relu;
    int n_chunks, wg_per_chunk;
    int tiles_per_wave;    // 16-pixel tiles in a wavefront's contiguous range
};

__global__ __launch_bounds__(256) void dynq_clear_kernel(uint32_t *amax_bits, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) amax_bits[i] = 0u;
}

// Channel (relative to the chunk) of D row i = 4*gr + r of tile t of a chunk of NT tiles: whole
// groups of four tiles are interleaved so that the four tiles' rows of one lane are 16 consecutive
// channels (one 16-byte store); the one to three tiles behind them keep their own 16 channels
// (4-byte stores).
template <int NT>
__device__ __forceinline__ int dynq_chan(int t, int i)
{
    return t < (NT & ~3) ? 16 * (t & ~3) + 16 * (i >> 2) + 4 * (t & 3) + (i & 3) : 16 * t + i;
}
constexpr int kDynqSlots = 32;  // images whose maxima a workgroup combines in LDS

// real value of an accumulator: three float32 operations, each rounded once, in this order.  (The
// compiler's default for device code fuses a product with a following sum into one operation with
// a single rounding, also through __fmul_rn and __fadd_rn; the pragma takes that licence away.)
__device__ __forceinline__ float dynq_real(int acc, float ws, float xs, float b, bool relu)
{
#pragma clang fp contract(off)
    const float t = (float)acc * ws;
    const float u = t * xs;
    float z = u + b;
    if (relu) z = fmaxf(z, 0.0f);
    return z;
}

template <int NT, int PASS>
__global__ __launch_bounds__(256, 2) void pw_dynq_kernel(const DynqArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int KS = a.KS, K = a.K, Nc = a.Nc;
    v4i *frag = reinterpret_cast<v4i *>(lds_raw);                                   // [NT][KS][64]
    float *lws = reinterpret_cast<float *>(lds_raw + (size_t)NT * KS * 1024);        // [NT][16]
    float *lbias = lws + NT * 16;                                                    // [NT][16]
    uint32_t *limg = reinterpret_cast<uint32_t *>(lbias + NT * 16);                  // [kDynqSlots], pass 1
    const int chunk = blockIdx.x / a.wg_per_chunk, wg = blockIdx.x - chunk * a.wg_per_chunk;
    const int cbase = chunk * 16 * NT;

    if (PASS == 2 && blockIdx.x == 0)
        for (int i = tid; i < a.n_img; i += 256)
            a.scale[i] = 127.0f / fmaxf(__uint_as_float(a.amax_bits[i]), a.eps);

    // ---- the chunk's decoded weights and per-channel factors into LDS -------------------------
    {
        const int total = NT * KS * 64;
        constexpr int U = 8;
        for (int e0 = 0; e0 < total; e0 += 256 * U) {
            uint32_t wv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int e = e0 + 256 * u + tid;
                const int l = e & 63, tk = e >> 6;  // entry (t, ks) = tk, lane l of the operand
                const int t = tk / KS, ks = tk - t * KS;
                const int c = cbase + dynq_chan<NT>(t, l & 15);
                const int word = 4 * ks + (l >> 4);
                const bool ok = e < total && c < Nc && word < a.KW;
                // (unconditional loads from an address that is always valid: a load under a branch
                // costs a wait for everything in flight)
                const uint32_t v = a.wq[ok ? (long long)c * a.KW + word : 0];
                wv[u] = ok ? v : 0u;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int e = e0 + 256 * u + tid;
                if (e < total) frag[e] = decode_word(wv[u]);
            }
        }
        if (PASS == 1 && tid < kDynqSlots) limg[tid] = 0u;
        if (tid < NT * 16) {
            const int c = cbase + dynq_chan<NT>(tid >> 4, tid & 15);
            const float wsc = a.w_scale[c < Nc ? c : 0];
            const float bsc = a.bias ? a.bias[c < Nc ? c : 0] : 0.0f;
            lws[tid] = c < Nc ? wsc : 0.0f;
            lbias[tid] = c < Nc ? bsc : 0.0f;
        }
    }
    __syncthreads();

    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<int8_t *>(a.x), 0, a.M * K, kBufFlags);
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(a.q, 0, a.M * Nc, kBufFlags);
    const int col = lane & 15, gr = lane >> 4;
    const bool relu = a.relu != 0;
    const int n_tiles = (a.M + 15) >> 4;
    const int w_id = wg * 4 + wave;
    const int tile_lo = min(w_id * a.tiles_per_wave, n_tiles);
    const int tile_hi = min(tile_lo + a.tiles_per_wave, n_tiles);

    // Pass 1 keeps, per lane and channel, the smallest and the largest accumulator of the image the
    // lane is in.  The real value is a non-decreasing or non-increasing function of the accumulator
    // (a float32 product with a fixed factor and a float32 sum with a fixed term are monotonic, so
    // is max(., 0)), hence the largest |z| of a channel in an image is |z| of one of these two, and
    // the float32 arithmetic runs once per image and channel instead of once per output.
    const int img_base = (int)(((long long)wg * 4 * a.tiles_per_wave * 16) / a.HW);  // first image of the workgroup's pixels
    int cur_img = -1;     // the image the lane's extremes belong to
    float cur_xs = 0.0f;  // its input step
    v4i acc_lo[PASS == 1 ? NT : 1], acc_hi[PASS == 1 ? NT : 1];
    // Hands the extremes of the lanes in `leaving` to their images.
    auto flush = [&](const bool leaving) __attribute__((always_inline)) {
        float run_max = 0.0f;
        if constexpr (PASS == 1) {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const float4 ws = *reinterpret_cast<const float4 *>(&lws[t * 16 + 4 * gr]);
                const float4 bs = *reinterpret_cast<const float4 *>(&lbias[t * 16 + 4 * gr]);
                const float wsv[4] = {ws.x, ws.y, ws.z, ws.w}, bsv[4] = {bs.x, bs.y, bs.z, bs.w};
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    // (channels beyond the layer's have zero weights, factors and terms: z = 0)
                    const float z0 = dynq_real(acc_lo[t][r], wsv[r], cur_xs, bsv[r], a.relu != 0);
                    const float z1 = dynq_real(acc_hi[t][r], wsv[r], cur_xs, bsv[r], a.relu != 0);
                    run_max = fmaxf(run_max, fmaxf(fabsf(z0), fabsf(z1)));
                }
            }
        }
        // Combined per workgroup in LDS first: atomics of many workgroups on one address in memory
        // take about 0.1 to 0.7 us each, one after the other (measured: 22 of 44 us at 56x56 with
        // one per wavefront, 90 of 100 us at 7x7, where every tile spans two images).
        if (leaving && cur_img >= 0) {
            const int slot = cur_img - img_base;
            if (slot < kDynqSlots)
                atomicMax(&limg[slot], __float_as_uint(run_max));
            else
                atomicMax(&a.amax_bits[cur_img], __float_as_uint(run_max));
        }
    };

    // the loads of KU k steps are issued together; other wavefronts cover their latency
    // What a tile needs from global memory -- the first KU k steps of its activations, its image's
    // input step and (pass 2) its image's maximum -- is fetched one tile ahead, so that these
    // latencies overlap with the matrix instructions and the epilogue of the tile before.
    constexpr int KU = 4;
    struct TileIn {
        v4i b[KU];
        float xs, am;
        int img;
    };
    auto fetch = [&](const int tile, TileIn &in) __attribute__((always_inline)) {
        const int p = tile * 16 + col;
        const bool valid = tile < tile_hi && p < a.M;
        const unsigned xrow = valid ? (unsigned)p * (unsigned)K + 16u * gr : (unsigned)kOobOffset;
#pragma unroll
        for (int u = 0; u < KU; ++u)
            // (a k step beyond KS reads the next pixels' bytes or zeros; its weights are not used)
            in.b[u] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)min(xrow + 64u * u, (unsigned)kOobOffset), 0, 0);
        const int img_raw = p / a.HW;  // (unconditional division and loads: see the weights above)
        in.img = valid ? img_raw : -1;
        const int ic = valid ? img_raw : 0;
        in.xs = a.x_step[ic];
        in.am = PASS == 2 ? __uint_as_float(a.amax_bits[ic]) : 0.0f;
    };
    auto process = [&](const int tile, const TileIn &cur) __attribute__((always_inline)) {
        const int p = tile * 16 + col;
        const bool valid = p < a.M;
        // (the per-channel factors are re-read from LDS for every tile, at an offset the optimiser
        // cannot see through: hoisted out of the loop they would cost 8 registers per channel tile
        // and with them half of the resident wavefronts)
        // (an opaque offset, not an opaque pointer: the pointer would lose its address space and the
        // reads would become flat loads, which wait for every store in flight)
        int opaque_zero = 0;
        asm volatile("" : "+v"(opaque_zero));
        const float *lws_t = lws + opaque_zero, *lbias_t = lbias + opaque_zero;
        v4i acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[t] = v4i{0, 0, 0, 0};
#pragma unroll
        for (int u = 0; u < KU; ++u) {
            if (u < KS) {
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(frag[(t * KS + u) * 64 + lane], cur.b[u], acc[t], 0, 0, 0);
            }
        }
        // the k steps beyond the prefetched ones (more than 256 input channels)
        const unsigned xrow = min((unsigned)p * (unsigned)K + 16u * gr, (unsigned)kOobOffset);
        for (int k0 = KU; k0 < KS; k0 += KU) {
            v4i b[KU];
#pragma unroll
            for (int u = 0; u < KU; ++u)
                b[u] = __builtin_amdgcn_raw_buffer_load_b128(rx, (int)min(xrow + 64u * (k0 + u), (unsigned)kOobOffset), 0, 0);
#pragma unroll
            for (int u = 0; u < KU; ++u) {
                if (k0 + u < KS) {
#pragma unroll
                    for (int t = 0; t < NT; ++t)
                        acc[t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(frag[(t * KS + k0 + u) * 64 + lane], b[u], acc[t], 0, 0, 0);
                }
            }
        }
        // ---- epilogue: lane (col, gr) holds channels cbase + 64*(t/4) + 16*gr + 4*(t%4) + r of pixel p
        const int img = cur.img;
        const float xs = cur.xs;
        if constexpr (PASS == 1) {
            const bool change = img != cur_img;
            if (__any(change)) {  // (wave-uniform: the loop bounds are, so all 64 lanes are here)
                if (__any(change && cur_img >= 0)) flush(change);
                if (change) {
                    cur_img = img;
                    cur_xs = xs;
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        acc_lo[t] = v4i{0x7fffffff, 0x7fffffff, 0x7fffffff, 0x7fffffff};
                        acc_hi[t] = -acc_lo[t];
                    }
                }
            }
            if (valid) {
#pragma unroll
                for (int t = 0; t < NT; ++t) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        acc_lo[t][r] = min(acc_lo[t][r], acc[t][r]);
                        acc_hi[t][r] = max(acc_hi[t][r], acc[t][r]);
                    }
                }
            }
        } else {
            const float s = valid ? 127.0f / fmaxf(cur.am, a.eps) : 0.0f;
            auto codes = [&](const int t) __attribute__((always_inline)) {
                const float4 ws = *reinterpret_cast<const float4 *>(&lws_t[t * 16 + 4 * gr]);
                const float4 bs = *reinterpret_cast<const float4 *>(&lbias_t[t * 16 + 4 * gr]);
                const float wsv[4] = {ws.x, ws.y, ws.z, ws.w}, bsv[4] = {bs.x, bs.y, bs.z, bs.w};
                int v[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float z = dynq_real(acc[t][r], wsv[r], xs, bsv[r], relu);
                    const float c = rintf(__fmul_rn(z, s));
                    v[r] = (int)fminf(fmaxf(c, -128.0f), 127.0f);
                }
                return (int)pack4_low_bytes(v[0], v[1], v[2], v[3]);
            };
            constexpr int NT4 = NT & ~3;
#pragma unroll
            for (int t0 = 0; t0 < NT4; t0 += 4) {
                v4i out;
#pragma unroll
                for (int tt = 0; tt < 4; ++tt) out[tt] = codes(t0 + tt);
                const int c0 = cbase + 16 * t0 + 16 * gr;  // the lane's 16 consecutive channels
                const unsigned off = (valid && c0 < Nc) ? (unsigned)p * (unsigned)Nc + (unsigned)c0 : (unsigned)kOobOffset;
                store_b128_guarded(out, rq, (int)min(off, (unsigned)kOobOffset));
            }
#pragma unroll
            for (int t = NT4; t < NT; ++t) {
                const int out = codes(t);
                const int c0 = cbase + 16 * t + 4 * gr;  // the lane's 4 consecutive channels
                const unsigned off = (valid && c0 < Nc) ? (unsigned)p * (unsigned)Nc + (unsigned)c0 : (unsigned)kOobOffset;
                __builtin_amdgcn_raw_buffer_store_b32(out, rq, (int)min(off, (unsigned)kOobOffset), 0, 0);
            }
        }
    };
    // Two buffers that alternate by name (no register copies: a copy of a prefetched value would
    // wait for its load on the spot).
    TileIn in0, in1;
    fetch(tile_lo, in0);
    for (int tile = tile_lo; tile < tile_hi; tile += 2) {
        fetch(tile + 1, in1);
        process(tile, in0);
        fetch(tile + 2, in0);
        if (tile + 1 < tile_hi) process(tile + 1, in1);
    }
    if constexpr (PASS == 1) {
        if (__any(cur_img >= 0)) flush(true);
        __syncthreads();
        if (tid < kDynqSlots && img_base + tid < a.n_img) {
            const uint32_t v = limg[tid];
            if (v != 0u) atomicMax(&a.amax_bits[img_base + tid], v);
        }
    }
}

template <int NT>
static int launch_dynq(const DynqArgs &a1, int grid1, const DynqArgs &a, int grid, size_t lds, hipStream_t st)
{
    const auto k1 = pw_dynq_kernel<NT, 1>;
    const auto k2 = pw_dynq_kernel<NT, 2>;
    if (lds > 48 * 1024) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(k1), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(k2), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
            last_hip_error() = hipGetLastError();
            return PROM_EHIP;
        }
    }
    clear_hip_error();
    hipLaunchKernelGGL(dynq_clear_kernel, dim3((unsigned)((a.n_img + 255) / 256)), dim3(256), 0, st, a.amax_bits, a.n_img);
    hipLaunchKernelGGL(k1, dim3((unsigned)grid1), dim3(256), lds, st, a1);
    hipLaunchKernelGGL(k2, dim3((unsigned)grid), dim3(256), lds, st, a);
    return check_launch();
}

}  // namespace prom

extern "C" int prom_pw_conv_dynq(const int8_t *x, int n, int h, int w, int cin, const void *w_packed, int cout,
                                 const float *x_step, const float *w_scale, const float *bias, int relu, float eps,
                                 int8_t *q, float *amax, float *scale, void *stream)
{
    using namespace prom;
    if (!x || !w_packed || !x_step || !w_scale || !q || !amax || !scale) return PROM_EINVAL;
    if (n <= 0 || h <= 0 || w <= 0 || cin <= 0 || cout <= 0 || !(eps > 0.0f)) return PROM_EINVAL;
    if ((((uintptr_t)w_packed | (uintptr_t)x_step | (uintptr_t)w_scale | (uintptr_t)bias | (uintptr_t)amax |
          (uintptr_t)scale) & 3) != 0)
        return PROM_EINVAL;
    if ((((uintptr_t)x | (uintptr_t)q) & 15) != 0) return PROM_EINVAL;
    if (cin % 4 != 0 || cout % 16 != 0 || cin > 1024) return PROM_EUNSUPPORTED;  // dword-aligned rows, whole 16-byte stores
    const long long M = (long long)n * h * w;
    if ((M + 64) * (long long)(cin > cout ? cin : cout) >= (long long)kOobOffset) return PROM_EUNSUPPORTED;
    DynqArgs a;
    a.x = x;
    a.wq = static_cast<const uint32_t *>(w_packed);
    a.x_step = x_step;
    a.w_scale = w_scale;
    a.bias = bias;
    a.q = q;
    a.amax_bits = reinterpret_cast<uint32_t *>(amax);
    a.scale = scale;
    a.eps = eps;
    a.M = (int)M;
    a.HW = h * w;
    a.n_img = n;
    a.K = cin;
    a.Nc = cout;
    a.KW = (cin + 15) / 16;
    a.KS = (cin + 63) / 64;
    a.relu = relu != 0;
    // chunk width: as few chunks as 12 tiles per chunk and 64 KB of decoded weights allow, then the
    // narrowest width that still gives that many chunks
    const int n_tiles_c = cout / 16;
    int nt_max = 64 / a.KS;  // >= 4 since KS <= 16
    if (nt_max > 12) nt_max = 12;
    a.n_chunks = (n_tiles_c + nt_max - 1) / nt_max;
    const int nt = (n_tiles_c + a.n_chunks - 1) / a.n_chunks;
    const size_t lds = (size_t)nt * a.KS * 1024 + 2 * nt * 16 * sizeof(float) + kDynqSlots * sizeof(uint32_t);
    // Pass 1 (many registers: two wavefronts per SIMD) runs as one resident round of about two
    // workgroups per CU, pass 2 with about four; at least 2 pixel tiles per wavefront.
    const int n_ptiles = (int)((M + 15) / 16);
    auto size_pass = [&](DynqArgs &p, const int target) {
        long long wgs = target / p.n_chunks;
        if (wgs < 1) wgs = 1;
        const long long max_wgs = (n_ptiles + 4 * 2 - 1) / (4 * 2);
        if (wgs > max_wgs) wgs = max_wgs;
        p.wg_per_chunk = (int)wgs;
        p.tiles_per_wave = (int)((n_ptiles + 4 * wgs - 1) / (4 * wgs));
        return (int)(wgs * p.n_chunks);
    };
    DynqArgs a1 = a;
    const int grid1 = size_pass(a1, 512), grid = size_pass(a, 1024);
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (nt) {
    case 1: return launch_dynq<1>(a1, grid1, a, grid, lds, st);
    case 2: return launch_dynq<2>(a1, grid1, a, grid, lds, st);
    case 3: return launch_dynq<3>(a1, grid1, a, grid, lds, st);
    case 4: return launch_dynq<4>(a1, grid1, a, grid, lds, st);
    case 5: return launch_dynq<5>(a1, grid1, a, grid, lds, st);
    case 6: return launch_dynq<6>(a1, grid1, a, grid, lds, st);
    case 7: return launch_dynq<7>(a1, grid1, a, grid, lds, st);
    case 8: return launch_dynq<8>(a1, grid1, a, grid, lds, st);
    case 9: return launch_dynq<9>(a1, grid1, a, grid, lds, st);
    case 10: return launch_dynq<10>(a1, grid1, a, grid, lds, st);
    case 11: return launch_dynq<11>(a1, grid1, a, grid, lds, st);
    default: return launch_dynq<12>(a1, grid1, a, grid, lds, st);
    }
}
