// Weight preparation on the device: float32 weights -> what the convolution kernels take.
//   pointwise: channel-wise absmean ternary quantisation (paper Section 3.1, Eq. 1-3; its
//              pseudocode of the weight quantisation clamps the mean at eps, taken here) straight
//              into the 2-bit packed layout of prom_pack_ternary;
//   depthwise: channel-wise absmax 8-bit quantisation (Eq. 4-5 with the factor 127 of the
//              pseudocode) into the [3][3][C] layout of prom_dw_conv.
// A quantised code is decided by one float32 product, as in the paper's float32 code:
//   mean  = float32( sum_j |w[j]| in float64 / cin )
//   scale = 1.0f / max(mean, eps)          (one correctly rounded division; 127.0f / ... for absmax)
//   code  = clamp(rint(w * scale))         (float32 product, round half to even)
// One wavefront per output channel; a lane owns whole 16-weight words of the packed row.
// Also here: the paper's activation quantiser (one absmax scale per batch element).
#include "prom.h"
#include "prom_launch.h"

#include <hip/hip_runtime.h>

namespace prom {

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__global__ __launch_bounds__(256) void quant_pw_kernel(const float *__restrict__ w, int cout, int cin, float eps,
                                                       uint32_t *__restrict__ packed, int8_t *__restrict__ codes,
                                                       float *__restrict__ scale_out)
{
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (row >= cout) return;
    const float *wr = w + (size_t)row * cin;
    const int kw = (cin + 15) / 16;
    double s = 0.0;
    for (int j = lane; j < kw; j += 64)
        for (int e = 0; e < 16; ++e) {
            const int k = 16 * j + e;
            if (k < cin) s += (double)fabsf(wr[k]);
        }
    s = wave_sum(s);
    const float mean = (float)(s / (double)cin);
    const float scale = __fdiv_rn(1.0f, fmaxf(mean, eps));
    if (lane == 0) scale_out[row] = scale;
    for (int j = lane; j < kw; j += 64) {
        uint32_t word = 0;
        for (int e = 0; e < 16; ++e) {
            const int k = 16 * j + e;
            if (k >= cin) break;
            float q = rintf(__fmul_rn(wr[k], scale));
            q = fminf(fmaxf(q, -1.0f), 1.0f);
            const int c = (int)q;
            if (codes) codes[(size_t)row * cin + k] = (int8_t)c;
            word |= ((uint32_t)c & 3u) << (8 * (e & 3) + 2 * (e >> 2));
        }
        packed[(size_t)row * kw + j] = word;
    }
}

// one thread per channel: 9 weights
__global__ __launch_bounds__(256) void quant_dw_kernel(const float *__restrict__ w, int c, float eps,
                                                       int8_t *__restrict__ wq, float *__restrict__ scale_out)
{
    const int ch = blockIdx.x * 256 + threadIdx.x;
    if (ch >= c) return;
    float v[9];
    float amax = 0.0f;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        v[t] = w[(size_t)ch * 9 + t];
        amax = fmaxf(amax, fabsf(v[t]));
    }
    const float scale = __fdiv_rn(127.0f, fmaxf(amax, eps));
    scale_out[ch] = scale;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        float q = rintf(__fmul_rn(v[t], scale));
        q = fminf(fmaxf(q, -128.0f), 127.0f);
        wq[(size_t)t * c + ch] = (int8_t)(int)q;
    }
}

// Grouped 3x3 weights [c][gs][3][3]: one wavefront per output channel over its 9*gs weights
// (butterfly maximum, then the codes in the layout prom_gconv3x3 takes, [3][3][c][gs]).
__global__ __launch_bounds__(256) void quant_gconv_kernel(const float *__restrict__ w, int c, int gs, float eps,
                                                          int8_t *__restrict__ wq, float *__restrict__ scale_out)
{
    const int lane = threadIdx.x & 63;
    const int ch = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (ch >= c) return;  // whole wavefronts leave together
    const int n = 9 * gs;
    const float *wc = w + (size_t)ch * n;
    float amax = 0.0f;
    for (int i = lane; i < n; i += 64) amax = fmaxf(amax, fabsf(wc[i]));
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
    const float scale = __fdiv_rn(127.0f, fmaxf(amax, eps));
    if (lane == 0) scale_out[ch] = scale;
    for (int i = lane; i < n; i += 64) {
        const int k = i / 9, t = i - 9 * k;  // input channel of the group, tap
        float q = rintf(__fmul_rn(wc[i], scale));
        q = fminf(fmaxf(q, -128.0f), 127.0f);
        wq[((size_t)t * c + ch) * gs + k] = (int8_t)(int)q;
    }
}

// ---- activations: one absmax scale per batch element (paper Section 3.1, Eq. 6-7) -------------
// Pass 1: absmax per image.  |x| >= 0, so the float bits order like unsigned integers and the
// per-image maximum is an atomic max on the bit pattern (the target is cleared by a fill kernel).
// Pass 2: scale = 127 / max(absmax, eps); q = clamp(rint(x * scale), -128, 127), 4 per dword.
// Pass 3 turns the stored absmax into the scale the caller gets.
__global__ __launch_bounds__(256) void act_clear_kernel(uint32_t *amax_bits, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) amax_bits[i] = 0u;
}

__global__ __launch_bounds__(256) void act_absmax_kernel(const float *__restrict__ x, long long per_image,
                                                         uint32_t *__restrict__ amax_bits)
{
    __shared__ float part[4];
    const int img = blockIdx.y;
    const float *xi = x + (long long)img * per_image;
    const long long n4 = per_image >> 2;  // whole float4 groups (the image base is 16-byte aligned when per_image % 4 == 0)
    const bool vec = ((per_image & 3) == 0) && ((((uintptr_t)x) & 15) == 0);
    float m = 0.0f;
    const long long stride = (long long)gridDim.x * 256;
    if (vec) {
        const float4 *x4 = reinterpret_cast<const float4 *>(xi);
        for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
            const float4 v = x4[i];
            m = fmaxf(m, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
        }
    } else {
        for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < per_image; i += stride)
            m = fmaxf(m, fabsf(xi[i]));
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        m = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
        atomicMax(&amax_bits[img], __float_as_uint(m));
    }
}

__device__ __forceinline__ int quant_i8(float v, float scale)
{
    const float q = rintf(__fmul_rn(v, scale));
    return (int)fminf(fmaxf(q, -128.0f), 127.0f);
}

__global__ __launch_bounds__(256) void act_quant_kernel(const float *__restrict__ x, long long per_image, float eps,
                                                        const uint32_t *__restrict__ amax_bits,
                                                        int8_t *__restrict__ q)
{
    const int img = blockIdx.y;
    const float scale = __fdiv_rn(127.0f, fmaxf(__uint_as_float(amax_bits[img]), eps));
    const float *xi = x + (long long)img * per_image;
    int8_t *qi = q + (long long)img * per_image;
    const bool vec = ((per_image & 3) == 0) && ((((uintptr_t)x) & 15) == 0) && ((((uintptr_t)q) & 3) == 0);
    const long long stride = (long long)gridDim.x * 256;
    if (vec) {
        const float4 *x4 = reinterpret_cast<const float4 *>(xi);
        uint32_t *q4 = reinterpret_cast<uint32_t *>(qi);
        const long long n4 = per_image >> 2;
        for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
            const float4 v = x4[i];
            q4[i] = ((uint32_t)quant_i8(v.x, scale) & 255u) | (((uint32_t)quant_i8(v.y, scale) & 255u) << 8) |
                    (((uint32_t)quant_i8(v.z, scale) & 255u) << 16) | ((uint32_t)quant_i8(v.w, scale) << 24);
        }
    } else {
        for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < per_image; i += stride)
            qi[i] = (int8_t)quant_i8(xi[i], scale);
    }
}

__global__ __launch_bounds__(256) void act_scale_kernel(uint32_t *amax_bits, int n, float eps)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) amax_bits[i] = __float_as_uint(__fdiv_rn(127.0f, fmaxf(__uint_as_float(amax_bits[i]), eps)));
}

}  // namespace prom

extern "C" int prom_quantize_activation_absmax(const float *x, int n, long long per_image, float eps, int8_t *q,
                                               float *scale, void *stream)
{
    using namespace prom;
    if (!x || !q || !scale || n <= 0 || per_image <= 0 || !(eps > 0.0f)) return PROM_EINVAL;
    if ((((uintptr_t)x | (uintptr_t)scale) & 3) != 0 || n > 65535) return PROM_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint32_t *bits = reinterpret_cast<uint32_t *>(scale);
    // enough workgroups per image to fill the chip, each with at least a few KB to stream
    long long per = (per_image / 4 + 255) / 256;
    long long want = (256LL * 8 + n - 1) / n;
    if (want < 1) want = 1;
    const unsigned bx = (unsigned)(per < want ? (per < 1 ? 1 : per) : want);
    clear_hip_error();
    hipLaunchKernelGGL(act_clear_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, bits, n);
    hipLaunchKernelGGL(act_absmax_kernel, dim3(bx, (unsigned)n), dim3(256), 0, st, x, per_image, bits);
    hipLaunchKernelGGL(act_quant_kernel, dim3(bx, (unsigned)n), dim3(256), 0, st, x, per_image, eps,
                       static_cast<const uint32_t *>(bits), q);
    hipLaunchKernelGGL(act_scale_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, bits, n, eps);
    return check_launch();
}

extern "C" int prom_quantize_pw_absmean(const float *w, int cout, int cin, float eps, void *packed,
                                        size_t packed_bytes, int8_t *codes, float *scale, void *stream)
{
    if (!w || !packed || !scale || cout <= 0 || cin <= 0 || !(eps > 0.0f)) return PROM_EINVAL;
    if ((((uintptr_t)w | (uintptr_t)packed | (uintptr_t)scale) & 3) != 0) return PROM_EINVAL;
    if (packed_bytes < prom_packed_size(cout, cin)) return PROM_EWORKSPACE;
    prom::clear_hip_error();
    hipLaunchKernelGGL(prom::quant_pw_kernel, dim3((unsigned)((cout + 3) / 4)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), w, cout, cin, eps, static_cast<uint32_t *>(packed), codes,
                       scale);
    return prom::check_launch();
}

extern "C" int prom_quantize_dw_absmax(const float *w, int c, float eps, int8_t *wq, float *scale, void *stream)
{
    if (!w || !wq || !scale || c <= 0 || !(eps > 0.0f)) return PROM_EINVAL;
    if ((((uintptr_t)w | (uintptr_t)scale) & 3) != 0) return PROM_EINVAL;
    prom::clear_hip_error();
    hipLaunchKernelGGL(prom::quant_dw_kernel, dim3((unsigned)((c + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), w, c, eps, wq, scale);
    return prom::check_launch();
}

extern "C" int prom_quantize_gconv_absmax(const float *w, int c, int group_size, float eps, int8_t *wq,
                                          float *scale, void *stream)
{
    if (!w || !wq || !scale || c <= 0 || group_size <= 0 || c % group_size != 0 || !(eps > 0.0f)) return PROM_EINVAL;
    if ((((uintptr_t)w | (uintptr_t)scale) & 3) != 0) return PROM_EINVAL;
    if (group_size > 4096) return PROM_EUNSUPPORTED;
    prom::clear_hip_error();
    hipLaunchKernelGGL(prom::quant_gconv_kernel, dim3((unsigned)((c + 3) / 4)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), w, c, group_size, eps, wq, scale);
    return prom::check_launch();
}
