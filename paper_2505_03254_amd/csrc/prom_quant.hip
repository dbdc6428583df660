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

}  // namespace prom

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
