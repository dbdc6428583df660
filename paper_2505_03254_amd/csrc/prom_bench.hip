// Measurement utilities: streaming kernels that give the HBM ceilings of this machine beside the
// data-sheet figure (read only, write only; the copy is prom_copy_bytes), and a register-resident
// int8 MFMA loop that gives the matrix-core ceiling.  None of them is part of the path.
#include "prom.h"
#include "prom_device.h"
#include "prom_launch.h"

namespace prom {

// Grid-stride read of n16 16-byte pieces; the sum is kept live through a store that never happens
// for data that is not all 0x12345678.
__global__ __launch_bounds__(256) void stream_read_kernel(const v4i *__restrict__ src, long long n16, int *sink)
{
    const long long stride = (long long)gridDim.x * 256;
    v4i acc = {0, 0, 0, 0};
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) acc += src[i];
    if (acc[0] + acc[1] + acc[2] + acc[3] == 0x12345678) sink[0] = 1;
}

__global__ __launch_bounds__(256) void stream_write_kernel(v4i *__restrict__ dst, long long n16, int value)
{
    const long long stride = (long long)gridDim.x * 256;
    const v4i v = {value, value, value, value};
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = v;
}

// Every wavefront issues iters * 8 independent-in-pairs v_mfma_i32_16x16x64_i8 on registers only.
__global__ __launch_bounds__(256) void mfma_i8_loop_kernel(int iters, int *sink)
{
    const int lane = threadIdx.x & 63;
    v4i a = {lane, lane + 1, lane + 2, lane + 3}, bq = {3 * lane, 5, 7, 11};
    v4i acc[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u] = v4i{u, 0, 0, 0};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u) acc[u] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, bq, acc[u], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) s += acc[u][0] + acc[u][1] + acc[u][2] + acc[u][3];
    if (s == 0x12345678) sink[0] = s;
}

}  // namespace prom

extern "C" int prom_stream_read(const void *src, size_t nbytes, int *sink, void *stream)
{
    if (!src || !sink || nbytes == 0 || (nbytes & 15) != 0 || ((uintptr_t)src & 15) != 0) return PROM_EINVAL;
    prom::clear_hip_error();
    // four workgroups per compute unit: measured best of 1 to 64 per CU for the grid-stride form
    hipLaunchKernelGGL(prom::stream_read_kernel, dim3(1024), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const prom::v4i *>(src), (long long)(nbytes / 16), sink);
    return prom::check_launch();
}

extern "C" int prom_stream_write(void *dst, size_t nbytes, int value, void *stream)
{
    if (!dst || nbytes == 0 || (nbytes & 15) != 0 || ((uintptr_t)dst & 15) != 0) return PROM_EINVAL;
    prom::clear_hip_error();
    // one workgroup per compute unit: more concurrent writers lower the write bandwidth
    hipLaunchKernelGGL(prom::stream_write_kernel, dim3(256), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<prom::v4i *>(dst), (long long)(nbytes / 16), value);
    return prom::check_launch();
}

extern "C" long long prom_mfma_i8_loop(int iters, int *sink, void *stream)
{
    if (iters <= 0 || !sink) return PROM_EINVAL;
    prom::clear_hip_error();
    const int wgs = 256 * 4;  // four workgroups of four wavefronts per compute unit: 4 wavefronts per SIMD
    hipLaunchKernelGGL(prom::mfma_i8_loop_kernel, dim3(wgs), dim3(256), 0, static_cast<hipStream_t>(stream), iters, sink);
    const int rc = prom::check_launch();
    if (rc != PROM_OK) return rc;
    // multiply-accumulates count twice: 16 x 16 x 64 x 2 operations per instruction
    return (long long)wgs * 4 * (long long)iters * 8 * 32768;
}
