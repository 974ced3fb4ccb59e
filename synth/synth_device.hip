/*
 * Device fill kernels of the synthetic input generator (see synth_core.h).
 * Built by hipcc for gfx950 into libsynth_device.so; loaded through ctypes.
 * Pointers are device pointers; `stream` is a hipStream_t passed as void*.
 * Returns 0 on success, the hipError_t value otherwise.  Asynchronous.
 */
#include <hip/hip_runtime.h>
#include "synth_core.h"

#define SYNTH_EXPORT extern "C" __attribute__((visibility("default")))

namespace {

constexpr int kBlock = 256;

inline int grid_for(int64_t n)
{
    int64_t blocks = (n + kBlock - 1) / kBlock;
    const int64_t cap = 256 * 32;
    return (int)(blocks < cap ? blocks : cap);
}

__global__ void __launch_bounds__(kBlock)
fill_normal_f32(float* out, int64_t j0, int64_t n, uint64_t key, float scale)
{
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride)
        out[i] = synth_normal_f32(key, j0 + i, scale);
}

__global__ void __launch_bounds__(kBlock)
fill_uniform_f32(float* out, int64_t j0, int64_t n, uint64_t key, float scale)
{
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride)
        out[i] = synth_uniform_f32(key, j0 + i, scale);
}

__global__ void __launch_bounds__(kBlock)
fill_grad_bf16(uint16_t* out, int64_t j0, int64_t n, synth_grad_spec sp)
{
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride)
        out[i] = synth_grad_bf16(&sp, j0 + i);
}

}  // namespace

SYNTH_EXPORT int synth_device_fill_normal_f32(float* out, int64_t j0, int64_t n, uint64_t key,
                                              float scale, void* stream)
{
    if (n <= 0) return 0;
    hipLaunchKernelGGL(fill_normal_f32, dim3(grid_for(n)), dim3(kBlock), 0, (hipStream_t)stream,
                       out, j0, n, key, scale);
    return (int)hipGetLastError();
}

SYNTH_EXPORT int synth_device_fill_uniform_f32(float* out, int64_t j0, int64_t n, uint64_t key,
                                               float scale, void* stream)
{
    if (n <= 0) return 0;
    hipLaunchKernelGGL(fill_uniform_f32, dim3(grid_for(n)), dim3(kBlock), 0, (hipStream_t)stream,
                       out, j0, n, key, scale);
    return (int)hipGetLastError();
}

SYNTH_EXPORT int synth_device_fill_grad_bf16(uint16_t* out, int64_t j0, int64_t n,
                                             const synth_grad_spec* sp, void* stream)
{
    if (n <= 0) return 0;
    hipLaunchKernelGGL(fill_grad_bf16, dim3(grid_for(n)), dim3(kBlock), 0, (hipStream_t)stream,
                       out, j0, n, *sp);
    return (int)hipGetLastError();
}
