/*
 * Device build of the synthetic-input generator (see synth_gen.h): a fill
 * kernel that writes a slice of a stream into device memory.  It stands in for
 * the backward pass that would produce a layer's gradients; it is not part of
 * the optimizer library and is never inside a timed region.
 * hipcc --offload-arch=gfx950 -O3 -ffp-contract=off -shared -fPIC
 */
#include <hip/hip_runtime.h>

#include "synth_gen.h"

__global__ void __launch_bounds__(256) synth_fill_kernel(void *out, int dtype, uint64_t n, uint64_t first, synth_spec sp)
{
    uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        synth_store(out, dtype, i, synth_value(&sp, first + i));
}

/* Enqueue the fill on `stream`; out is device memory.  Returns 0, 1 on a bad argument, 2 on a HIP error. */
extern "C" int synth_fill_device(void *out, int dtype, uint64_t n, uint64_t first, const synth_spec *spec, void *stream)
{
    if (n == 0) return 0;
    if (!out || !spec || dtype < SYNTH_F32 || dtype > SYNTH_F16) return 1;
    uint64_t blocks = (n + 255) / 256;
    if (blocks > 256u * 64u) blocks = 256u * 64u;
    hipLaunchKernelGGL(synth_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, out, dtype, n, first, *spec);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

/* A plain 16-byte-per-lane copy of `bytes` bytes (multiple of 16, 16-byte aligned): the known-size
   reference that hardware traffic counters are scaled against. */
typedef float synth_f32x4 __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256) synth_copy_kernel(synth_f32x4 *dst, const synth_f32x4 *src, uint64_t n16)
{
    uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

extern "C" int synth_copy_device(void *dst, const void *src, uint64_t bytes, void *stream)
{
    if (bytes == 0) return 0;
    if (!dst || !src || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return 1;
    hipLaunchKernelGGL(synth_copy_kernel, dim3(256u * 32u), dim3(256), 0, (hipStream_t)stream,
                       (synth_f32x4 *)dst, (const synth_f32x4 *)src, bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : 2;
}
