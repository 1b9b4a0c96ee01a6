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
