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

/* ---- traffic-mix probe ----
   Streams with the access mix of the optimizer's kernels and none of its arithmetic, to measure what
   the memory system delivers for a given read : write ratio: one workgroup of BLOCK threads per chunk
   of BLOCK*4 elements, one 16-byte access per lane per float32 array (8-byte for the 16-bit array),
   every access non-temporal.  A mode is described by which arrays are read and which are written:
     g16 : a 2-byte-per-element array, read only          (a bf16 / fp16 gradient)
     g32 : a 4-byte-per-element array, read only          (an fp32 gradient, or a moment the update only reads)
     rw  : number of float32 arrays read and written back (moments, parameters)
     ro  : number of further float32 arrays read only
     wo  : number of float32 arrays written only
   Arrays are taken from a0, a1, a2 in the order rw, ro, wo. */
typedef uint32_t synth_u32x2 __attribute__((ext_vector_type(2)));
#define SYNTH_GLOBAL __attribute__((address_space(1)))

/* Four float32 values of magnitude about 3e-5 with hashed mantissas: what a store-only probe writes, so that
   the lines it writes are no easier to move than a workload's (all-zero lines stream faster). */
__device__ __forceinline__ synth_f32x4 synth_varied(uint32_t seed)
{
    uint32_t h = seed * 2654435761u;
    h ^= h >> 15;
    synth_f32x4 r;
    r.x = __builtin_bit_cast(float, (h & 0x807fffffu) | 0x38000000u);
    h *= 2246822519u;
    r.y = __builtin_bit_cast(float, (h & 0x807fffffu) | 0x38000000u);
    h ^= h >> 13;
    r.z = __builtin_bit_cast(float, (h & 0x807fffffu) | 0x38000000u);
    h *= 3266489917u;
    r.w = __builtin_bit_cast(float, (h & 0x807fffffu) | 0x38000000u);
    return r;
}

template <int BLOCK, int U, int G16, int G32, int RW, int RO, int WO>
__global__ void __launch_bounds__(BLOCK) synth_stream_probe_kernel(const void *g, float *a0, float *a1, float *a2, float *sink)
{
    static_assert(RW + RO + WO <= 3, "three float32 arrays at most");
    const uint64_t e0 = (uint64_t)blockIdx.x * (BLOCK * 4 * U);
    float *arr[3] = {a0, a1, a2};
    synth_f32x4 x[3][U];
    synth_f32x4 acc[U];
    /* all loads of the chunk first, then, group by group, the stores */
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t i = u * BLOCK + threadIdx.x;
        acc[u] = synth_f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        if (G16 + G32 + RW + RO == 0) acc[u] = synth_varied((uint32_t)e0 + i);
        if (G16) {
            synth_u32x2 w = __builtin_nontemporal_load((const SYNTH_GLOBAL synth_u32x2 *)((const uint16_t *)g + e0) + i);
            acc[u].x += __builtin_bit_cast(float, w.x << 16);
            acc[u].y += __builtin_bit_cast(float, w.y << 16);
        }
        if (G32) acc[u] += __builtin_nontemporal_load((const SYNTH_GLOBAL synth_f32x4 *)((const float *)g + e0) + i);
#pragma unroll
        for (int k = 0; k < RW + RO; ++k) x[k][u] = __builtin_nontemporal_load((SYNTH_GLOBAL synth_f32x4 *)(arr[k] + e0) + i);
    }
    /* every load above is issued before anything below: without this the instruction scheduler may sink a
       load behind the first use of another one, which doubles a workgroup's time in flight */
    __builtin_amdgcn_sched_barrier(0);
    float keep = 0.0f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t i = u * BLOCK + threadIdx.x;
#pragma unroll
        for (int k = RW; k < RW + RO; ++k) acc[u] += x[k][u];
#pragma unroll
        for (int k = 0; k < RW; ++k) __builtin_nontemporal_store(x[k][u] + acc[u], (SYNTH_GLOBAL synth_f32x4 *)(arr[k] + e0) + i);
#pragma unroll
        for (int k = RW + RO; k < RW + RO + WO; ++k) __builtin_nontemporal_store(acc[u], (SYNTH_GLOBAL synth_f32x4 *)(arr[k] + e0) + i);
        keep += acc[u].x + acc[u].y + acc[u].z + acc[u].w;
    }
    if (RW + WO == 0 && keep == 12345.678f) *sink = keep;   /* keeps read-only loads alive */
}

template <int BLOCK, int U>
static int synth_stream_probe_launch(int mode, unsigned grid, unsigned lds_bytes, const void *g, float *a0, float *a1, float *a2,
                                     float *sink, hipStream_t s)
{
    /* more than 64 KiB of dynamic LDS has to be asked for per kernel */
#define SYNTH_PROBE(G16, G32, RW, RO, WO)                                                                                   \
    do {                                                                                                                    \
        auto kern = synth_stream_probe_kernel<BLOCK, U, G16, G32, RW, RO, WO>;                                              \
        if (lds_bytes > 65536u &&                                                                                           \
            hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess) \
            return 2;                                                                                                       \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(BLOCK), lds_bytes, s, g, a0, a1, a2, sink);                               \
    } while (0)
    switch (mode) {
    case 0: SYNTH_PROBE(1, 0, 0, 2, 0); break;   /* read only, fold's inputs: g16, m, v         10 B/element */
    case 1: SYNTH_PROBE(0, 0, 0, 0, 2); break;   /* write only, fold's outputs: m, v             8 */
    case 2: SYNTH_PROBE(1, 0, 2, 0, 0); break;   /* fold mix, 16-bit gradient: r g,m,v  w m,v   18 */
    case 3: SYNTH_PROBE(0, 1, 2, 0, 0); break;   /* fold mix, fp32 gradient                     20 */
    case 4: SYNTH_PROBE(0, 0, 2, 0, 0); break;   /* decay mix: r m,v  w m,v                     16 */
    case 5: SYNTH_PROBE(0, 0, 1, 2, 0); break;   /* update mix: r theta,m,v  w theta            16 */
    case 6: SYNTH_PROBE(0, 0, 3, 0, 0); break;   /* rescale mix: r and w theta,m,v              24 */
    case 7: SYNTH_PROBE(0, 0, 0, 3, 0); break;   /* read only, three fp32 arrays                12 */
    default: return 1;
    }
#undef SYNTH_PROBE
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

/* The same streams from a persistent grid: `grid` workgroups, workgroup w taking chunks w, w + grid, ...
   of BLOCK*4 elements one after the other (no workgroup start-up between chunks; the number of
   workgroups, not the hardware's residency limit, sets how many requests are in flight). */
template <int BLOCK, int G16, int G32, int RW, int RO, int WO>
__global__ void __launch_bounds__(BLOCK) synth_stream_probe_persistent_kernel(const void *g, float *a0, float *a1, float *a2,
                                                                              float *sink, uint32_t nchunks)
{
    float *arr[3] = {a0, a1, a2};
    const uint32_t i = threadIdx.x;
    float keep = 0.0f;
#pragma unroll 1
    for (uint32_t c = blockIdx.x; c < nchunks; c += gridDim.x) {
        const uint64_t e = (uint64_t)c * (BLOCK * 4);
        synth_f32x4 x[3];
        synth_f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
        synth_u32x2 w16 = {0u, 0u};
        synth_f32x4 w32 = acc;
        if (G16) w16 = __builtin_nontemporal_load((const SYNTH_GLOBAL synth_u32x2 *)((const uint16_t *)g + e) + i);
        if (G32) w32 = __builtin_nontemporal_load((const SYNTH_GLOBAL synth_f32x4 *)((const float *)g + e) + i);
#pragma unroll
        for (int k = 0; k < RW + RO; ++k) x[k] = __builtin_nontemporal_load((SYNTH_GLOBAL synth_f32x4 *)(arr[k] + e) + i);
        __builtin_amdgcn_sched_barrier(0);
        if (G16) {
            acc.x += __builtin_bit_cast(float, w16.x << 16);
            acc.y += __builtin_bit_cast(float, w16.y << 16);
        }
        if (G32) acc += w32;
#pragma unroll
        for (int k = RW; k < RW + RO; ++k) acc += x[k];
#pragma unroll
        for (int k = 0; k < RW; ++k) __builtin_nontemporal_store(x[k] + acc, (SYNTH_GLOBAL synth_f32x4 *)(arr[k] + e) + i);
#pragma unroll
        for (int k = RW + RO; k < RW + RO + WO; ++k) __builtin_nontemporal_store(acc, (SYNTH_GLOBAL synth_f32x4 *)(arr[k] + e) + i);
        keep += acc.x + acc.y + acc.z + acc.w;
    }
    if (RW + WO == 0 && keep == 12345.678f) *sink = keep;
}

template <int BLOCK>
static int synth_stream_probe_persistent_launch(int mode, unsigned grid, const void *g, float *a0, float *a1, float *a2, float *sink,
                                                uint32_t nchunks, hipStream_t s)
{
#define SYNTH_PROBE(G16, G32, RW, RO, WO) \
    hipLaunchKernelGGL((synth_stream_probe_persistent_kernel<BLOCK, G16, G32, RW, RO, WO>), dim3(grid), dim3(BLOCK), 0, s, g, a0, a1, a2, sink, nchunks)
    switch (mode) {
    case 0: SYNTH_PROBE(1, 0, 0, 2, 0); break;
    case 1: SYNTH_PROBE(0, 0, 0, 0, 2); break;
    case 2: SYNTH_PROBE(1, 0, 2, 0, 0); break;
    case 3: SYNTH_PROBE(0, 1, 2, 0, 0); break;
    case 4: SYNTH_PROBE(0, 0, 2, 0, 0); break;
    case 5: SYNTH_PROBE(0, 0, 1, 2, 0); break;
    case 6: SYNTH_PROBE(0, 0, 3, 0, 0); break;
    case 7: SYNTH_PROBE(0, 0, 0, 3, 0); break;
    default: return 1;
    }
#undef SYNTH_PROBE
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

/* Enqueue one persistent probe launch of `grid` workgroups of `block` threads (64, 128 or 256) over the first n
   elements (a multiple of block*4); other arguments as synth_stream_probe_shape. */
extern "C" int synth_stream_probe_persistent(int mode, int block, unsigned grid, const void *g, float *a0, float *a1, float *a2,
                                             float *sink, uint64_t n, void *stream)
{
    if (n == 0) return 0;
    if (mode < 0 || mode > 7 || grid == 0 || !a0 || !a1 || !a2 || !sink) return 1;
    if (block != 64 && block != 128 && block != 256) return 1;
    const uint64_t chunk = (uint64_t)block * 4;
    if (n % chunk || n / chunk > 0x7FFFFFFFull) return 1;
    if ((mode == 0 || mode == 2 || mode == 3) && !g) return 1;
    if (((uintptr_t)g | (uintptr_t)a0 | (uintptr_t)a1 | (uintptr_t)a2) & 15) return 1;
    const uint32_t nchunks = (uint32_t)(n / chunk);
    hipStream_t s = (hipStream_t)stream;
    if (block == 64) return synth_stream_probe_persistent_launch<64>(mode, grid, g, a0, a1, a2, sink, nchunks, s);
    if (block == 128) return synth_stream_probe_persistent_launch<128>(mode, grid, g, a0, a1, a2, sink, nchunks, s);
    return synth_stream_probe_persistent_launch<256>(mode, grid, g, a0, a1, a2, sink, nchunks, s);
}

/* Cache-policy probe: the fold's access mix (read a 16-bit array and two float32 arrays, write the two
   float32 arrays back; 18 B/element) or its read half or write half alone, with a chosen combination of the
   documented sc0 / sc1 / nt modifiers on the global loads and on the global stores.  The compiler's builtins
   reach only "" and "nt", so the memory instructions are written out: every operand is a vector register
   (hardware-interlocked), the loads are waited for explicitly (the compiler does not count loads it cannot
   see), and each store is followed by the one wait state a store of more than 8 bytes needs before its data
   registers may be overwritten. */
#define SYNTH_POLICY_CASES(OP, ...)                                                         \
    if constexpr (P == 0) asm volatile(OP " %0, %1, off" __VA_ARGS__);                      \
    if constexpr (P == 1) asm volatile(OP " %0, %1, off nt" __VA_ARGS__);                   \
    if constexpr (P == 2) asm volatile(OP " %0, %1, off sc0" __VA_ARGS__);                  \
    if constexpr (P == 3) asm volatile(OP " %0, %1, off sc1" __VA_ARGS__);                  \
    if constexpr (P == 4) asm volatile(OP " %0, %1, off sc0 sc1" __VA_ARGS__);              \
    if constexpr (P == 5) asm volatile(OP " %0, %1, off sc0 sc1 nt" __VA_ARGS__);           \
    if constexpr (P == 6) asm volatile(OP " %0, %1, off sc0 nt" __VA_ARGS__);               \
    if constexpr (P == 7) asm volatile(OP " %0, %1, off sc1 nt" __VA_ARGS__)

template <int P> __device__ __forceinline__ synth_f32x4 synth_policy_ld16(const float *p)
{
    synth_f32x4 r;
    SYNTH_POLICY_CASES("global_load_dwordx4", : "=v"(r) : "v"(p) : "memory");
    return r;
}
template <int P> __device__ __forceinline__ synth_u32x2 synth_policy_ld8(const uint16_t *p)
{
    synth_u32x2 r;
    SYNTH_POLICY_CASES("global_load_dwordx2", : "=v"(r) : "v"(p) : "memory");
    return r;
}
template <int P> __device__ __forceinline__ void synth_policy_st16(float *p, synth_f32x4 x)
{
#define SYNTH_ST_CASE(N, MODS) if constexpr (P == N) asm volatile("global_store_dwordx4 %0, %1, off" MODS "\n\ts_nop 0" : : "v"(p), "v"(x) : "memory")
    SYNTH_ST_CASE(0, ""); SYNTH_ST_CASE(1, " nt"); SYNTH_ST_CASE(2, " sc0"); SYNTH_ST_CASE(3, " sc1"); SYNTH_ST_CASE(4, " sc0 sc1");
    SYNTH_ST_CASE(5, " sc0 sc1 nt"); SYNTH_ST_CASE(6, " sc0 nt"); SYNTH_ST_CASE(7, " sc1 nt");
#undef SYNTH_ST_CASE
}

/* WHAT: 0 = the mix, 1 = the reads alone, 2 = the writes alone.  One workgroup of 128 threads per 512 elements. */
template <int LP, int SP, int WHAT>
__global__ void __launch_bounds__(128) synth_cache_policy_kernel(const uint16_t *g, float *a0, float *a1, float *sink)
{
    const uint64_t e = (uint64_t)blockIdx.x * 512 + threadIdx.x * 4;
    synth_f32x4 x0 = {0.0f, 0.0f, 0.0f, 0.0f}, x1 = x0;
    synth_u32x2 w = {0u, 0u};
    if (WHAT == 2) {
        x0 = synth_varied((uint32_t)e);
        x1 = synth_varied((uint32_t)e + 1u);
    }
    if (WHAT != 2) {
        w = synth_policy_ld8<LP>(g + e);
        x0 = synth_policy_ld16<LP>(a0 + e);
        x1 = synth_policy_ld16<LP>(a1 + e);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    synth_f32x4 gg;
    gg.x = __builtin_bit_cast(float, w.x << 16);
    gg.y = __builtin_bit_cast(float, w.x & 0xffff0000u);
    gg.z = __builtin_bit_cast(float, w.y << 16);
    gg.w = __builtin_bit_cast(float, w.y & 0xffff0000u);
    const synth_f32x4 y0 = x0 + gg, y1 = x1 + gg;
    if (WHAT != 1) {
        synth_policy_st16<SP>(a0 + e, y0);
        synth_policy_st16<SP>(a1 + e, y1);
    } else {
        const float keep = y0.x + y0.y + y0.z + y0.w + y1.x + y1.y + y1.z + y1.w;
        if (keep == 12345.678f) *sink = keep;
    }
}

template <int LP, int WHAT>
static void synth_cache_policy_launch(int sp, unsigned grid, const uint16_t *g, float *a0, float *a1, float *sink, hipStream_t s)
{
#define SYNTH_SP(N) case N: hipLaunchKernelGGL((synth_cache_policy_kernel<LP, N, WHAT>), dim3(grid), dim3(128), 0, s, g, a0, a1, sink); break
    switch (sp) { SYNTH_SP(0); SYNTH_SP(1); SYNTH_SP(2); SYNTH_SP(3); SYNTH_SP(4); SYNTH_SP(5); SYNTH_SP(6); SYNTH_SP(7); }
#undef SYNTH_SP
}

/* Enqueue one cache-policy probe launch over the first n elements (a multiple of 512) of g (16-bit elements), a0
   and a1 (float32), all 16-byte aligned device memory of at least n elements.  load_policy and store_policy:
   0 none, 1 nt, 2 sc0, 3 sc1, 4 sc0 sc1, 5 sc0 sc1 nt, 6 sc0 nt, 7 sc1 nt.  what: 0 mix (18 B/element), 1 reads
   alone (10), 2 writes alone (8).  Returns 0, 1 on a bad argument, 2 on a HIP error. */
extern "C" int synth_cache_policy_probe(int load_policy, int store_policy, int what, const void *g, float *a0, float *a1,
                                        float *sink, uint64_t n, void *stream)
{
    if (n == 0) return 0;
    if (load_policy < 0 || load_policy > 7 || store_policy < 0 || store_policy > 7 || what < 0 || what > 2) return 1;
    if (!g || !a0 || !a1 || !sink || n % 512 || n / 512 > 0x7FFFFFFFull) return 1;
    if (((uintptr_t)g | (uintptr_t)a0 | (uintptr_t)a1) & 15) return 1;
    const unsigned grid = (unsigned)(n / 512);
    const uint16_t *gp = (const uint16_t *)g;
    hipStream_t s = (hipStream_t)stream;
#define SYNTH_LP(N)                                                                              \
    case N:                                                                                      \
        if (what == 0) synth_cache_policy_launch<N, 0>(store_policy, grid, gp, a0, a1, sink, s); \
        else if (what == 1) synth_cache_policy_launch<N, 1>(store_policy, grid, gp, a0, a1, sink, s); \
        else synth_cache_policy_launch<N, 2>(store_policy, grid, gp, a0, a1, sink, s);           \
        break
    switch (load_policy) { SYNTH_LP(0); SYNTH_LP(1); SYNTH_LP(2); SYNTH_LP(3); SYNTH_LP(4); SYNTH_LP(5); SYNTH_LP(6); SYNTH_LP(7); }
#undef SYNTH_LP
    return hipGetLastError() == hipSuccess ? 0 : 2;
}

/* Bytes per element of a probe mode, 0 for an unknown mode. */
extern "C" int synth_stream_probe_bytes(int mode)
{
    static const int bytes[8] = {10, 8, 18, 20, 16, 16, 24, 12};
    return mode >= 0 && mode < 8 ? bytes[mode] : 0;
}

/* Enqueue one probe launch over the first n elements: workgroups of `block` threads (64, 128, 256, 512 or
   1024), each thread moving `groups` 4-element groups per array (1, 2 or 4), one workgroup per chunk of
   block*4*groups elements; n must be a multiple of the chunk; arrays are 16-byte aligned device memory of
   at least n elements each; g may be NULL for modes without one.  lds_bytes of (unused) dynamic LDS per
   workgroup (at most 160 KiB) limit how many workgroups a compute unit holds at once: the knob for
   measuring how the number of requests in flight changes the delivered bandwidth.
   Returns 0, 1 on a bad argument, 2 on a HIP error. */
extern "C" int synth_stream_probe_shape(int mode, int block, int groups, unsigned lds_bytes, const void *g, float *a0, float *a1,
                                        float *a2, float *sink, uint64_t n, void *stream)
{
    if (n == 0) return 0;
    if (mode < 0 || mode > 7 || groups < 1 || block < 64 || !a0 || !a1 || !a2 || !sink || lds_bytes > 160u * 1024u) return 1;
    const uint64_t chunk = (uint64_t)block * 4 * (uint64_t)groups;
    if (n % chunk || n / chunk > 0x7FFFFFFFull) return 1;
    if ((mode == 0 || mode == 2 || mode == 3) && !g) return 1;
    if (((uintptr_t)g | (uintptr_t)a0 | (uintptr_t)a1 | (uintptr_t)a2) & 15) return 1;
    const unsigned grid = (unsigned)(n / chunk);
    hipStream_t s = (hipStream_t)stream;
#define SYNTH_SHAPE(B, G) if (block == B && groups == G) return synth_stream_probe_launch<B, G>(mode, grid, lds_bytes, g, a0, a1, a2, sink, s)
    SYNTH_SHAPE(64, 1); SYNTH_SHAPE(64, 2); SYNTH_SHAPE(64, 4);
    SYNTH_SHAPE(128, 1); SYNTH_SHAPE(128, 2); SYNTH_SHAPE(128, 4);
    SYNTH_SHAPE(256, 1); SYNTH_SHAPE(256, 2); SYNTH_SHAPE(256, 4);
    SYNTH_SHAPE(512, 1); SYNTH_SHAPE(512, 2);
    SYNTH_SHAPE(1024, 1);
#undef SYNTH_SHAPE
    return 1;
}

extern "C" int synth_stream_probe(int mode, int block, const void *g, float *a0, float *a1, float *a2, float *sink,
                                  uint64_t n, void *stream)
{
    return synth_stream_probe_shape(mode, block, 1, 0, g, a0, a1, a2, sink, n, stream);
}
