// Device kernels of libadama (gfx950).
//
// One kernel template serves the three memory-bound elementwise steps of AdamA
// (paper Alg. 2): the once-per-mini-batch moment decay, the per-layer
// per-micro-batch fold, and the bias-corrected update.  Each is a pure stream:
//
//   decay : read m, v            write m, v        16 B / element
//   fold  : read grad, m, v      write m, v        16 + sizeof(grad) B / element
//   apply : read theta, m, v     write theta       16 B / element
//
// so the design goal is HBM bandwidth, not arithmetic: no MFMA, no LDS tiling of
// data (there is no reuse), only wide coalesced accesses and enough of them in
// flight.  A workgroup of 256 threads walks chunks of 1024*U elements; inside
// an interior chunk each thread issues all of its U 16-byte loads per array
// before the first use, so a wavefront has 2U..3U independent 1-KiB requests
// outstanding.  The table of tensors of the launch arrives in the kernel
// argument block, together with the per-tensor chunk prefix that maps a chunk
// number to its tensor; both are read through the scalar cache.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adama_index.hpp"

namespace adama {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

enum GradType : int { kF32 = 0, kBF16 = 1, kF16 = 2 };

// Every data pointer of a launch is device global memory.  The descriptors travel through LDS as
// integers, so the address space is restored here: global (not flat) loads and stores return in
// order, which lets the hardware counters wait for the oldest of many outstanding loads.
#define ADAMA_GLOBAL __attribute__((address_space(1)))
template <typename T>
__device__ __forceinline__ ADAMA_GLOBAL T *global_ptr(const void *p, uint64_t elem_offset_bytes = 0)
{
    return (ADAMA_GLOBAL T *)(reinterpret_cast<uintptr_t>(p) + elem_offset_bytes);
}

// Policy bits of a kernel instantiation: which streams use non-temporal accesses, and whether interior
// chunks address memory through buffer descriptors (scalar base + 32-bit lane offset) instead of
// 64-bit per-lane global addresses.
enum : int { kNtGradLoad = 1, kNtStateLoad = 2, kNtStore = 4, kBufferAddressing = 8 };

// decay: s0 = beta1, s1 = beta2.  fold: s0 = (1-beta1)/N, s1 = (1-beta2)/N^2.
// apply: s0 = lr/(1-beta1^t), s1 = 1/sqrt(1-beta2^t), s2 = eps.
struct Scalars {
    float s0, s1, s2;
};

template <bool NT, typename T>
__device__ __forceinline__ T ld(const ADAMA_GLOBAL T *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <bool NT, typename T>
__device__ __forceinline__ void st(ADAMA_GLOBAL T *p, T x)
{
    if constexpr (NT) __builtin_nontemporal_store(x, p);
    else *p = x;
}

// Buffer-descriptor access to one chunk: base is wave-uniform, `bytes` bounds the range (the hardware
// drops anything outside it), offsets are 32-bit.  aux bit 1 is the non-temporal hint on gfx950.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t chunk_rsrc(const void *base, uint64_t byte_offset, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void *>(reinterpret_cast<uintptr_t>(base) + byte_offset),
                                             0, bytes, 0x00020000);
}

template <bool NT, typename T>
__device__ __forceinline__ T buf_ld(__amdgpu_buffer_rsrc_t r, uint32_t byte_offset)
{
    constexpr int aux = NT ? 2 : 0;
    if constexpr (sizeof(T) == 16) return __builtin_bit_cast(T, __builtin_amdgcn_raw_buffer_load_b128(r, byte_offset, 0, aux));
    else return __builtin_bit_cast(T, __builtin_amdgcn_raw_buffer_load_b64(r, byte_offset, 0, aux));
}

template <bool NT>
__device__ __forceinline__ void buf_st(__amdgpu_buffer_rsrc_t r, uint32_t byte_offset, f32x4 x)
{
    constexpr int aux = NT ? 2 : 0;
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, x), r, byte_offset, 0, aux);
}

// ---- gradient storage formats: 4-element vector type, element type, exact widening to float32 ----
template <int GT> struct Grad;

template <> struct Grad<kF32> {
    using Vec = f32x4;
    using Elem = float;
    static __device__ __forceinline__ f32x4 widen(f32x4 g) { return g; }
    static __device__ __forceinline__ float widen1(float g) { return g; }
};

template <> struct Grad<kBF16> {   // bfloat16 is the upper half of a float32 word
    using Vec = u32x2;
    using Elem = uint16_t;
    static __device__ __forceinline__ f32x4 widen(u32x2 w)
    {
        f32x4 g;
        g.x = __builtin_bit_cast(float, w.x << 16);
        g.y = __builtin_bit_cast(float, w.x & 0xFFFF0000u);
        g.z = __builtin_bit_cast(float, w.y << 16);
        g.w = __builtin_bit_cast(float, w.y & 0xFFFF0000u);
        return g;
    }
    static __device__ __forceinline__ float widen1(uint16_t h) { return __builtin_bit_cast(float, (uint32_t)h << 16); }
};

template <> struct Grad<kF16> {    // hardware conversion; exact, subnormals included
    using Vec = f16x4;
    using Elem = _Float16;
    static __device__ __forceinline__ f32x4 widen(f16x4 h) { return __builtin_convertvector(h, f32x4); }
    static __device__ __forceinline__ float widen1(_Float16 h) { return (float)h; }
};

// ---- the arithmetic of the three steps, one element at a time ----
// Alg. 2 inner body with c1 = (1-beta1)/N, c2 = (1-beta2)/N^2 applied to the raw gradient:
// m += c1*g, v += c2*g^2.  g*g is exact in float32 for bf16 and fp16 inputs.
__device__ __forceinline__ void fold1(float &m, float &v, float g, const Scalars &sc)
{
    m = __builtin_fmaf(sc.s0, g, m);
    v = __builtin_fmaf(sc.s1, g * g, v);
}

__device__ __forceinline__ void decay1(float &m, float &v, const Scalars &sc)
{
    m = sc.s0 * m;
    v = sc.s1 * v;
}

// Alg. 2 Update: theta - lr*m_hat/(sqrt(v_hat)+eps) with m_hat = m/(1-beta1^t), v_hat = v/(1-beta2^t),
// written as theta - s0*m / (sqrt(v)*s1 + eps).  IEEE square root and division.
__device__ __forceinline__ float apply1(float theta, float m, float v, const Scalars &sc)
{
    float denom = __builtin_fmaf(__builtin_sqrtf(v), sc.s1, sc.s2);
    return theta - (sc.s0 * m) / denom;
}

// The same three steps on a 16-byte group, element by element.
__device__ __forceinline__ void fold4(f32x4 &m, f32x4 &v, f32x4 g, const Scalars &sc)
{
#pragma unroll
    for (int j = 0; j < kGroup; ++j) {
        float mj = m[j], vj = v[j];
        fold1(mj, vj, g[j], sc);
        m[j] = mj;
        v[j] = vj;
    }
}

__device__ __forceinline__ void decay4(f32x4 &m, f32x4 &v, const Scalars &sc)
{
#pragma unroll
    for (int j = 0; j < kGroup; ++j) {
        float mj = m[j], vj = v[j];
        decay1(mj, vj, sc);
        m[j] = mj;
        v[j] = vj;
    }
}

__device__ __forceinline__ void apply4(f32x4 &th, f32x4 m, f32x4 v, const Scalars &sc)
{
#pragma unroll
    for (int j = 0; j < kGroup; ++j) th[j] = apply1(th[j], m[j], v[j], sc);
}

__device__ __forceinline__ uint64_t uniform64(uint64_t x)
{
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x);
    uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
    return ((uint64_t)hi << 32) | lo;
}

// ---- one interior chunk: every group is a full aligned group; all loads first ----
template <int OpK, int GT, int U, int NT>
__device__ __forceinline__ void interior_chunk(const Desc &d, uint64_t e0, uint32_t tid, const Scalars &sc)
{
    constexpr bool ntg = (NT & kNtGradLoad) != 0, ntl = (NT & kNtStateLoad) != 0, nts = (NT & kNtStore) != 0;
    if constexpr ((NT & kBufferAddressing) != 0) {
        constexpr uint32_t chunk = kBlock * kGroup * U;
        __amdgpu_buffer_rsrc_t ra = chunk_rsrc(d.a, e0 * 4, chunk * 4);
        __amdgpu_buffer_rsrc_t rb = chunk_rsrc(d.b, e0 * 4, chunk * 4);
        if constexpr (OpK == kFold) {
            using G = Grad<GT>;
            constexpr uint32_t gsz = sizeof(typename G::Vec);
            __amdgpu_buffer_rsrc_t rc = chunk_rsrc(d.c, e0 * sizeof(typename G::Elem), chunk * sizeof(typename G::Elem));
            typename G::Vec g[U];
            f32x4 m[U], v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                uint32_t i = u * kBlock + tid;
                g[u] = buf_ld<ntg, typename G::Vec>(rc, i * gsz);
                m[u] = buf_ld<ntl, f32x4>(ra, i * 16);
                v[u] = buf_ld<ntl, f32x4>(rb, i * 16);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                uint32_t i = u * kBlock + tid;
                fold4(m[u], v[u], G::widen(g[u]), sc);
                buf_st<nts>(ra, i * 16, m[u]);
                buf_st<nts>(rb, i * 16, v[u]);
            }
        } else if constexpr (OpK == kDecay) {
            f32x4 m[U], v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                uint32_t i = u * kBlock + tid;
                m[u] = buf_ld<ntl, f32x4>(ra, i * 16);
                v[u] = buf_ld<ntl, f32x4>(rb, i * 16);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                uint32_t i = u * kBlock + tid;
                decay4(m[u], v[u], sc);
                buf_st<nts>(ra, i * 16, m[u]);
                buf_st<nts>(rb, i * 16, v[u]);
            }
        } else {
            __amdgpu_buffer_rsrc_t rc = chunk_rsrc(d.c, e0 * 4, chunk * 4);
            f32x4 th[U], m[U], v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                uint32_t i = u * kBlock + tid;
                th[u] = buf_ld<ntl, f32x4>(ra, i * 16);
                m[u] = buf_ld<ntl, f32x4>(rb, i * 16);
                v[u] = buf_ld<ntl, f32x4>(rc, i * 16);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                uint32_t i = u * kBlock + tid;
                apply4(th[u], m[u], v[u], sc);
                buf_st<nts>(ra, i * 16, th[u]);
            }
        }
        return;
    }
    ADAMA_GLOBAL f32x4 *A = global_ptr<f32x4>(d.a, e0 * 4);
    ADAMA_GLOBAL f32x4 *B = global_ptr<f32x4>(d.b, e0 * 4);
    if constexpr (OpK == kFold) {
        using G = Grad<GT>;
        const ADAMA_GLOBAL typename G::Vec *C = global_ptr<typename G::Vec>(d.c, e0 * sizeof(typename G::Elem));
        typename G::Vec g[U];
        f32x4 m[U], v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint32_t i = u * kBlock + tid;
            g[u] = ld<ntg>(C + i);
            m[u] = ld<ntl>(A + i);
            v[u] = ld<ntl>(B + i);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint32_t i = u * kBlock + tid;
            f32x4 gf = G::widen(g[u]);
            fold4(m[u], v[u], gf, sc);
            st<nts>(A + i, m[u]);
            st<nts>(B + i, v[u]);
        }
    } else if constexpr (OpK == kDecay) {
        f32x4 m[U], v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint32_t i = u * kBlock + tid;
            m[u] = ld<ntl>(A + i);
            v[u] = ld<ntl>(B + i);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint32_t i = u * kBlock + tid;
            decay4(m[u], v[u], sc);
            st<nts>(A + i, m[u]);
            st<nts>(B + i, v[u]);
        }
    } else {
        const ADAMA_GLOBAL f32x4 *C = global_ptr<f32x4>(d.c, e0 * 4);
        f32x4 th[U], m[U], v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint32_t i = u * kBlock + tid;
            th[u] = ld<ntl>(A + i);
            m[u] = ld<ntl>(B + i);
            v[u] = ld<ntl>(C + i);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            uint32_t i = u * kBlock + tid;
            apply4(th[u], m[u], v[u], sc);
            st<nts>(A + i, th[u]);
        }
    }
}

// ---- one group of a boundary chunk: a full aligned group, or element by element ----
template <int OpK, int GT>
__device__ __forceinline__ void boundary_group(const Desc &d, bool vec, uint32_t pre, uint64_t coord, const Scalars &sc)
{
    int kind = group_kind(vec, pre, d.n, coord);
    if (kind == 0) return;
    ADAMA_GLOBAL float *a = global_ptr<float>(d.a);
    ADAMA_GLOBAL float *b = global_ptr<float>(d.b);
    if (kind == 2) {
        uint64_t e = coord - pre;
        ADAMA_GLOBAL f32x4 *A = global_ptr<f32x4>(d.a, e * 4);
        ADAMA_GLOBAL f32x4 *B = global_ptr<f32x4>(d.b, e * 4);
        if constexpr (OpK == kFold) {
            using G = Grad<GT>;
            f32x4 gf = G::widen(*global_ptr<typename G::Vec>(d.c, e * sizeof(typename G::Elem)));
            f32x4 m = *A, v = *B;
            fold4(m, v, gf, sc);
            *A = m;
            *B = v;
        } else if constexpr (OpK == kDecay) {
            f32x4 m = *A, v = *B;
            decay4(m, v, sc);
            *A = m;
            *B = v;
        } else {
            f32x4 th = *A, m = *B, v = *global_ptr<f32x4>(d.c, e * 4);
            apply4(th, m, v, sc);
            *A = th;
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < kGroup; ++j) {
        uint64_t x = coord + j;
        if (x < pre || x >= pre + d.n) continue;
        uint64_t e = x - pre;
        if constexpr (OpK == kFold) {
            using G = Grad<GT>;
            float g = G::widen1(global_ptr<typename G::Elem>(d.c)[e]);
            float m = a[e], v = b[e];
            fold1(m, v, g, sc);
            a[e] = m;
            b[e] = v;
        } else if constexpr (OpK == kDecay) {
            float m = a[e], v = b[e];
            decay1(m, v, sc);
            a[e] = m;
            b[e] = v;
        } else {
            a[e] = apply1(a[e], b[e], global_ptr<float>(d.c)[e], sc);
        }
    }
}

// OpK: Op.  GT: GradType (fold only).  U: 16-byte groups per thread per chunk (chunk = 1024*U elements).
// NT: cache-policy bits.  Grid: any number of workgroups >= 1; workgroup w takes chunks w, w+grid, ...
//
// The tensor table stays in the kernel argument block and is read with scalar loads: the chunk number
// depends on the workgroup id alone, so the search for its tensor and the fetch of the descriptor are
// wave-uniform and are served by the scalar cache.  (Staging the table in LDS first was measured and
// dropped: in a kernel that saturates the vector memory path, the vector loads that would fill LDS
// queue behind the streaming traffic and delay every workgroup's first data load by microseconds.)
template <int OpK, int GT, int U, int NT>
__global__ void __launch_bounds__(kBlock) multi_tensor_kernel(const Table<kMaxTensors> tab, const Scalars sc)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t count = tab.count;
    constexpr uint32_t chunk = kBlock * kGroup * U;
    constexpr uint32_t c_bytes = OpK == kDecay ? 0u : (OpK == kApply || GT == kF32) ? 4u : 2u;
    const uint32_t total = tab.total;
    for (uint32_t c = blockIdx.x; c < total; c += gridDim.x) {
        const uint32_t k = count > 1 ? find_tensor(tab.chunk_start, count, c) : 0u;
        const Desc d = tab.t[k];
        const uint64_t lc = c - tab.chunk_start[k];
        const uint32_t pre = misalign_elems(d.a);
        const bool vec = coaligned(d.a, d.b, d.c, c_bytes);
        if (chunk_is_interior(vec, pre, d.n, lc, chunk)) {
            interior_chunk<OpK, GT, U, NT>(d, lc * chunk - pre, tid, sc);
        } else {
#pragma unroll 1
            for (int u = 0; u < U; ++u)
                boundary_group<OpK, GT>(d, vec, pre, lc * chunk + (uint64_t)(u * kBlock + tid) * kGroup, sc);
        }
    }
}

}  // namespace adama
