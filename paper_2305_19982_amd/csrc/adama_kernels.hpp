// Device kernels of libadama (gfx950).
//
// One kernel template serves the memory-bound elementwise steps of AdamA
// (paper Alg. 2): the once-per-mini-batch moment decay, the per-layer
// per-micro-batch fold, the bias-corrected update, and the two fused edge
// forms (decay inside the first micro-batch's fold, update inside the last
// one's).  Each is a pure stream:
//
//   decay           : read m, v                 write m, v          16 B / element
//   fold            : read grad, m, v           write m, v          16 + sizeof(grad)
//   apply           : read theta, m, v          write theta         16
//   fold_first      : as fold (the decay rides along)               16 + sizeof(grad)
//   fold_last_apply : read grad, theta, m, v    write theta, m, v   24 + sizeof(grad)
//   rescale_apply   : read theta, m, v          write theta, m, v   24
//
// and the same five steps for SGD with momentum, which keeps one moment (the buffer b):
//
//   sgd decay 8, sgd fold / fold_first 8 + sizeof(grad), sgd apply 12, sgd fold_last_apply 16 + sizeof(grad)
//
// so the design goal is HBM bandwidth, not arithmetic: no MFMA, no LDS tiling of
// data (there is no reuse), only wide coalesced accesses and enough of them in
// flight.  A workgroup of BLOCK threads handles one chunk of BLOCK*4*U elements;
// inside an interior chunk each thread issues all of its U 16-byte loads per
// array before the first use, so a wavefront has U..4U independent 1-KiB
// requests outstanding.  The table of tensors of the launch arrives in the
// kernel argument block, together with the per-tensor chunk prefix that maps a
// chunk number to its tensor; both are read through the scalar cache.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "adama_index.hpp"

namespace adama {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
// The same vectors declared with the alignment of one element only.  The compiler still emits one
// wide memory instruction for them on this target (unaligned global accesses are part of the HSA
// memory model); it would split them itself on a target without that guarantee.
typedef float f32x4_u __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t u32x2_u __attribute__((ext_vector_type(2), aligned(2)));
typedef _Float16 f16x4_u __attribute__((ext_vector_type(4), aligned(2)));

enum GradType : int { kF32 = 0, kBF16 = 1, kF16 = 2 };

// Every data pointer of a launch is device global memory; say so, so that the compiler emits global
// (not flat) loads and stores, which return in order and let the hardware counters wait for the
// oldest of many outstanding loads.
#define ADAMA_GLOBAL __attribute__((address_space(1)))
template <typename T>
__device__ __forceinline__ ADAMA_GLOBAL T *global_ptr(const void *p, uint64_t byte_offset = 0)
{
    return (ADAMA_GLOBAL T *)(reinterpret_cast<uintptr_t>(p) + byte_offset);
}

// Cache-policy bits of a kernel instantiation: which streams use non-temporal accesses.
enum : int { kNtGradLoad = 1, kNtStateLoad = 2, kNtStore = 4, kScopedStore = 8 };

// Per-launch scalars, already rounded to float32 from double on the host.
//   c1 = (1-beta1)/N, c2 = (1-beta2)/N^2            fold, fold_first, fold_last_apply
//        (with a gradient scale s: c1 = (1-beta1) s/N, c2 = (1-beta2) (s/N)^2;  SGD: c1 = s/N)
//   d1 = beta1, d2 = beta2                           decay, fold_first (rescale_apply: 1/M, 1/M^2;  SGD: d1 = momentum)
//   d1lo, d2lo = the part of each factor that float32 d1, d2 miss (factor - (double)d)
//   step = lr/(1-beta1^t), rs2 = 1/sqrt(1-beta2^t), eps     apply, fold_last_apply, rescale_apply  (SGD: step = lr)
//   wd = lr*lambda                                   decoupled weight decay of the updates; 0 = none
struct Scalars {
    float c1, c2, d1, d2, step, rs2, eps, wd, d1lo, d2lo;
};

template <bool NT, typename T>
__device__ __forceinline__ T ld(const ADAMA_GLOBAL T *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

// Scope bits on the streaming stores of the interior path of the ops whose policy carries kScopedStore
// (ADAMA_STORE_SCOPE): 1 = "sc1 nt" (agent scope), 2 = "sc0 sc1 nt" (system scope), 0 = never, i.e. "nt"
// alone, which is what __builtin_nontemporal_store emits.  A wider scope than the program needs is always
// correct: it only tells the caches to write the line through sooner.  Measured on 18 GB of realistic
// state: with the fold's access mix and none of its arithmetic, stores with sc1 set stream about 1 % faster
// than plain non-temporal ones (8 % faster on their own); what the kernels gain depends on the op and on how
// many workgroups a compute unit holds, so the bit is part of the per-op launch policy.
#ifndef ADAMA_STORE_SCOPE
#define ADAMA_STORE_SCOPE 1
#endif

template <bool NT, typename T>
__device__ __forceinline__ void st(ADAMA_GLOBAL T *p, T x)
{
    if constexpr (NT) __builtin_nontemporal_store(x, p);
    else *p = x;
}

// One 16-byte streaming store.  The compiler has no builtin that sets the scope bits of a non-temporal
// store (a volatile qualifier is dropped by the builtin), hence the instruction is written out.
//  - Every operand is a vector register: the hardware interlocks on those.  (A scalar-register base
//    written by v_readfirstlane would need five wait states before a memory instruction may read it,
//    which the compiler's hazard pass does not insert around inline assembly.)
//  - The trailing s_nop is the one wait state a store of more than 8 bytes needs before a vector
//    instruction may overwrite its data registers; the compiler cannot see that either.
//  - No "memory" clobber: the data operand orders the store after the load it depends on, and nothing
//    in the kernel reads the location again.
template <typename T>
__device__ __forceinline__ void st_stream16(ADAMA_GLOBAL T *p, T x)
{
    static_assert(sizeof(T) == 16, "one dwordx4 store");
#if ADAMA_STORE_SCOPE == 1
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 0" : : "v"(p), "v"(x));
#elif ADAMA_STORE_SCOPE == 2
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 0" : : "v"(p), "v"(x));
#else
    __builtin_nontemporal_store(x, p);
#endif
}

// ---- gradient storage formats: 4-element vector type, element type, exact widening to float32 ----
template <int GT> struct Grad;

template <> struct Grad<kF32> {
    using Vec = f32x4;
    using VecU = f32x4_u;
    using Elem = float;
    static __device__ __forceinline__ f32x4 widen(f32x4 g) { return g; }
    static __device__ __forceinline__ float widen1(float g) { return g; }
};

template <> struct Grad<kBF16> {   // bfloat16 is the upper half of a float32 word
    using Vec = u32x2;
    using VecU = u32x2_u;
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
    using VecU = f16x4_u;
    using Elem = _Float16;
    static __device__ __forceinline__ f32x4 widen(f16x4 h) { return __builtin_convertvector(h, f32x4); }
    static __device__ __forceinline__ float widen1(_Float16 h) { return (float)h; }
};

// ---- the arithmetic, one element at a time ----
// s[] holds the element of each state array of the op (see op_states): [theta,] m, v or [theta,] b.
// Every product and sum below is rounded on its own (contraction is off), so a fused edge form
// produces the very bits the separate steps would.
//
//   decay  (Alg. 2, first line of the loop):  m <- beta1*m, v <- beta2*v.  The factor is applied as
//                                             hi*x + lo*x with hi = float32(beta), lo = beta - hi: float32(0.999)
//                                             alone is 1.3e-8 too large, and since v averages over ~1000
//                                             mini-batches that bias would compound to 1.3e-5 of v
//   fold   (Alg. 2, inner body):              m <- m + c1*g, v <- v + c2*g^2   (g the raw gradient;
//                                             g*g is exact in float32 for bf16 and fp16 inputs)
//   apply  (Alg. 2, Update):                  theta <- theta - step*m / (sqrt(v)*rs2 + eps)
//                                             = theta - lr*m_hat/(sqrt(v_hat)+eps); IEEE sqrt and divide
//   rescale_apply (Sec. 3.3, after Eq. 5):    m <- m/M, v <- v/M^2 on the all-reduced sums, then apply
//
// Variants the paper's Discussion (Sec. 5) points at (the same scheme for other momentum-based optimizers):
//   decoupled weight decay:  theta <- theta - (lr*lambda*theta + Adam step); the two are summed first
//                            so theta is rounded once.  With wd == 0 the plain expression is selected,
//                            bit for bit.
//   SGD with momentum:       b <- mu*b;  b <- b + c1*g;  theta <- theta - (lr*lambda*theta + lr*b)
// x * (hi + lo) with one rounding at x's magnitude: the small product is rounded first, the fused
// multiply-add rounds the sum.  With lo == 0 (a factor float32 holds exactly) this is hi * x.  An
// infinite x also takes hi * x: lo may be negative (float32(0.999) is above 0.999), and then
// hi * inf + lo * inf would be inf - inf = NaN where the product x * (hi + lo) is plainly infinite.
// (A NaN stays a NaN on either route.)
__device__ __forceinline__ float scale_hi_lo(float hi, float lo, float x)
{
    const float whole = __builtin_fmaf(hi, x, lo * x);
    const bool split = lo != 0.0f && __builtin_fabsf(x) < __builtin_inff();
    return split ? whole : hi * x;
}

template <int OpK>
__device__ __forceinline__ void element_op(float (&s)[3], float g, const Scalars &sc)
{
    constexpr int im = op_updates(OpK) ? 1 : 0, iv = im + 1;
    if constexpr (op_decays(OpK)) {
        s[im] = scale_hi_lo(sc.d1, sc.d1lo, s[im]);
        if constexpr (!op_is_sgd(OpK)) s[iv] = scale_hi_lo(sc.d2, sc.d2lo, s[iv]);
    }
    if constexpr (op_has_grad(OpK)) {
        s[im] = __builtin_fmaf(sc.c1, g, s[im]);
        if constexpr (!op_is_sgd(OpK)) s[iv] = __builtin_fmaf(sc.c2, g * g, s[iv]);
    }
    if constexpr (op_updates(OpK)) {
        float delta;
        if constexpr (op_is_sgd(OpK)) {
            delta = sc.step * s[im];
        } else {
            const float denom = __builtin_fmaf(__builtin_sqrtf(s[iv]), sc.rs2, sc.eps);
            delta = (sc.step * s[im]) / denom;
        }
        const float decayed = __builtin_fmaf(sc.wd, s[0], delta);
        s[0] = s[0] - (sc.wd != 0.0f ? decayed : delta);
    }
}

// The table search of adama_index.hpp's find_tensor, spelled for the scalar unit: the chunk number is
// wave-uniform, so every compare runs on the scalar ALU.  Each entry costs one compare and one
// add-with-carry (the compare's result is the carry); written this way the compiler cannot route half of
// the compares through the vector unit and back, which it does for the portable form.  Same result as
// find_tensor for every input (the GPU tests compare list launches with single-tensor launches bitwise).
#ifndef ADAMA_SEARCH
#define ADAMA_SEARCH 1
#endif
__device__ __forceinline__ uint32_t find_tensor_scalar(const uint32_t *next, uint32_t c)
{
#if ADAMA_SEARCH == 0
    return find_tensor(next, c);
#else
    typedef uint32_t u32x16 __attribute__((ext_vector_type(16), aligned(4)));
    uint32_t k = 0;
    for (uint32_t base = 0;; base += 16) {
        const u32x16 block = *reinterpret_cast<const u32x16 *>(next + base);     // one 64-byte scalar load
        uint32_t hits = 0;
#pragma unroll
        for (uint32_t j = 0; j < 16; ++j) {
            const uint32_t s = block[j];
#if ADAMA_SEARCH == 1
            asm("s_cmp_le_u32 %1, %2\n\ts_addc_u32 %0, %0, 0" : "+s"(hits) : "s"(s), "s"(c) : "scc");
#else
            hits += 1u - ((c - s) >> 31);       // entries and c stay below 2^31; sentinels are 0xFFFFFFFF: c + 1 < 2^31
#endif
        }
        k += hits;
        if (hits < 16) break;
    }
    return k;
#endif
}

// Picks the aligned or the element-aligned flavour of a vector type.
template <bool ALIGNED, typename A, typename U_> struct Pick { using T = A; };
template <typename A, typename U_> struct Pick<false, A, U_> { using T = U_; };

// ---- one interior chunk: every group is a full group; all loads first ----
// ALIGNED: the tensor's arrays are co-aligned, so every access falls on a 16-byte boundary (8-byte for
// 16-bit gradients); otherwise the accesses are declared element-aligned.
template <int OpK, int GT, int BLOCK, int U, int NT, bool ALIGNED>
__device__ __forceinline__ void interior_chunk(const Desc &d, uint64_t e0, uint32_t tid, const Scalars &sc)
{
    constexpr bool ntg = (NT & kNtGradLoad) != 0, ntl = (NT & kNtStateLoad) != 0, nts = (NT & kNtStore) != 0;
    constexpr bool scoped = nts && (NT & kScopedStore) != 0;
    constexpr int NS = op_states(OpK);
    using G = Grad<GT>;
    using SV = typename Pick<ALIGNED, f32x4, f32x4_u>::T;
    using GV = typename Pick<ALIGNED, typename G::Vec, typename G::VecU>::T;
    ADAMA_GLOBAL SV *S[NS];
#pragma unroll
    for (int k = 0; k < NS; ++k) S[k] = global_ptr<SV>(d.s[k], e0 * 4);
    const ADAMA_GLOBAL GV *Gp = global_ptr<GV>(d.g, e0 * sizeof(typename G::Elem));
    typename G::Vec g[U];
    f32x4 x[NS][U];
    // All loads first, then, group by group, arithmetic and stores: a group's stores are issued as soon
    // as its own loads have landed, while later groups' loads are still in flight.  The instruction
    // scheduler is left free here on purpose.  Measured on 18 GB of state: holding every store back
    // until all arithmetic is done costs 4 %, array-major order (all of g, all of m, all of v; stores
    // likewise) costs 4 %, and pinning any fixed load order with scheduling barriers costs 1 %.
    // (On small footprints array-major wins by 2 % instead; the order that holds up at scale is kept.)
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t i = u * BLOCK + tid;
        if constexpr (op_has_grad(OpK)) g[u] = ld<ntg>(Gp + i);
#pragma unroll
        for (int k = 0; k < NS; ++k) x[k][u] = ld<ntl>(S[k] + i);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t i = u * BLOCK + tid;
        f32x4 gf = {0.0f, 0.0f, 0.0f, 0.0f};
        if constexpr (op_has_grad(OpK)) gf = G::widen(g[u]);
#pragma unroll
        for (int j = 0; j < kGroup; ++j) {
            float e[3] = {0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int k = 0; k < NS; ++k) e[k] = x[k][u][j];
            element_op<OpK>(e, gf[j], sc);
#pragma unroll
            for (int k = 0; k < NS; ++k) x[k][u][j] = e[k];
        }
#pragma unroll
        for (int k = 0; k < NS; ++k)
            if ((op_store_mask(OpK) >> k) & 1) {
                if constexpr (scoped) st_stream16(S[k] + i, (SV)x[k][u]);
                else st<nts>(S[k] + i, (SV)x[k][u]);
            }
    }
}

// ---- one group of a boundary chunk: a full group (one wide access per array), or element by element ----
template <int OpK, int GT>
__device__ __forceinline__ void boundary_group(const Desc &d, bool aligned, uint32_t pre, uint64_t coord, const Scalars &sc)
{
    constexpr int NS = op_states(OpK);
    using G = Grad<GT>;
    const int kind = group_kind(pre, d.n, coord);
    if (kind == 0) return;
    if (kind == 2) {
        const uint64_t e = coord - pre;
        f32x4 x[NS];
        f32x4 gf = {0.0f, 0.0f, 0.0f, 0.0f};
        if (aligned) {
#pragma unroll
            for (int k = 0; k < NS; ++k) x[k] = *global_ptr<f32x4>(d.s[k], e * 4);
            if constexpr (op_has_grad(OpK)) gf = G::widen(*global_ptr<typename G::Vec>(d.g, e * sizeof(typename G::Elem)));
        } else {
#pragma unroll
            for (int k = 0; k < NS; ++k) x[k] = *global_ptr<f32x4_u>(d.s[k], e * 4);
            if constexpr (op_has_grad(OpK)) gf = G::widen(*global_ptr<typename G::VecU>(d.g, e * sizeof(typename G::Elem)));
        }
#pragma unroll
        for (int j = 0; j < kGroup; ++j) {
            float el[3] = {0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int k = 0; k < NS; ++k) el[k] = x[k][j];
            element_op<OpK>(el, gf[j], sc);
#pragma unroll
            for (int k = 0; k < NS; ++k) x[k][j] = el[k];
        }
#pragma unroll
        for (int k = 0; k < NS; ++k)
            if ((op_store_mask(OpK) >> k) & 1) {
                if (aligned) *global_ptr<f32x4>(d.s[k], e * 4) = x[k];
                else *global_ptr<f32x4_u>(d.s[k], e * 4) = (f32x4_u)x[k];
            }
        return;
    }
#pragma unroll
    for (int j = 0; j < kGroup; ++j) {
        const uint64_t xc = coord + j;
        if (xc < pre || xc >= pre + d.n) continue;
        const uint64_t e = xc - pre;
        float el[3] = {0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int k = 0; k < NS; ++k) el[k] = global_ptr<float>(d.s[k])[e];
        float g = 0.0f;
        if constexpr (op_has_grad(OpK)) g = G::widen1(global_ptr<typename G::Elem>(d.g)[e]);
        element_op<OpK>(el, g, sc);
#pragma unroll
        for (int k = 0; k < NS; ++k)
            if ((op_store_mask(OpK) >> k) & 1) global_ptr<float>(d.s[k])[e] = el[k];
    }
}

// OpK: Op.  GT: GradType (ops with a gradient).  BLOCK: threads per workgroup.  U: 16-byte groups per
// thread per chunk (chunk = BLOCK*4*U elements).  NT: cache-policy bits.  SINGLE: the launch holds
// exactly one tensor.
// Launch contract: gridDim.x == tab.total, one workgroup per chunk.
//
// The tensor table stays in the kernel argument block and is read with scalar loads: the chunk number
// is the workgroup id, so the search for its tensor and the fetch of the descriptor are wave-uniform
// and are served by the scalar cache.  Nothing the first data load depends on takes more than two
// scalar-load round trips (one for a single-tensor launch).  (Staging the table in LDS first was
// measured and dropped: in a kernel that saturates the vector memory path, the vector loads that
// would fill LDS queue behind the streaming traffic and delay every workgroup's first data load.)
template <int OpK, int GT, int BLOCK, int U, int NT, bool SINGLE>
__global__ void __launch_bounds__(BLOCK) multi_tensor_kernel(const Table<kMaxTensors> tab, const Scalars sc)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t c = blockIdx.x;
    constexpr uint32_t chunk = BLOCK * kGroup * U;
    constexpr uint32_t g_bytes = !op_has_grad(OpK) ? 0u : GT == kF32 ? 4u : 2u;
    const uint32_t k = SINGLE ? 0u : find_tensor_scalar(tab.next_start, c);
    const Desc d = tab.t[k];
    const uint64_t lc = SINGLE ? c : c - tab.chunk_start[k];
    const uint32_t pre = misalign_elems(d.s[0]);
    const bool aligned = coaligned(d, op_states(OpK), g_bytes);
    if (chunk_is_interior(pre, d.n, lc, chunk)) {
        if (aligned) interior_chunk<OpK, GT, BLOCK, U, NT, true>(d, lc * chunk - pre, tid, sc);
        else interior_chunk<OpK, GT, BLOCK, U, NT, false>(d, lc * chunk - pre, tid, sc);
    } else {
#pragma unroll 1
        for (int u = 0; u < U; ++u)
            boundary_group<OpK, GT>(d, aligned, pre, lc * chunk + (uint64_t)(u * BLOCK + tid) * kGroup, sc);
    }
}

}  // namespace adama
