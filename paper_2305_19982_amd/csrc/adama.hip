// C ABI of libadama (see include/adama.h): argument checking, derivation of the float32 scalars
// from the double hyper-parameters, packing of the per-launch tensor table, kernel launches.
// Host code here never allocates device memory, never synchronises and never touches a default
// stream other than the one the caller passes.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>

#include "adama.h"
#include "adama_kernels.hpp"

using namespace adama;

static_assert(ADAMA_MAX_TENSORS_PER_LAUNCH == kMaxTensors, "header and kernel table size disagree");
static_assert(sizeof(Table<kMaxTensors>) + sizeof(Scalars) <= 4096, "launch table must fit the kernel argument block");
static_assert(sizeof(Desc) == 40, "descriptor layout");
static_assert(kMaxTensors % 16 == 0, "the table search reads whole blocks of 16 entries");
static_assert((int)ADAMA_F32 == kF32 && (int)ADAMA_BF16 == kBF16 && (int)ADAMA_F16 == kF16, "dtype codes");

namespace {

thread_local char g_error[512] = "";

// Identifies the sources and flags this library was built from (the build script passes a hash of
// them); the marker in front lets a build script find it in the file without loading the library.
#ifndef ADAMA_BUILD_ID
#define ADAMA_BUILD_ID "unidentified"
#endif
const char kBuildId[] = "ADAMA_BUILD_ID=" ADAMA_BUILD_ID;

adama_status fail(adama_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof g_error, fmt, ap);
    va_end(ap);
    return st;
}

// ---- launch policy (measured on MI355X: sweeps over workgroup size, groups per thread, grid shape, cache policy) ----
// Every byte is touched once per launch and the working set of a layer is far larger than L2 and
// the memory-side cache, so all streams are marked non-temporal: +12 % over default policy.
constexpr int kNtPolicy = kNtGradLoad | kNtStateLoad | kNtStore;
// The ops (bit = Op) whose streaming stores also carry the agent-scope bit.  What it is worth depends on
// how many workgroups a compute unit holds, so it was measured together with the residency bound
// (in-process A/B on the GPT-2-shaped state): fold +1.2 %, fold with fp32 gradients +2.2 %, first fold
// +1.8 %, SGD folds +0.5 % (+5..9 % on launches of 2^26 elements and more), decay +3.2 % (128 x 1 at 10
// workgroups per compute unit against 128 x 2 plain), fused last fold +2.7 % (128 x 2 at 4), SGD decay
// +2.0 %, SGD update +3.3 %, SGD fused last fold +4.6 % (128 x 1 at 13 against 256 x 2 plain).  The update
// and the rescale gain nothing from it under any bound (-2..-5 % unbounded) and keep plain non-temporal
// stores.
#ifndef ADAMA_SCOPED_STORE_OPS
#define ADAMA_SCOPED_STORE_OPS ((1 << kFold) | (1 << kFoldFirst) | (1 << kSgdFold) | (1 << kSgdFoldFirst) | \
                                (1 << kDecay) | (1 << kFoldLastApply) | (1 << kSgdDecay) | (1 << kSgdApply) | \
                                (1 << kSgdFoldLastApply))
#endif
// Only launches of at least 2^23 elements carry it: a store with the scope bit has to reach memory before its
// kernel can end, which adds about 2 us to a launch and is paid back by the faster streaming of a long one
// only (a launch of 20 small tensors replayed from a HIP graph: 3.8 us without, 4.35 us with).
constexpr int cache_policy(int op, bool long_launch)
{
    return kNtPolicy |
           ((ADAMA_STORE_SCOPE != 0 && long_launch && ((ADAMA_SCOPED_STORE_OPS >> op) & 1)) ? kScopedStore : 0);
}
// One workgroup per chunk (grid == number of chunks): the hardware dispatcher refills a CU as soon as
// a workgroup retires, which beat every persistent grid size tried (2..16 workgroups per CU) by 2..8 %.
constexpr uint64_t kMaxLaunchElems = ADAMA_MAX_ELEMS;   // keeps the 32-bit chunk numbers of one launch in range
constexpr uint64_t kBigLaunchElems = 1u << 20;           // "big" launches: at least this many elements
constexpr uint64_t kHugeLaunchElems = 1u << 26;          // "huge" launches: at least 67.1 M elements
#ifndef ADAMA_LONG_LAUNCH_ELEMS
#define ADAMA_LONG_LAUNCH_ELEMS (1u << 23)
#endif
// a policy's residency bound and store scope apply from this launch length on
constexpr uint64_t kBoundedLaunchElems = ADAMA_LONG_LAUNCH_ELEMS;

// Launch policy per op (index = Op) for small, big and huge launches: threads per workgroup, 16-byte groups
// per thread, and how many workgroups of the launch a compute unit may hold at once (0: no bound).
// Measured per op on MI355X, in one process or as alternating processes on one box, on whole transformer
// blocks (12.6 M .. 315 M elements per launch) and whole-state lists, with realistic array contents
// (all-zero arrays stream 1..3 % faster and respond differently to every knob below, so they are no guide):
//  * the folds and the decay stream best through many small workgroups (128 threads x 1 group =
//    512-element chunks: +2 % on 30 M-element launches over 256 x 1, +4 % over 256 x 2 and 128 x 2; a compute
//    unit refills at a finer grain and the grid's tail is shorter).  Launches of 2^26 elements and more
//    ("huge") differ in the residency bound and, for SGD, in shape: the fold 10 workgroups per compute unit
//    (one-tensor folds of 134 M / 315 M elements: 6619 / 6537 GB/s at 10, 6320 / 6261 unbounded, 5975 / 5863 for
//    the 256 x 4 these launches used while the stores carried no scope bit), the first fold 13 (6611 / 6532
//    against 6512 / 6421 unbounded), the SGD folds 128 x 2 at 10 (6547 / 6570 against 6217 / 6023 for 256 x 2,
//    which stays 2 % ahead at 30 M elements);
//  * the decay (as many bytes written as read) does best with 128 x 1 at 10 workgroups per compute unit and
//    scoped stores (6570 GB/s against 6365 for 128 x 2 unbounded with plain stores), in launches of at most
//    2^26 elements (+2.4 % over 80-tensor launches of 205 M elements);
//  * the plain update does best with 256 x 1 (128 x 1 is 3 % slower there, 256 x 4 is 8 % slower: three
//    read streams and long dependent arithmetic); the fused last fold with 128 x 2 at 4 workgroups per
//    compute unit and scoped stores (6315 against 6150 for 128 x 1 unbounded with plain stores);
//  * the single-moment SGD ops move fewer bytes per element and need two groups per thread to keep
//    enough in flight (128 x 1 costs their fold 13 %): 256 x 2 for the folds below 2^26 elements, 128 x 2 for
//    decay (at 10 workgroups per compute unit) and update (at 8), both with scoped stores;
//  * bounding how many workgroups a compute unit holds (fewer requests in flight) pays together with
//    scoped stores (with plain stores every op but the rescale is flat within 1 % until the launch becomes
//    latency-bound and falls off a cliff): fold 13 (10 from 2^26 elements on), first fold 13 from 2^26 on,
//    decay 10, fused last fold 4, SGD folds 10 from 2^26 on, SGD decay 10, SGD update 8, SGD fused last
//    fold 13.  The data-parallel rescale, which writes three streams with plain stores, gains 7 % with 4
//    workgroups of 128 x 2.  The update runs unbounded.  Launches under 2^23 elements, which need every
//    slot to ramp up, stay unbounded and keep plain stores;
//  * launches under 2^20 elements are latency-bound and use 256 x 1.
struct Policy {
    Shape small, big, huge;
    uint64_t max_launch_elems;   // a list is cut so that no launch of this op exceeds this many elements (0: no such cut)
};
#ifndef ADAMA_POLICY_TABLE
#define ADAMA_POLICY_TABLE {                                                                      \
    /* decay             */ {{256, 1}, {128, 1, 10}, {128, 1, 10}, ADAMA_DECAY_LAUNCH_CAP},       \
    /* fold              */ {{256, 1}, {128, 1, 13}, {128, 1, 10}, 0},                            \
    /* apply             */ {{256, 1}, {256, 1}, {256, 1}, 0},                                    \
    /* fold_first        */ {{256, 1}, {128, 1}, {128, 1, 13}, 0},                                \
    /* fold_last_apply   */ {{256, 1}, {128, 2, 4}, {128, 2, 4}, 0},                              \
    /* rescale_apply     */ {{256, 1}, {128, 2, 4}, {128, 2, 4}, 0},                              \
    /* sgd decay         */ {{256, 1}, {128, 2, 10}, {128, 2, 10}, 0},                            \
    /* sgd fold          */ {{256, 1}, {256, 2}, {128, 2, 10}, 0},                                \
    /* sgd apply         */ {{256, 1}, {128, 2, 8}, {128, 2, 8}, 0},                              \
    /* sgd fold_first    */ {{256, 1}, {256, 2}, {128, 2, 10}, 0},                                \
    /* sgd fold_last_apply */ {{256, 1}, {128, 1, 13}, {128, 1, 13}, 0},                          \
}
#endif
#ifndef ADAMA_DECAY_LAUNCH_CAP
#define ADAMA_DECAY_LAUNCH_CAP (1ull << 26)
#endif
constexpr Policy kPolicy[kNumOps] = ADAMA_POLICY_TABLE;

// Residency override for measurements (adama_debug_set_residency): -1 = the policy's own value.
int g_residency_override[kNumOps][3];
bool g_residency_override_set = false;

// Size class of a launch: 0 small (latency-bound), 1 big, 2 huge.
int launch_class(uint64_t elems) { return elems >= kHugeLaunchElems ? 2 : elems >= kBigLaunchElems ? 1 : 0; }

Shape launch_shape_for(int op, uint64_t elems)
{
    const int cls = launch_class(elems);
    Shape s = cls == 2 ? kPolicy[op].huge : cls == 1 ? kPolicy[op].big : kPolicy[op].small;
    if (elems < kBoundedLaunchElems) s.wgs = 0;
    if (g_residency_override_set && g_residency_override[op][cls] >= 0) s.wgs = g_residency_override[op][cls];
    return s;
}

// A compute unit of this chip has 160 KiB of LDS.  The kernels use none of it; a launch may ask for an
// (unused) share of it per workgroup only to bound how many of its workgroups a compute unit holds at
// once, which bounds the number of memory requests in flight (see the launch policy for where that pays).
constexpr uint32_t kLdsPerComputeUnit = 160u * 1024u;
uint32_t residency_lds_bytes(int wgs_per_cu)
{
    if (wgs_per_cu <= 0) return 0;
    const uint32_t share = (kLdsPerComputeUnit / (uint32_t)wgs_per_cu) & ~1023u;   // whole KiB, rounded down
    return share > 65536u ? 65536u : share;                                      // 64 KiB needs no opt-in
}

uint32_t grad_bytes(int op, int gdt) { return !op_has_grad(op) ? 0u : gdt == kF32 ? 4u : 2u; }

// One launch: tensors [first, first+count) of the caller's list with their chunk prefix.
struct Batch {
    Table<kMaxTensors> tab;
    Shape shape;           // workgroup size and groups per thread
    int size_class;        // 0 small, 1 big, 2 huge: which of the op's three shapes `shape` is
    bool long_launch;      // at least kBoundedLaunchElems elements: residency bound and store scope apply
    uint32_t total;        // chunks
};

// Cuts descs[0..count) into launches.  Calls emit(batch, index of its first tensor) for each; stops at the first failure.
template <typename Emit>
adama_status for_each_batch(int op, const Desc *descs, int count, Emit &&emit)
{
    int i = 0;
    while (i < count) {
        Batch b;
        std::memset(&b.tab, 0, sizeof b.tab);
        uint64_t elems = 0;
        int k = 0;
        const uint64_t cap = kPolicy[op].max_launch_elems ? kPolicy[op].max_launch_elems : kMaxLaunchElems;
        // a tensor longer than the op's cut still goes into a launch of its own (kMaxLaunchElems bounds every tensor)
        while (i + k < count && k < kMaxTensors && (elems + descs[i + k].n <= cap || (k == 0 && descs[i].n <= kMaxLaunchElems))) {
            b.tab.t[k] = descs[i + k];
            elems += descs[i + k].n;
            ++k;
        }
        b.shape = launch_shape_for(op, elems);
        b.size_class = launch_class(elems);
        b.long_launch = elems >= kBoundedLaunchElems;
        const uint32_t chunk = chunk_elems(b.shape);
        uint64_t start = 0;
        for (int j = 0; j < k; ++j) {
            b.tab.chunk_start[j] = (uint32_t)start;
            start += chunks_of(misalign_elems(b.tab.t[j].s[0]), b.tab.t[j].n, chunk);
            b.tab.next_start[j] = (uint32_t)start;
        }
        for (int j = k; j < kMaxTensors + 16; ++j) b.tab.next_start[j] = 0xFFFFFFFFu;
        b.tab.count = (uint32_t)k;
        b.tab.total = (uint32_t)start;
        b.total = (uint32_t)start;
        if (start >= (1ull << 31)) return fail(ADAMA_ERR_TOO_LARGE, "launch of %llu chunks", (unsigned long long)start);
        if (b.total > 0) {
            adama_status st = emit(b, i);
            if (st != ADAMA_OK) return st;
        }
        i += k;
    }
    return ADAMA_OK;
}

template <int OpK, int GT, int BLOCK, int U, int NT>
void launch_one(const Batch &b, const Scalars &sc, hipStream_t stream)
{
    static_assert(BLOCK % 64 == 0 && BLOCK <= kMaxBlock && U >= 1, "workgroup shape");
    const uint32_t lds = residency_lds_bytes(b.shape.wgs);
    if (b.tab.count == 1)
        hipLaunchKernelGGL((multi_tensor_kernel<OpK, GT, BLOCK, U, NT, true>), dim3(b.total), dim3(BLOCK), lds, stream, b.tab, sc);
    else
        hipLaunchKernelGGL((multi_tensor_kernel<OpK, GT, BLOCK, U, NT, false>), dim3(b.total), dim3(BLOCK), lds, stream, b.tab, sc);
}

// Picks the instantiation for the batch's shape, which is one of the op's three.
template <int OpK, int GT>
void launch_u(const Batch &b, const Scalars &sc, hipStream_t stream)
{
    constexpr Policy P = kPolicy[OpK];
    if (b.size_class == 0) launch_one<OpK, GT, P.small.block, P.small.u, cache_policy(OpK, false)>(b, sc, stream);
    else if (b.size_class == 2) launch_one<OpK, GT, P.huge.block, P.huge.u, cache_policy(OpK, true)>(b, sc, stream);
    else if (b.long_launch) launch_one<OpK, GT, P.big.block, P.big.u, cache_policy(OpK, true)>(b, sc, stream);
    else launch_one<OpK, GT, P.big.block, P.big.u, cache_policy(OpK, false)>(b, sc, stream);
}

template <int OpK>
void launch_gdt(int gdt, const Batch &b, const Scalars &sc, hipStream_t stream)
{
    if constexpr (!op_has_grad(OpK)) launch_u<OpK, kF32>(b, sc, stream);
    else if (gdt == kF32) launch_u<OpK, kF32>(b, sc, stream);
    else if (gdt == kBF16) launch_u<OpK, kBF16>(b, sc, stream);
    else launch_u<OpK, kF16>(b, sc, stream);
}

adama_status launch_all(int op, int gdt, const Desc *descs, int count, const Scalars &sc, hipStream_t stream)
{
    return for_each_batch(op, descs, count, [&](const Batch &b, int) -> adama_status {
        switch (op) {
        case kDecay: launch_gdt<kDecay>(gdt, b, sc, stream); break;
        case kFold: launch_gdt<kFold>(gdt, b, sc, stream); break;
        case kApply: launch_gdt<kApply>(gdt, b, sc, stream); break;
        case kFoldFirst: launch_gdt<kFoldFirst>(gdt, b, sc, stream); break;
        case kFoldLastApply: launch_gdt<kFoldLastApply>(gdt, b, sc, stream); break;
        case kRescaleApply: launch_gdt<kRescaleApply>(gdt, b, sc, stream); break;
        case kSgdDecay: launch_gdt<kSgdDecay>(gdt, b, sc, stream); break;
        case kSgdFold: launch_gdt<kSgdFold>(gdt, b, sc, stream); break;
        case kSgdApply: launch_gdt<kSgdApply>(gdt, b, sc, stream); break;
        case kSgdFoldFirst: launch_gdt<kSgdFoldFirst>(gdt, b, sc, stream); break;
        case kSgdFoldLastApply: launch_gdt<kSgdFoldLastApply>(gdt, b, sc, stream); break;
        default: return fail(ADAMA_ERR_INVALID_ARG, "op = %d", op);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(ADAMA_ERR_HIP, "kernel launch: %s", hipGetErrorString(e));
        return ADAMA_OK;
    });
}

// ---- argument checks ----
bool finite_nonneg(double x) { return std::isfinite(x) && x >= 0.0; }
bool unit_interval(double x) { return std::isfinite(x) && x >= 0.0 && x < 1.0; }
bool aligned_to(const void *p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

adama_status check_array(const char *what, int idx, const void *p, size_t elem_bytes, size_t n)
{
    if (n == 0) return ADAMA_OK;
    if (!p) return fail(ADAMA_ERR_INVALID_ARG, "tensor %d: %s is NULL with n = %zu", idx, what, n);
    if (!aligned_to(p, elem_bytes))
        return fail(ADAMA_ERR_INVALID_ARG, "tensor %d: %s (%p) is not aligned to its %zu-byte element", idx, what, p, elem_bytes);
    return ADAMA_OK;
}

adama_status check_len(int idx, size_t n)
{
    if (n > ADAMA_MAX_ELEMS) return fail(ADAMA_ERR_TOO_LARGE, "tensor %d: n = %zu exceeds ADAMA_MAX_ELEMS", idx, n);
    return ADAMA_OK;
}

adama_status check_dtype(adama_dtype gdt)
{
    if (gdt != ADAMA_F32 && gdt != ADAMA_BF16 && gdt != ADAMA_F16)
        return fail(ADAMA_ERR_UNSUPPORTED_DTYPE, "gradient dtype %d is not ADAMA_F32/BF16/F16", (int)gdt);
    return ADAMA_OK;
}

#define ADAMA_TRY(expr) do { adama_status st_ = (expr); if (st_ != ADAMA_OK) return st_; } while (0)

adama_status check_list(int count, const void *list)
{
    if (count < 0) return fail(ADAMA_ERR_INVALID_ARG, "count = %d is negative", count);
    if (count > 0 && !list) return fail(ADAMA_ERR_INVALID_ARG, "list is NULL with count = %d", count);
    return ADAMA_OK;
}

adama_status check_micro_batches(int N)
{
    if (N < 1) return fail(ADAMA_ERR_INVALID_ARG, "N = %d: the number of micro-batches must be >= 1", N);
    return ADAMA_OK;
}

adama_status check_fold_hyper(adama_dtype gdt, int count, const void *list, int N, double beta1, double beta2)
{
    ADAMA_TRY(check_dtype(gdt));
    ADAMA_TRY(check_list(count, list));
    ADAMA_TRY(check_micro_batches(N));
    if (!unit_interval(beta1) || !unit_interval(beta2))
        return fail(ADAMA_ERR_INVALID_ARG, "beta1 = %g, beta2 = %g must lie in [0, 1)", beta1, beta2);
    return ADAMA_OK;
}

// The options of the variant calls; a NULL pointer selects no weight decay and a gradient scale of 1.
struct Options {
    double weight_decay = 0.0, grad_scale = 1.0;
};

adama_status read_options(const adama_options *opt, Options &out)
{
    if (!opt) return ADAMA_OK;
    if (!finite_nonneg(opt->weight_decay))
        return fail(ADAMA_ERR_INVALID_ARG, "weight_decay = %g must be finite and >= 0", opt->weight_decay);
    if (!(std::isfinite(opt->grad_scale) && opt->grad_scale > 0.0))
        return fail(ADAMA_ERR_INVALID_ARG, "grad_scale = %g must be finite and > 0", opt->grad_scale);
    out.weight_decay = opt->weight_decay;
    out.grad_scale = opt->grad_scale;
    return ADAMA_OK;
}

adama_status check_fold_args(const adama_tensor *list, int count, adama_dtype gdt, int N, double beta1, double beta2)
{
    ADAMA_TRY(check_fold_hyper(gdt, count, list, N, beta1, beta2));
    const size_t gb = gdt == ADAMA_F32 ? 4 : 2;
    for (int i = 0; i < count; ++i) {
        ADAMA_TRY(check_len(i, list[i].n));
        ADAMA_TRY(check_array("m", i, list[i].m, 4, list[i].n));
        ADAMA_TRY(check_array("v", i, list[i].v, 4, list[i].n));
        ADAMA_TRY(check_array("grad", i, list[i].grad, gb, list[i].n));
    }
    return ADAMA_OK;
}

adama_status check_update_args(const adama_update_tensor *list, int count, adama_dtype gdt, int N, double beta1,
                               double beta2)
{
    ADAMA_TRY(check_fold_hyper(gdt, count, list, N, beta1, beta2));
    const size_t gb = gdt == ADAMA_F32 ? 4 : 2;
    for (int i = 0; i < count; ++i) {
        ADAMA_TRY(check_len(i, list[i].n));
        ADAMA_TRY(check_array("theta", i, list[i].theta, 4, list[i].n));
        ADAMA_TRY(check_array("m", i, list[i].m, 4, list[i].n));
        ADAMA_TRY(check_array("v", i, list[i].v, 4, list[i].n));
        ADAMA_TRY(check_array("grad", i, list[i].grad, gb, list[i].n));
    }
    return ADAMA_OK;
}

adama_status check_state_args(const adama_state *list, int count, bool need_theta)
{
    ADAMA_TRY(check_list(count, list));
    for (int i = 0; i < count; ++i) {
        ADAMA_TRY(check_len(i, list[i].n));
        if (need_theta) ADAMA_TRY(check_array("theta", i, list[i].theta, 4, list[i].n));
        ADAMA_TRY(check_array("m", i, list[i].m, 4, list[i].n));
        ADAMA_TRY(check_array("v", i, list[i].v, 4, list[i].n));
    }
    return ADAMA_OK;
}

adama_status check_apply_hyper(double lr, double eps, double beta1, double beta2, long long t)
{
    if (t < 1) return fail(ADAMA_ERR_INVALID_ARG, "t = %lld: the step counter is advanced before its first use, so t >= 1", t);
    if (!unit_interval(beta1) || !unit_interval(beta2))
        return fail(ADAMA_ERR_INVALID_ARG, "beta1 = %g, beta2 = %g must lie in [0, 1)", beta1, beta2);
    if (!std::isfinite(lr)) return fail(ADAMA_ERR_INVALID_ARG, "lr = %g is not finite", lr);
    if (!finite_nonneg(eps)) return fail(ADAMA_ERR_INVALID_ARG, "eps = %g must be finite and >= 0", eps);
    return ADAMA_OK;
}

// Descriptor lists are converted in pieces of this many tensors so that no call allocates.
constexpr int kPiece = 4 * kMaxTensors;

// grad_scale == 1 leaves both constants exactly as (1-beta1)/N and (1-beta2)/N^2.
void set_fold_scalars(Scalars &sc, int N, double beta1, double beta2, double grad_scale)
{
    const double dn = (double)N;
    sc.c1 = (float)((1.0 - beta1) * grad_scale / dn);
    sc.c2 = (float)((1.0 - beta2) * (grad_scale * grad_scale) / (dn * dn));
}

// A decay factor as float32 hi + lo, so that the factor the kernel applies is the double to about 1e-15.
void set_decay_scalars(Scalars &sc, double beta1, double beta2)
{
    sc.d1 = (float)beta1;
    sc.d2 = (float)beta2;
    sc.d1lo = (float)(beta1 - (double)sc.d1);
    sc.d2lo = (float)(beta2 - (double)sc.d2);
}

void set_apply_scalars(Scalars &sc, double lr, double eps, double beta1, double beta2, long long t)
{
    const double bias1 = 1.0 - std::pow(beta1, (double)t);
    const double bias2 = 1.0 - std::pow(beta2, (double)t);
    sc.step = (float)(lr / bias1);
    sc.rs2 = (float)(1.0 / std::sqrt(bias2));
    sc.eps = (float)eps;
}

void set_weight_decay(Scalars &sc, double lr, double weight_decay) { sc.wd = (float)(lr * weight_decay); }

adama_status check_sgdm_args(const adama_sgdm_tensor *list, int count, int op, adama_dtype gdt)
{
    ADAMA_TRY(check_list(count, list));
    const size_t gb = gdt == ADAMA_F32 ? 4 : 2;
    for (int i = 0; i < count; ++i) {
        ADAMA_TRY(check_len(i, list[i].n));
        if (op_updates(op)) ADAMA_TRY(check_array("theta", i, list[i].theta, 4, list[i].n));
        ADAMA_TRY(check_array("b", i, list[i].b, 4, list[i].n));
        if (op_has_grad(op)) ADAMA_TRY(check_array("grad", i, list[i].grad, gb, list[i].n));
    }
    return ADAMA_OK;
}

// Converts the caller's list piece by piece with `to_desc` and launches `op` over it.
template <typename T, typename ToDesc>
adama_status run_list(int op, int gdt, const T *list, int count, const Scalars &sc, hipStream_t stream, ToDesc &&to_desc)
{
    Desc piece[kPiece];
    for (int i = 0; i < count; i += kPiece) {
        const int k = count - i < kPiece ? count - i : kPiece;
        for (int j = 0; j < k; ++j) piece[j] = to_desc(list[i + j]);
        ADAMA_TRY(launch_all(op, gdt, piece, k, sc, stream));
    }
    return ADAMA_OK;
}

Desc fold_desc(const adama_tensor &t) { return Desc{{t.m, t.v, nullptr}, t.grad, t.n}; }
Desc update_desc(const adama_update_tensor &t) { return Desc{{t.theta, t.m, t.v}, t.grad, t.n}; }
Desc state_desc(const adama_state &t) { return Desc{{t.theta, t.m, t.v}, nullptr, t.n}; }

// The arrays op `op` uses out of [theta,] m, v, grad: theta leads when the op updates it, the SGD ops
// have no v, and ops without a fold ignore the gradient.
Desc op_desc(int op, float *theta, float *m, float *v, const void *grad, size_t n)
{
    Desc d{{nullptr, nullptr, nullptr}, op_has_grad(op) ? grad : nullptr, n};
    int k = 0;
    if (op_updates(op)) d.s[k++] = theta;
    d.s[k++] = m;
    if (!op_is_sgd(op)) d.s[k++] = v;
    return d;
}

Desc walk_desc(int op, const adama_update_tensor &t) { return op_desc(op, t.theta, t.m, t.v, t.grad, t.n); }

adama_status run_sgdm(int op, adama_dtype gdt, const adama_sgdm_tensor *list, int count, const Scalars &sc,
                      hipStream_t stream)
{
    return run_list(op, (int)gdt, list, count, sc, stream,
                    [op](const adama_sgdm_tensor &t) { return op_desc(op, t.theta, t.b, nullptr, t.grad, t.n); });
}

}  // namespace

extern "C" {

const char *adama_last_error(void) { return g_error; }

int adama_max_tensors_per_launch(void) { return kMaxTensors; }

const char *adama_build_id(void) { return kBuildId + sizeof("ADAMA_BUILD_ID=") - 1; }

int adama_launch_chunk(int op, unsigned long long launch_elems)
{
    if (op < 0 || op >= kNumOps) return 0;
    return (int)chunk_elems(launch_shape_for(op, launch_elems));
}

void adama_tuning(int op, unsigned long long launch_elems, int *block, int *groups_per_thread,
                  unsigned long long *big_launch_elems, int *policy_bits)
{
    const Shape s = (op >= 0 && op < kNumOps) ? launch_shape_for(op, launch_elems) : Shape{0, 0, 0};
    if (block) *block = s.block;
    if (groups_per_thread) *groups_per_thread = s.u;
    if (big_launch_elems) *big_launch_elems = kBigLaunchElems;
    if (policy_bits) *policy_bits = (op >= 0 && op < kNumOps) ? cache_policy(op, launch_elems >= kBoundedLaunchElems) : 0;
}

void adama_debug_set_residency(int op, int size_class, int wgs_per_cu)
{
    if (!g_residency_override_set) {
        for (int o = 0; o < kNumOps; ++o)
            for (int c = 0; c < 3; ++c) g_residency_override[o][c] = -1;
        g_residency_override_set = true;
    }
    if (op < 0 || op >= kNumOps || size_class < 0 || size_class > 2) return;
    g_residency_override[op][size_class] = wgs_per_cu;
}

int adama_residency(int op, unsigned long long launch_elems)
{
    return (op >= 0 && op < kNumOps) ? launch_shape_for(op, launch_elems).wgs : -1;
}

adama_status adama_fold_opt_multi(const adama_tensor *list, int count, adama_dtype gdt, int N, double beta1,
                                  double beta2, const adama_options *opt, hipStream_t stream)
{
    ADAMA_TRY(check_fold_args(list, count, gdt, N, beta1, beta2));
    Options o;
    ADAMA_TRY(read_options(opt, o));
    Scalars sc{};
    set_fold_scalars(sc, N, beta1, beta2, o.grad_scale);
    return run_list(kFold, (int)gdt, list, count, sc, stream, fold_desc);
}

adama_status adama_fold_multi(const adama_tensor *list, int count, adama_dtype gdt, int N, double beta1,
                              double beta2, hipStream_t stream)
{
    return adama_fold_opt_multi(list, count, gdt, N, beta1, beta2, nullptr, stream);
}

adama_status adama_fold(float *m, float *v, const void *grad, adama_dtype gdt, size_t n, int N, double beta1,
                        double beta2, hipStream_t stream)
{
    adama_tensor one{m, v, grad, n};
    return adama_fold_multi(&one, 1, gdt, N, beta1, beta2, stream);
}

adama_status adama_fold_first_opt_multi(const adama_tensor *list, int count, adama_dtype gdt, int N, double beta1,
                                        double beta2, const adama_options *opt, hipStream_t stream)
{
    ADAMA_TRY(check_fold_args(list, count, gdt, N, beta1, beta2));
    Options o;
    ADAMA_TRY(read_options(opt, o));
    Scalars sc{};
    set_fold_scalars(sc, N, beta1, beta2, o.grad_scale);
    set_decay_scalars(sc, beta1, beta2);
    return run_list(kFoldFirst, (int)gdt, list, count, sc, stream, fold_desc);
}

adama_status adama_fold_first_multi(const adama_tensor *list, int count, adama_dtype gdt, int N, double beta1,
                                    double beta2, hipStream_t stream)
{
    return adama_fold_first_opt_multi(list, count, gdt, N, beta1, beta2, nullptr, stream);
}

adama_status adama_fold_first(float *m, float *v, const void *grad, adama_dtype gdt, size_t n, int N,
                              double beta1, double beta2, hipStream_t stream)
{
    adama_tensor one{m, v, grad, n};
    return adama_fold_first_multi(&one, 1, gdt, N, beta1, beta2, stream);
}

adama_status adama_fold_last_apply_opt_multi(const adama_update_tensor *list, int count, adama_dtype gdt, int N,
                                             double lr, double eps, double beta1, double beta2, long long t,
                                             const adama_options *opt, hipStream_t stream)
{
    ADAMA_TRY(check_update_args(list, count, gdt, N, beta1, beta2));
    ADAMA_TRY(check_apply_hyper(lr, eps, beta1, beta2, t));
    Options o;
    ADAMA_TRY(read_options(opt, o));
    Scalars sc{};
    set_fold_scalars(sc, N, beta1, beta2, o.grad_scale);
    set_apply_scalars(sc, lr, eps, beta1, beta2, t);
    set_weight_decay(sc, lr, o.weight_decay);
    return run_list(kFoldLastApply, (int)gdt, list, count, sc, stream, update_desc);
}

adama_status adama_fold_last_apply_multi(const adama_update_tensor *list, int count, adama_dtype gdt, int N,
                                         double lr, double eps, double beta1, double beta2, long long t,
                                         hipStream_t stream)
{
    return adama_fold_last_apply_opt_multi(list, count, gdt, N, lr, eps, beta1, beta2, t, nullptr, stream);
}

adama_status adama_fold_last_apply(float *theta, float *m, float *v, const void *grad, adama_dtype gdt,
                                   size_t n, int N, double lr, double eps, double beta1, double beta2,
                                   long long t, hipStream_t stream)
{
    adama_update_tensor one{theta, m, v, grad, n};
    return adama_fold_last_apply_multi(&one, 1, gdt, N, lr, eps, beta1, beta2, t, stream);
}

adama_status adama_begin_step_multi(const adama_state *list, int count, double beta1, double beta2,
                                    hipStream_t stream)
{
    ADAMA_TRY(check_state_args(list, count, false));
    if (!finite_nonneg(beta1) || !finite_nonneg(beta2))
        return fail(ADAMA_ERR_INVALID_ARG, "beta1 = %g, beta2 = %g must be finite and >= 0", beta1, beta2);
    Scalars sc{};
    set_decay_scalars(sc, beta1, beta2);
    return run_list(kDecay, kF32, list, count, sc, stream,
                    [](const adama_state &t) { return Desc{{t.m, t.v, nullptr}, nullptr, t.n}; });
}

adama_status adama_begin_step(float *m, float *v, size_t n, double beta1, double beta2, hipStream_t stream)
{
    adama_state one{nullptr, m, v, n};
    return adama_begin_step_multi(&one, 1, beta1, beta2, stream);
}

adama_status adama_apply_opt_multi(const adama_state *list, int count, double lr, double eps, double beta1,
                                   double beta2, long long t, const adama_options *opt, hipStream_t stream)
{
    ADAMA_TRY(check_state_args(list, count, true));
    ADAMA_TRY(check_apply_hyper(lr, eps, beta1, beta2, t));
    Options o;
    ADAMA_TRY(read_options(opt, o));
    Scalars sc{};
    set_apply_scalars(sc, lr, eps, beta1, beta2, t);
    set_weight_decay(sc, lr, o.weight_decay);
    return run_list(kApply, kF32, list, count, sc, stream, state_desc);
}

adama_status adama_apply_multi(const adama_state *list, int count, double lr, double eps, double beta1,
                               double beta2, long long t, hipStream_t stream)
{
    return adama_apply_opt_multi(list, count, lr, eps, beta1, beta2, t, nullptr, stream);
}

adama_status adama_apply(float *theta, const float *m, const float *v, size_t n, double lr, double eps,
                         double beta1, double beta2, long long t, hipStream_t stream)
{
    adama_state one{theta, const_cast<float *>(m), const_cast<float *>(v), n};
    return adama_apply_multi(&one, 1, lr, eps, beta1, beta2, t, stream);
}

adama_status adama_rescale_apply_opt_multi(const adama_state *list, int count, double m_scale, double v_scale,
                                           double lr, double eps, double beta1, double beta2, long long t,
                                           const adama_options *opt, hipStream_t stream)
{
    ADAMA_TRY(check_state_args(list, count, true));
    ADAMA_TRY(check_apply_hyper(lr, eps, beta1, beta2, t));
    if (!finite_nonneg(m_scale) || !finite_nonneg(v_scale))
        return fail(ADAMA_ERR_INVALID_ARG, "m_scale = %g, v_scale = %g must be finite and >= 0", m_scale, v_scale);
    Options o;
    ADAMA_TRY(read_options(opt, o));
    Scalars sc{};
    set_decay_scalars(sc, m_scale, v_scale);
    set_apply_scalars(sc, lr, eps, beta1, beta2, t);
    set_weight_decay(sc, lr, o.weight_decay);
    return run_list(kRescaleApply, kF32, list, count, sc, stream, state_desc);
}

adama_status adama_rescale_apply_multi(const adama_state *list, int count, double m_scale, double v_scale, double lr,
                                       double eps, double beta1, double beta2, long long t, hipStream_t stream)
{
    return adama_rescale_apply_opt_multi(list, count, m_scale, v_scale, lr, eps, beta1, beta2, t, nullptr, stream);
}

adama_status adama_rescale_apply(float *theta, float *m, float *v, size_t n, double m_scale, double v_scale,
                                 double lr, double eps, double beta1, double beta2, long long t, hipStream_t stream)
{
    adama_state one{theta, m, v, n};
    return adama_rescale_apply_multi(&one, 1, m_scale, v_scale, lr, eps, beta1, beta2, t, stream);
}

// ---- SGD with momentum ----
adama_status adama_sgdm_begin_step_multi(const adama_sgdm_tensor *list, int count, double momentum, hipStream_t stream)
{
    ADAMA_TRY(check_sgdm_args(list, count, kSgdDecay, ADAMA_F32));
    if (!finite_nonneg(momentum)) return fail(ADAMA_ERR_INVALID_ARG, "momentum = %g must be finite and >= 0", momentum);
    Scalars sc{};
    set_decay_scalars(sc, momentum, 0.0);
    return run_sgdm(kSgdDecay, ADAMA_F32, list, count, sc, stream);
}

adama_status adama_sgdm_fold_multi(const adama_sgdm_tensor *list, int count, adama_dtype gdt, int N,
                                   const adama_options *opt, hipStream_t stream)
{
    ADAMA_TRY(check_dtype(gdt));
    ADAMA_TRY(check_micro_batches(N));
    ADAMA_TRY(check_sgdm_args(list, count, kSgdFold, gdt));
    Options o;
    ADAMA_TRY(read_options(opt, o));
    Scalars sc{};
    sc.c1 = (float)(o.grad_scale / (double)N);
    return run_sgdm(kSgdFold, gdt, list, count, sc, stream);
}

adama_status adama_sgdm_fold_first_multi(const adama_sgdm_tensor *list, int count, adama_dtype gdt, int N,
                                         double momentum, const adama_options *opt, hipStream_t stream)
{
    ADAMA_TRY(check_dtype(gdt));
    ADAMA_TRY(check_micro_batches(N));
    ADAMA_TRY(check_sgdm_args(list, count, kSgdFoldFirst, gdt));
    if (!finite_nonneg(momentum)) return fail(ADAMA_ERR_INVALID_ARG, "momentum = %g must be finite and >= 0", momentum);
    Options o;
    ADAMA_TRY(read_options(opt, o));
    Scalars sc{};
    set_decay_scalars(sc, momentum, 0.0);
    sc.c1 = (float)(o.grad_scale / (double)N);
    return run_sgdm(kSgdFoldFirst, gdt, list, count, sc, stream);
}

adama_status adama_sgdm_apply_multi(const adama_sgdm_tensor *list, int count, double lr, const adama_options *opt,
                                    hipStream_t stream)
{
    ADAMA_TRY(check_sgdm_args(list, count, kSgdApply, ADAMA_F32));
    if (!std::isfinite(lr)) return fail(ADAMA_ERR_INVALID_ARG, "lr = %g is not finite", lr);
    Options o;
    ADAMA_TRY(read_options(opt, o));
    Scalars sc{};
    sc.step = (float)lr;
    set_weight_decay(sc, lr, o.weight_decay);
    return run_sgdm(kSgdApply, ADAMA_F32, list, count, sc, stream);
}

adama_status adama_sgdm_fold_last_apply_multi(const adama_sgdm_tensor *list, int count, adama_dtype gdt, int N,
                                              double lr, const adama_options *opt, hipStream_t stream)
{
    ADAMA_TRY(check_dtype(gdt));
    ADAMA_TRY(check_micro_batches(N));
    ADAMA_TRY(check_sgdm_args(list, count, kSgdFoldLastApply, gdt));
    if (!std::isfinite(lr)) return fail(ADAMA_ERR_INVALID_ARG, "lr = %g is not finite", lr);
    Options o;
    ADAMA_TRY(read_options(opt, o));
    Scalars sc{};
    sc.c1 = (float)(o.grad_scale / (double)N);
    sc.step = (float)lr;
    set_weight_decay(sc, lr, o.weight_decay);
    return run_sgdm(kSgdFoldLastApply, gdt, list, count, sc, stream);
}

adama_status adama_debug_walk(const adama_update_tensor *list, int count, int op, adama_dtype gdt,
                              unsigned char *const *touched, unsigned long long *vector_accesses,
                              unsigned long long *scalar_accesses, int *launches)
{
    if (op < 0 || op >= kNumOps) return fail(ADAMA_ERR_INVALID_ARG, "op = %d", op);
    ADAMA_TRY(check_dtype(gdt));
    if (count < 0 || (count > 0 && (!list || !touched))) return fail(ADAMA_ERR_INVALID_ARG, "bad list");
    const uint32_t gb = grad_bytes(op, (int)gdt);
    const int ns = op_states(op);
    unsigned long long nvec = 0, nsc = 0;
    int nlaunch = 0;
    for (int i0 = 0; i0 < count; i0 += kPiece) {
        const int kp = count - i0 < kPiece ? count - i0 : kPiece;
        Desc piece[kPiece];
        for (int j = 0; j < kp; ++j) piece[j] = walk_desc(op, list[i0 + j]);
        adama_status st = for_each_batch(op, piece, kp, [&](const Batch &b, int first) -> adama_status {
            ++nlaunch;
            const uint32_t chunk = chunk_elems(b.shape);
            const uint32_t cnt = b.tab.count;
            const int base = i0 + first;   // list index of the batch's first tensor
            for (uint32_t c = 0; c < b.total; ++c) {
                const uint32_t k = cnt > 1 ? find_tensor(b.tab.next_start, c) : 0u;
                const Desc &d = b.tab.t[k];
                const uint64_t lc = c - b.tab.chunk_start[k];
                const uint32_t pre = misalign_elems(d.s[0]);
                const bool aligned = coaligned(d, ns, gb);
                unsigned char *tch = touched[base + (int)k];
                const bool interior = chunk_is_interior(pre, d.n, lc, chunk);
                for (int u = 0; u < b.shape.u; ++u) {
                    for (uint32_t tid = 0; tid < (uint32_t)b.shape.block; ++tid) {
                        const uint64_t coord = lc * chunk + (uint64_t)(u * b.shape.block + tid) * kGroup;
                        const int kind = interior ? 2 : group_kind(pre, d.n, coord);
                        if (kind == 2) {
                            if (coord < pre) return fail(ADAMA_ERR_INVALID_ARG, "vector access before tensor %d", base + (int)k);
                            const uint64_t e = coord - pre;
                            if (e + kGroup > d.n) return fail(ADAMA_ERR_INVALID_ARG, "vector access past tensor %d", base + (int)k);
                            // the first state array is always reached on a 16-byte boundary; the others
                            // too when the tensor is co-aligned (then the kernel declares them aligned)
                            bool ok = aligned_to((const float *)d.s[0] + e, 16);
                            if (aligned) {
                                ok = ok && (gb == 0 || aligned_to((const char *)d.g + e * gb, 4 * gb));
                                for (int a = 1; a < ns; ++a) ok = ok && aligned_to((const float *)d.s[a] + e, 16);
                            }
                            if (!ok) return fail(ADAMA_ERR_INVALID_ARG, "misaligned vector access in tensor %d", base + (int)k);
                            for (int j = 0; j < kGroup; ++j) ++tch[e + j];
                            ++nvec;
                        } else if (kind == 1) {
                            for (int j = 0; j < kGroup; ++j) {
                                const uint64_t x = coord + j;
                                if (x < pre || x >= pre + d.n) continue;
                                ++tch[x - pre];
                                ++nsc;
                            }
                        }
                    }
                }
            }
            return ADAMA_OK;
        });
        if (st != ADAMA_OK) return st;
    }
    if (vector_accesses) *vector_accesses = nvec;
    if (scalar_accesses) *scalar_accesses = nsc;
    if (launches) *launches = nlaunch;
    return ADAMA_OK;
}

}  // extern "C"
