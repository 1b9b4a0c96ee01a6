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
static_assert((int)ADAMA_F32 == kF32 && (int)ADAMA_BF16 == kBF16 && (int)ADAMA_F16 == kF16, "dtype codes");

namespace {

thread_local char g_error[512] = "";

adama_status fail(adama_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof g_error, fmt, ap);
    va_end(ap);
    return st;
}

// ---- tuning constants (measured on MI355X with a sweep over U, grid shape and cache policy) ----
constexpr int kUSmall = 1;                    // chunk = 1024 elements: many workgroups for small launches
constexpr int kUBig = 4;                      // chunk = 4096 elements: 8..12 16-byte loads in flight per thread
// Every byte is touched once per launch and the working set of a layer is far larger than L2 and
// the memory-side cache, so all streams are marked non-temporal: +13 % over default policy.
constexpr int kNtPolicy = kNtGradLoad | kNtStateLoad | kNtStore;
constexpr uint64_t kBigLaunchElems = 1u << 20;   // launches at least this long use kUBig
// One workgroup per chunk: the hardware dispatcher refills a CU as soon as a workgroup retires,
// which beat every persistent grid size tried (2..16 workgroups per CU) by 2..8 %.
constexpr uint32_t kMaxGrid = 1u << 30;
constexpr uint64_t kMaxLaunchElems = ADAMA_MAX_ELEMS;   // keeps the 32-bit chunk numbers of one launch in range

uint32_t grad_bytes(int op, int gdt) { return op == kDecay ? 0u : (op == kApply || gdt == kF32) ? 4u : 2u; }

// One launch: tensors [first, first+count) of the caller's list with their chunk prefix.
struct Batch {
    Table<kMaxTensors> tab;
    int u;                 // groups per thread per chunk
    uint32_t total;        // chunks
};

// Cuts descs[0..count) into launches.  Calls emit(batch, index of its first tensor) for each; stops at the first failure.
template <typename Emit>
adama_status for_each_batch(const Desc *descs, int count, Emit &&emit)
{
    int i = 0;
    while (i < count) {
        Batch b;
        std::memset(&b.tab, 0, sizeof b.tab);
        uint64_t elems = 0;
        int k = 0;
        while (i + k < count && k < kMaxTensors && elems + descs[i + k].n <= kMaxLaunchElems) {
            b.tab.t[k] = descs[i + k];
            elems += descs[i + k].n;
            ++k;
        }
        b.u = elems >= kBigLaunchElems ? kUBig : kUSmall;
        const uint32_t chunk = kBlock * kGroup * b.u;
        uint64_t start = 0;
        for (int j = 0; j < k; ++j) {
            b.tab.chunk_start[j] = (uint32_t)start;
            start += chunks_of(misalign_elems(b.tab.t[j].a), b.tab.t[j].n, chunk);
        }
        b.tab.chunk_start[k] = (uint32_t)start;
        for (int j = k + 1; j < kMaxTensors + 17; ++j) b.tab.chunk_start[j] = 0xFFFFFFFFu;
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

template <int OpK, int GT, int U>
void launch_one(const Batch &b, const Scalars &sc, unsigned grid, hipStream_t stream)
{
    hipLaunchKernelGGL((multi_tensor_kernel<OpK, GT, U, kNtPolicy>), dim3(grid), dim3(kBlock), 0, stream, b.tab, sc);
}

template <int OpK, int GT>
void launch_u(const Batch &b, const Scalars &sc, unsigned grid, hipStream_t stream)
{
    if (b.u == kUBig) launch_one<OpK, GT, kUBig>(b, sc, grid, stream);
    else launch_one<OpK, GT, kUSmall>(b, sc, grid, stream);
}

adama_status launch_all(int op, int gdt, const Desc *descs, int count, const Scalars &sc, hipStream_t stream)
{
    return for_each_batch(descs, count, [&](const Batch &b, int) -> adama_status {
        const unsigned grid = b.total < kMaxGrid ? b.total : kMaxGrid;
        if (op == kDecay) launch_u<kDecay, kF32>(b, sc, grid, stream);
        else if (op == kApply) launch_u<kApply, kF32>(b, sc, grid, stream);
        else if (gdt == kF32) launch_u<kFold, kF32>(b, sc, grid, stream);
        else if (gdt == kBF16) launch_u<kFold, kBF16>(b, sc, grid, stream);
        else launch_u<kFold, kF16>(b, sc, grid, stream);
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

adama_status check_fold_args(const adama_tensor *list, int count, adama_dtype gdt, int N, double beta1, double beta2)
{
    ADAMA_TRY(check_dtype(gdt));
    if (count < 0) return fail(ADAMA_ERR_INVALID_ARG, "count = %d is negative", count);
    if (count > 0 && !list) return fail(ADAMA_ERR_INVALID_ARG, "list is NULL with count = %d", count);
    if (N < 1) return fail(ADAMA_ERR_INVALID_ARG, "N = %d: the number of micro-batches must be >= 1", N);
    if (!unit_interval(beta1) || !unit_interval(beta2))
        return fail(ADAMA_ERR_INVALID_ARG, "beta1 = %g, beta2 = %g must lie in [0, 1)", beta1, beta2);
    const size_t gb = gdt == ADAMA_F32 ? 4 : 2;
    for (int i = 0; i < count; ++i) {
        ADAMA_TRY(check_len(i, list[i].n));
        ADAMA_TRY(check_array("m", i, list[i].m, 4, list[i].n));
        ADAMA_TRY(check_array("v", i, list[i].v, 4, list[i].n));
        ADAMA_TRY(check_array("grad", i, list[i].grad, gb, list[i].n));
    }
    return ADAMA_OK;
}

adama_status check_state_args(const adama_state *list, int count, bool need_theta)
{
    if (count < 0) return fail(ADAMA_ERR_INVALID_ARG, "count = %d is negative", count);
    if (count > 0 && !list) return fail(ADAMA_ERR_INVALID_ARG, "list is NULL with count = %d", count);
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

Scalars fold_scalars(int N, double beta1, double beta2)
{
    const double dn = (double)N;
    return Scalars{(float)((1.0 - beta1) / dn), (float)((1.0 - beta2) / (dn * dn)), 0.0f};
}

Scalars apply_scalars(double lr, double eps, double beta1, double beta2, long long t)
{
    const double bias1 = 1.0 - std::pow(beta1, (double)t);
    const double bias2 = 1.0 - std::pow(beta2, (double)t);
    return Scalars{(float)(lr / bias1), (float)(1.0 / std::sqrt(bias2)), (float)eps};
}

}  // namespace

extern "C" {

const char *adama_last_error(void) { return g_error; }

int adama_max_tensors_per_launch(void) { return kMaxTensors; }

void adama_tuning(int *u_small, int *u_big, unsigned long long *big_launch_elems, int *policy_bits)
{
    if (u_small) *u_small = kUSmall;
    if (u_big) *u_big = kUBig;
    if (big_launch_elems) *big_launch_elems = kBigLaunchElems;
    if (policy_bits) *policy_bits = kNtPolicy;
}

adama_status adama_fold_multi(const adama_tensor *list, int count, adama_dtype gdt, int N, double beta1,
                              double beta2, hipStream_t stream)
{
    ADAMA_TRY(check_fold_args(list, count, gdt, N, beta1, beta2));
    const Scalars sc = fold_scalars(N, beta1, beta2);
    Desc piece[kPiece];
    for (int i = 0; i < count; i += kPiece) {
        int k = count - i < kPiece ? count - i : kPiece;
        for (int j = 0; j < k; ++j) piece[j] = Desc{list[i + j].m, list[i + j].v, list[i + j].grad, list[i + j].n};
        ADAMA_TRY(launch_all(kFold, (int)gdt, piece, k, sc, stream));
    }
    return ADAMA_OK;
}

adama_status adama_fold(float *m, float *v, const void *grad, adama_dtype gdt, size_t n, int N, double beta1,
                        double beta2, hipStream_t stream)
{
    adama_tensor one{m, v, grad, n};
    return adama_fold_multi(&one, 1, gdt, N, beta1, beta2, stream);
}

adama_status adama_begin_step_multi(const adama_state *list, int count, double beta1, double beta2,
                                    hipStream_t stream)
{
    ADAMA_TRY(check_state_args(list, count, false));
    if (!finite_nonneg(beta1) || !finite_nonneg(beta2))
        return fail(ADAMA_ERR_INVALID_ARG, "beta1 = %g, beta2 = %g must be finite and >= 0", beta1, beta2);
    const Scalars sc{(float)beta1, (float)beta2, 0.0f};
    Desc piece[kPiece];
    for (int i = 0; i < count; i += kPiece) {
        int k = count - i < kPiece ? count - i : kPiece;
        for (int j = 0; j < k; ++j) piece[j] = Desc{list[i + j].m, list[i + j].v, nullptr, list[i + j].n};
        ADAMA_TRY(launch_all(kDecay, kF32, piece, k, sc, stream));
    }
    return ADAMA_OK;
}

adama_status adama_begin_step(float *m, float *v, size_t n, double beta1, double beta2, hipStream_t stream)
{
    adama_state one{nullptr, m, v, n};
    return adama_begin_step_multi(&one, 1, beta1, beta2, stream);
}

adama_status adama_apply_multi(const adama_state *list, int count, double lr, double eps, double beta1,
                               double beta2, long long t, hipStream_t stream)
{
    ADAMA_TRY(check_state_args(list, count, true));
    ADAMA_TRY(check_apply_hyper(lr, eps, beta1, beta2, t));
    const Scalars sc = apply_scalars(lr, eps, beta1, beta2, t);
    Desc piece[kPiece];
    for (int i = 0; i < count; i += kPiece) {
        int k = count - i < kPiece ? count - i : kPiece;
        for (int j = 0; j < k; ++j) piece[j] = Desc{list[i + j].theta, list[i + j].m, list[i + j].v, list[i + j].n};
        ADAMA_TRY(launch_all(kApply, kF32, piece, k, sc, stream));
    }
    return ADAMA_OK;
}

adama_status adama_apply(float *theta, const float *m, const float *v, size_t n, double lr, double eps,
                         double beta1, double beta2, long long t, hipStream_t stream)
{
    adama_state one{theta, const_cast<float *>(m), const_cast<float *>(v), n};
    return adama_apply_multi(&one, 1, lr, eps, beta1, beta2, t, stream);
}

adama_status adama_debug_walk(const adama_tensor *list, int count, int op, adama_dtype gdt,
                              unsigned char *const *touched, unsigned long long *vector_accesses,
                              unsigned long long *scalar_accesses, int *launches)
{
    if (op < kDecay || op > kApply) return fail(ADAMA_ERR_INVALID_ARG, "op = %d", op);
    ADAMA_TRY(check_dtype(gdt));
    if (count < 0 || (count > 0 && (!list || !touched))) return fail(ADAMA_ERR_INVALID_ARG, "bad list");
    const uint32_t cb = grad_bytes(op, (int)gdt);
    unsigned long long nvec = 0, nsc = 0;
    int nlaunch = 0;
    for (int i0 = 0; i0 < count; i0 += kPiece) {
        int kp = count - i0 < kPiece ? count - i0 : kPiece;
        Desc piece[kPiece];
        for (int j = 0; j < kp; ++j) piece[j] = Desc{list[i0 + j].m, list[i0 + j].v, list[i0 + j].grad, list[i0 + j].n};
        adama_status st = for_each_batch(piece, kp, [&](const Batch &b, int first) -> adama_status {
            ++nlaunch;
            const uint32_t chunk = kBlock * kGroup * b.u;
            const uint32_t cnt = b.tab.count;
            const int base = i0 + first;   // list index of the batch's first tensor
            for (uint32_t c = 0; c < b.total; ++c) {
                const uint32_t k = find_tensor(b.tab.chunk_start, cnt, c);
                const Desc &d = b.tab.t[k];
                const uint64_t lc = c - b.tab.chunk_start[k];
                const uint32_t pre = misalign_elems(d.a);
                const bool vec = coaligned(d.a, d.b, d.c, cb);
                unsigned char *tch = touched[base + (int)k];
                const bool interior = chunk_is_interior(vec, pre, d.n, lc, chunk);
                for (int u = 0; u < b.u; ++u) {
                    for (uint32_t tid = 0; tid < (uint32_t)kBlock; ++tid) {
                        const uint64_t coord = lc * chunk + (uint64_t)(u * kBlock + tid) * kGroup;
                        int kind = interior ? 2 : group_kind(vec, pre, d.n, coord);
                        if (kind == 2) {
                            if (coord < pre) return fail(ADAMA_ERR_INVALID_ARG, "vector access before tensor %d", base + (int)k);
                            const uint64_t e = coord - pre;
                            if (e + kGroup > d.n) return fail(ADAMA_ERR_INVALID_ARG, "vector access past tensor %d", base + (int)k);
                            const bool ok = aligned_to((const float *)d.a + e, 16) && aligned_to((const float *)d.b + e, 16) &&
                                            (cb == 0 || aligned_to((const char *)d.c + e * cb, 4 * cb));
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
