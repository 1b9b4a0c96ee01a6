// Launch geometry shared by the kernels and by the host-side geometry walk.
//
// One launch processes up to kMaxTensors tensors.  Each tensor is cut into
// chunks of `chunk` elements (see Shape) measured in "aligned coordinates": element e of a
// tensor sits at coordinate pre + e, where pre (0..3) is the number of float32
// elements by which the tensor's first state array is past a 16-byte boundary.
// Coordinates that are multiples of 4 therefore fall on 16-byte boundaries of
// the first state array, whatever the tensor's start address.  Every 4-element
// group wholly inside the tensor is moved with one wide access per array:
// aligned when the other arrays of the tensor share that misalignment
// ("co-aligned"), otherwise declared with element alignment only, which the
// hardware serves by splitting an access where it straddles a boundary.  The at
// most one partial group at either end is moved element by element.
#pragma once

#include <stdint.h>

#if defined(__HIPCC__)
#define ADAMA_HD __host__ __device__ inline
#else
#define ADAMA_HD inline
#endif

namespace adama {

constexpr int kMaxBlock = 256;    // largest workgroup any launch uses: four 64-wide wavefronts
constexpr int kGroup = 4;         // elements per 16-byte float32 access
constexpr int kMaxTensors = 80;   // descriptors per launch (table lives in the kernel argument block)

// The steps of the path.  "First" folds perform the mini-batch's decay on the way (micro-batch 0),
// "LastApply" folds perform the parameter update on the way (micro-batch N-1).  "RescaleApply" is the
// update of the data-parallel scheme: the all-reduced moments are rescaled, written back, and used.
// The kSgd* ops are the same five steps for SGD with momentum, whose only moment is the buffer b.
enum Op : int {
    kDecay = 0, kFold = 1, kApply = 2, kFoldFirst = 3, kFoldLastApply = 4, kRescaleApply = 5,
    kSgdDecay = 6, kSgdFold = 7, kSgdApply = 8, kSgdFoldFirst = 9, kSgdFoldLastApply = 10,
    kNumOps = 11
};

ADAMA_HD constexpr bool op_is_sgd(int op) { return op >= kSgdDecay && op <= kSgdFoldLastApply; }
// The op scales the moments first (by beta1, beta2 / the momentum / the all-reduce factors).
ADAMA_HD constexpr bool op_decays(int op)
{
    return op == kDecay || op == kFoldFirst || op == kRescaleApply || op == kSgdDecay || op == kSgdFoldFirst;
}
// The op reads a gradient and folds it into the moments.
ADAMA_HD constexpr bool op_has_grad(int op)
{
    return op == kFold || op == kFoldFirst || op == kFoldLastApply || op == kSgdFold || op == kSgdFoldFirst ||
           op == kSgdFoldLastApply;
}
// The op ends with the parameter update; theta is then state array 0 and the moments follow it.
ADAMA_HD constexpr bool op_updates(int op)
{
    return op == kApply || op == kFoldLastApply || op == kRescaleApply || op == kSgdApply || op == kSgdFoldLastApply;
}
// Number of float32 state arrays an op touches: s = [theta,] m, v for the Adam ops, [theta,] b for the SGD ops.
ADAMA_HD constexpr int op_states(int op) { return (op_updates(op) ? 1 : 0) + (op_is_sgd(op) ? 1 : 2); }
// Bit k set: state array k is written back.  A plain update leaves the moments untouched.
ADAMA_HD constexpr int op_store_mask(int op)
{
    return (op == kApply || op == kSgdApply) ? 1 : (1 << op_states(op)) - 1;
}

// Shape of a launch's workgroups: `block` threads, each moving `u` 4-element groups per array, so one
// workgroup handles a chunk of block * 4 * u elements; `wgs` = how many workgroups of the launch a
// compute unit may hold at once (0: as many as fit).
struct Shape {
    int block, u, wgs;
};
ADAMA_HD constexpr uint32_t chunk_elems(Shape s) { return (uint32_t)(s.block * kGroup * s.u); }
ADAMA_HD constexpr bool same_shape(Shape a, Shape b) { return a.block == b.block && a.u == b.u; }

// The arrays of one tensor: up to three float32 state arrays and the gradient.
struct Desc {
    void *s[3];
    const void *g;
    uint64_t n;
};

template <int MaxT>
struct Table {
    // next_start[k] = number of chunks of tensors 0..k (= first chunk of tensor k+1; [count-1] = total);
    // entries from [count] on = 0xFFFFFFFF.  It leads the table so that the first 16-entry block of
    // find_tensor is one aligned 64-byte read of the kernel argument block.
    uint32_t next_start[MaxT + 16];
    Desc t[MaxT];
    uint32_t chunk_start[MaxT];       // chunk_start[k] = first chunk of tensor k
    uint32_t count;
    uint32_t total;                   // number of chunks of the launch
};

// Misalignment of the first state array, in float32 elements (0..3).
ADAMA_HD uint32_t misalign_elems(const void *a) { return (uint32_t)(((uintptr_t)a >> 2) & (kGroup - 1)); }

// True when every state array of the op, and the gradient (elements of g_bytes bytes) if the op
// reads one, reaches a 16-byte boundary at the same element index as the first state array does.
ADAMA_HD bool coaligned(const Desc &d, int n_states, uint32_t g_bytes)
{
    const uint32_t pre = misalign_elems(d.s[0]);
    for (int k = 1; k < n_states; ++k)
        if ((((uintptr_t)d.s[k] >> 2) & (kGroup - 1)) != pre) return false;
    if (g_bytes == 0) return true;
    const uint32_t shift = g_bytes == 4 ? 2 : 1;
    return (((uintptr_t)d.g >> shift) & (kGroup - 1)) == pre;
}

ADAMA_HD uint64_t chunks_of(uint32_t pre, uint64_t n, uint32_t chunk)
{
    return n == 0 ? 0 : (pre + n + chunk - 1) / chunk;
}

// The tensor that owns chunk c, given 0 <= c < total: the number of tensors that end at or before c,
// i.e. the number of entries of next[] that are <= c (next[] is non-decreasing and every entry past
// the launch's tensors is 0xFFFFFFFF).  A zero-length tensor ends where it starts, so it is counted
// together with its predecessor and never owns a chunk.  Entries are counted in blocks of 16 whose
// loads do not depend on one another (one scalar-cache latency per block instead of one per bisection
// step); a block with fewer than 16 hits ends the search, so the tensor count itself is never read
// and a launch of up to 16 tensors needs a single block.
template <typename NextArray>
ADAMA_HD uint32_t find_tensor(const NextArray &next, uint32_t c)
{
    uint32_t k = 0;
    for (uint32_t base = 0;; base += 16) {
        uint32_t hits = 0;
#if defined(__HIPCC__)
#pragma unroll
#endif
        for (uint32_t j = 0; j < 16; ++j) hits += (next[base + j] <= c) ? 1u : 0u;
        k += hits;
        if (hits < 16) break;
    }
    return k;
}

// Chunk lc of a tensor covers coordinates [lc*chunk, (lc+1)*chunk).  It is "interior" when the
// whole coordinate range lies inside [pre, pre+n): then every group of the chunk is a full group.
ADAMA_HD bool chunk_is_interior(uint32_t pre, uint64_t n, uint64_t lc, uint32_t chunk)
{
    uint64_t lo = lc * chunk;
    return lo >= pre && lo + chunk <= pre + n;
}

// How the group at coordinate `coord` (a multiple of 4) is moved: 2 = one wide access per array,
// 1 = element by element (only elements inside the tensor), 0 = nothing to do.
ADAMA_HD int group_kind(uint32_t pre, uint64_t n, uint64_t coord)
{
    if (coord + kGroup <= pre || coord >= pre + n) return 0;
    if (coord >= pre && coord + kGroup <= pre + n) return 2;
    return 1;
}

}  // namespace adama
