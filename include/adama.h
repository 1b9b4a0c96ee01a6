/*
 * libadama -- the AdamA (Adam Accumulation) optimizer hot path for AMD MI355X (gfx950).
 *
 * AdamA folds every freshly produced gradient tensor straight into Adam's first
 * and second moments, once per layer per micro-batch, so the gradient buffer can
 * be released at once instead of being accumulated over the mini-batch (paper,
 * Sec. 3.1, Alg. 1 red variant and Alg. 2).  One mini-batch is
 *
 *     adama_begin_step            m <- beta1 m, v <- beta2 v        (Alg. 2, first line of the loop)
 *     N x layers x adama_fold*    m += (1-beta1) g, v += (1-beta2) g^2, g = grad/N   (Alg. 2, inner body)
 *     adama_apply                 bias-corrected parameter update     (Alg. 2, "Update")
 *
 * or, with the same results bit for bit and 24 fewer bytes of memory traffic per parameter,
 *
 *     layers x adama_fold_first*         micro-batch 0: the decay rides along with the fold
 *     (N-2) x layers x adama_fold*       micro-batches 1 .. N-2
 *     layers x adama_fold_last_apply*    micro-batch N-1: the update rides along with the fold
 *
 * Conventions common to every call
 *  - All data pointers are DEVICE pointers owned by the caller; `list` arrays of
 *    descriptors are HOST memory and are consumed before the call returns.
 *  - m, v, theta are float32.  Gradients are float32, bfloat16 or float16 (adama_dtype).
 *    Pointers need only their natural element alignment.  Every array is moved with
 *    wide (16-byte; 8-byte for 16-bit gradients) accesses whatever its alignment; when the
 *    arrays of a tensor do not share the same offset from a 16-byte boundary, some of those
 *    accesses are unaligned (measured: full speed for a shifted gradient, 5 % less for a
 *    shifted moment array).
 *  - Work is enqueued on `stream` (0 = the null stream).  Nothing is allocated,
 *    nothing synchronises, the call returns as soon as the launches are queued.
 *    Stream order is the only ordering: a gradient buffer may be overwritten by
 *    any later operation on the same stream.
 *  - A gradient must not overlap m or v; tensors of one list must not overlap.
 *  - Hyper-parameters are doubles; derived scalars ((1-beta1)/N, (1-beta2)/N^2,
 *    1-beta^t, ...) are formed in double on the host and rounded to float once.  Decay
 *    factors, whose rounding error would compound from step to step, are applied as a
 *    float32 pair hi + lo that represents the double to about 1e-15.
 *  - Length 0 / count 0 is a successful no-op.  Errors are reported by the return
 *    value, with a message available from adama_last_error(); nothing aborts.
 *    Argument errors are detected before any device work is queued.
 *  - The library keeps no state between calls (the tensor table of a launch travels in the kernel
 *    arguments), so calls may be made from several host threads at once, each on its own stream, may be
 *    recorded into a HIP graph as they are, and work on whichever device is current in the calling
 *    thread; the pointers and the stream must belong to that device.
 */
#ifndef ADAMA_H
#define ADAMA_H

#include <stddef.h>

#include <hip/hip_runtime_api.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ADAMA_OK = 0,
    ADAMA_ERR_INVALID_ARG = 1,        /* null pointer, misaligned pointer, N < 1, t < 1, bad hyper-parameter */
    ADAMA_ERR_UNSUPPORTED_DTYPE = 2,  /* gradient dtype is not one of adama_dtype */
    ADAMA_ERR_TOO_LARGE = 3,          /* a tensor is longer than ADAMA_MAX_ELEMS */
    ADAMA_ERR_HIP = 4                 /* a HIP runtime call failed; text in adama_last_error() */
} adama_status;

/* Gradient storage formats.  The last member only widens the enum to the full int range, so that a
 * value outside the list reaches the library's check (ADAMA_ERR_UNSUPPORTED_DTYPE) as a defined value. */
typedef enum { ADAMA_F32 = 0, ADAMA_BF16 = 1, ADAMA_F16 = 2, ADAMA_DTYPE_INT_RANGE = 0x7fffffff } adama_dtype;

/* Longest tensor accepted by any call (elements). */
#define ADAMA_MAX_ELEMS (1ull << 40)

/* One tensor of a fold list: moments and the raw gradient of the micro-batch loss. */
typedef struct {
    float *m;          /* device, n floats, read and written */
    float *v;          /* device, n floats, read and written */
    const void *grad;  /* device, n elements of the list's gradient dtype, read only */
    size_t n;
} adama_tensor;

/* One tensor of a fused fold+update list. */
typedef struct {
    float *theta;      /* device, n floats, read and written */
    float *m;          /* device, n floats, read and written */
    float *v;          /* device, n floats, read and written */
    const void *grad;  /* device, n elements of the list's gradient dtype, read only */
    size_t n;
} adama_update_tensor;

/* One tensor of a state list (decay / update). theta may be NULL for adama_begin_step_multi. */
typedef struct {
    float *theta;      /* device, n floats, read and written by adama_apply_multi */
    float *m;          /* device, n floats */
    float *v;          /* device, n floats */
    size_t n;
} adama_state;

/* Alg. 2, first line of the while-loop body: once per mini-batch, before its first fold,
 *     m[k] <- beta1 * m[k],  v[k] <- beta2 * v[k]          k in [0, n)
 * (the step counter t <- t+1 is the caller's integer).  beta1, beta2 must be finite and >= 0;
 * values above 1 are accepted because the data-parallel scheme of Sec. 3.3 decays v by
 * (number of devices) * beta2. */
adama_status adama_begin_step(float *m, float *v, size_t n, double beta1, double beta2, hipStream_t stream);

/* The same decay over a host list of `count` tensors (theta fields ignored) in as few launches
 * as the descriptor table allows (ADAMA_MAX_TENSORS_PER_LAUNCH tensors each). */
adama_status adama_begin_step_multi(const adama_state *list, int count, double beta1, double beta2,
                                    hipStream_t stream);

/* Alg. 2, inner loop body, for one gradient tensor of one micro-batch:
 *     g <- grad[k] / N;  m[k] <- m[k] + (1-beta1) g;  v[k] <- v[k] + (1-beta2) g^2
 * `grad` is the raw gradient of the micro-batch loss (NOT pre-divided by N), stored as `gdt`;
 * N >= 1 is the number of micro-batches per mini-batch; beta1, beta2 in [0, 1).
 * The gradient is widened to float32 before scaling and squaring. */
adama_status adama_fold(float *m, float *v, const void *grad, adama_dtype gdt, size_t n, int N,
                        double beta1, double beta2, hipStream_t stream);

/* The fold of Alg. 2 over a whole layer: a ragged host list of `count` tensors, all with gradient
 * dtype `gdt`, in one launch per ADAMA_MAX_TENSORS_PER_LAUNCH tensors.  Results are bit-identical
 * to calling adama_fold on each tensor. */
adama_status adama_fold_multi(const adama_tensor *list, int count, adama_dtype gdt, int N,
                              double beta1, double beta2, hipStream_t stream);

/* Alg. 1 writes the decay and the accumulation as one statement, m_t = beta1 m_{t-1} + (1-beta1) sum_i g_i:
 * the fold of the mini-batch's FIRST micro-batch with the decay of Alg. 2's first line applied on the
 * way,
 *     m[k] <- beta1*m[k] + (1-beta1) g,  v[k] <- beta2*v[k] + (1-beta2) g^2,   g = grad[k]/N
 * with the product beta*m rounded before the addition, so the result is bit-identical to
 * adama_begin_step followed by adama_fold, at the traffic of the fold alone.  Call it instead of
 * adama_begin_step + adama_fold for every tensor in micro-batch 0.  beta1, beta2 in [0, 1). */
adama_status adama_fold_first(float *m, float *v, const void *grad, adama_dtype gdt, size_t n, int N,
                              double beta1, double beta2, hipStream_t stream);
adama_status adama_fold_first_multi(const adama_tensor *list, int count, adama_dtype gdt, int N,
                                    double beta1, double beta2, hipStream_t stream);

/* The fold of the mini-batch's LAST micro-batch followed, element by element, by the Update of Alg. 2
 * on the freshly folded moments (m and v are rounded to float32 before the update uses them):
 * bit-identical to adama_fold followed by adama_apply with step counter t >= 1, at 8 fewer bytes of
 * traffic per parameter.  Call it instead of adama_fold + adama_apply for every tensor in
 * micro-batch N-1.  Arguments as adama_fold and adama_apply. */
adama_status adama_fold_last_apply(float *theta, float *m, float *v, const void *grad, adama_dtype gdt,
                                   size_t n, int N, double lr, double eps, double beta1, double beta2,
                                   long long t, hipStream_t stream);
adama_status adama_fold_last_apply_multi(const adama_update_tensor *list, int count, adama_dtype gdt, int N,
                                         double lr, double eps, double beta1, double beta2, long long t,
                                         hipStream_t stream);

/* Alg. 2, "Update" (same as Alg. 1), after the last fold of mini-batch t >= 1:
 *     m_hat <- m[k] / (1 - beta1^t);  v_hat <- v[k] / (1 - beta2^t)
 *     theta[k] <- theta[k] - lr * m_hat / (sqrt(v_hat) + eps)
 * m and v are read only.  beta1, beta2 in [0, 1); lr, eps finite, eps >= 0. */
adama_status adama_apply(float *theta, const float *m, const float *v, size_t n, double lr, double eps,
                         double beta1, double beta2, long long t, hipStream_t stream);

/* The same update over a host list of `count` tensors. */
adama_status adama_apply_multi(const adama_state *list, int count, double lr, double eps, double beta1,
                               double beta2, long long t, hipStream_t stream);

/* The update of the data-parallel scheme of Sec. 3.3 (text after Eq. 5): every device has decayed v by
 * M*beta2 (adama_begin_step accepts that), folded its own micro-batches, and m and v have been summed
 * over the M devices by an all-reduce, which is the caller's (e.g. RCCL); this call then forms
 *     m[k] <- m[k] * m_scale,  v[k] <- v[k] * v_scale        (m_scale = 1/M, v_scale = 1/M^2)
 * writes both back (they are the next mini-batch's starting moments) and applies the Update of Alg. 2
 * with them.  m_scale, v_scale finite and >= 0; other arguments as adama_apply.  24 B per parameter. */
adama_status adama_rescale_apply(float *theta, float *m, float *v, size_t n, double m_scale, double v_scale,
                                 double lr, double eps, double beta1, double beta2, long long t, hipStream_t stream);
adama_status adama_rescale_apply_multi(const adama_state *list, int count, double m_scale, double v_scale, double lr,
                                       double eps, double beta1, double beta2, long long t, hipStream_t stream);

/* ------------------------------------------------------------------------------------------------
 * Variants.  The paper's Discussion (Sec. 5) notes that the same scheme -- fold each gradient into the
 * optimizer state as it is produced, then release it -- serves any momentum-based optimizer.  The
 * calls below carry it to Adam with decoupled weight decay (AdamW), to gradients taken on a scaled
 * loss (mixed-precision loss scaling), and to SGD with momentum.  The paper gives no formulas for
 * these; each follows the optimizer's usual definition, stated at the call.
 * ------------------------------------------------------------------------------------------------ */

/* Options of the *_opt calls.  A NULL pointer means {0.0, 1.0}, which makes every *_opt call
 * bit-identical to the call without the suffix. */
typedef struct {
    double weight_decay;  /* lambda >= 0, finite.  Decoupled decay: an update also subtracts
                             lr * lambda * theta[k] (theta from before the step); the moments never see it. */
    double grad_scale;    /* s > 0, finite.  Every gradient element is multiplied by s before use
                             (s = 1 / loss_scale when the loss was scaled up for float16 gradients). */
} adama_options;

/* adama_fold_multi / adama_fold_first_multi with g = opt->grad_scale * grad[k] / N.  The factor is
 * folded into the two host-side constants, so traffic and kernels are those of the plain calls. */
adama_status adama_fold_opt_multi(const adama_tensor *list, int count, adama_dtype gdt, int N, double beta1,
                                  double beta2, const adama_options *opt, hipStream_t stream);
adama_status adama_fold_first_opt_multi(const adama_tensor *list, int count, adama_dtype gdt, int N, double beta1,
                                        double beta2, const adama_options *opt, hipStream_t stream);

/* adama_apply_multi with decoupled weight decay:
 *     theta[k] <- theta[k] - (lr * lambda * theta[k] + lr * m_hat / (sqrt(v_hat) + eps))
 * (opt->grad_scale is not used: the moments already hold unscaled gradients). */
adama_status adama_apply_opt_multi(const adama_state *list, int count, double lr, double eps, double beta1,
                                   double beta2, long long t, const adama_options *opt, hipStream_t stream);

/* adama_fold_last_apply_multi with both options: bit-identical to adama_fold_opt_multi followed by
 * adama_apply_opt_multi. */
adama_status adama_fold_last_apply_opt_multi(const adama_update_tensor *list, int count, adama_dtype gdt, int N,
                                             double lr, double eps, double beta1, double beta2, long long t,
                                             const adama_options *opt, hipStream_t stream);

/* adama_rescale_apply_multi with decoupled weight decay. */
adama_status adama_rescale_apply_opt_multi(const adama_state *list, int count, double m_scale, double v_scale,
                                           double lr, double eps, double beta1, double beta2, long long t,
                                           const adama_options *opt, hipStream_t stream);

/* One tensor of an SGD-with-momentum list.  Fields a call does not use may be NULL. */
typedef struct {
    float *theta;      /* device, n floats; read and written by the two apply calls */
    float *b;          /* device, n floats; the momentum buffer */
    const void *grad;  /* device, n elements of the list's gradient dtype; read by the three fold calls */
    size_t n;
} adama_sgdm_tensor;

/* SGD with momentum mu on the mini-batch gradient g = (1/N) sum_i grad_i is
 *     b <- mu * b + g,   theta <- theta - lr * b            (no dampening, no Nesterov term).
 * b is linear in g, so it is built one layer of one micro-batch at a time, as AdamA builds m, and the
 * result equals the textbook step up to rounding (nothing is approximated, unlike AdamA's v):
 *
 *     adama_sgdm_begin_step_multi        once per mini-batch:         b[k] <- mu * b[k]
 *     adama_sgdm_fold_multi              per layer per micro-batch:   b[k] <- b[k] + s * grad[k] / N
 *     adama_sgdm_apply_multi             once per mini-batch:         theta[k] <- theta[k] - (lr*lambda*theta[k] + lr*b[k])
 *
 * and the fused edge forms, bit-identical to the separate calls:
 *
 *     adama_sgdm_fold_first_multi        micro-batch 0:    b[k] <- mu * b[k] + s * grad[k] / N
 *     adama_sgdm_fold_last_apply_multi   micro-batch N-1:  the fold, then the update with the new b
 *
 * mu finite and >= 0; N >= 1; lr finite; s and lambda from `opt` (NULL: s = 1, lambda = 0).
 * Traffic per element: 8 B decay, 8 B + gradient fold, 12 B apply, 16 B + gradient fold_last_apply. */
adama_status adama_sgdm_begin_step_multi(const adama_sgdm_tensor *list, int count, double momentum, hipStream_t stream);
adama_status adama_sgdm_fold_multi(const adama_sgdm_tensor *list, int count, adama_dtype gdt, int N,
                                   const adama_options *opt, hipStream_t stream);
adama_status adama_sgdm_fold_first_multi(const adama_sgdm_tensor *list, int count, adama_dtype gdt, int N,
                                         double momentum, const adama_options *opt, hipStream_t stream);
adama_status adama_sgdm_apply_multi(const adama_sgdm_tensor *list, int count, double lr, const adama_options *opt,
                                    hipStream_t stream);
adama_status adama_sgdm_fold_last_apply_multi(const adama_sgdm_tensor *list, int count, adama_dtype gdt, int N,
                                              double lr, const adama_options *opt, hipStream_t stream);

/* Message of the last failing call on this thread ("" if none).  Valid until the next call
 * on the same thread. */
const char *adama_last_error(void);

/* Host-only: 16 hexadecimal digits identifying the sources and compiler flags the loaded library was
 * built from (a hash the build script passes in), "unidentified" for a build without one.  Lets a
 * caller refuse a binary that does not match the sources beside it.  Static storage. */
const char *adama_build_id(void);

/* Number of tensors one launch's descriptor table holds. */
#define ADAMA_MAX_TENSORS_PER_LAUNCH 80
int adama_max_tensors_per_launch(void);

/* Host-only: the launch policy compiled into the library, for benchmark labels and profile filters.
 * For a launch of op `op` (numbering as in adama_debug_walk) over tensors totalling `launch_elems`
 * elements: *block = threads per workgroup, *groups_per_thread = 4-element groups each thread moves per
 * array (one workgroup handles block * 4 * groups elements; both 0 for an unknown op);
 * *big_launch_elems = the launch length from which the op's large-launch shape is used;
 * *policy_bits: 1 = non-temporal gradient loads, 2 = non-temporal state loads, 4 = non-temporal stores,
 * 8 = those stores also carry the agent-scope bit (written through the L2 at once).
 * Shapes come in three classes of launch length (under 2^20 elements, under 2^26, from 2^26 on); the
 * residency bound (adama_residency) and bit 8 apply from 2^23 elements per launch on.
 * Any pointer may be NULL. */
void adama_tuning(int op, unsigned long long launch_elems, int *block, int *groups_per_thread,
                  unsigned long long *big_launch_elems, int *policy_bits);

/* Host-only: how many workgroups of a launch of op `op` over `launch_elems` elements one compute unit
 * holds at once (0: as many as fit; -1 for an unknown op).  Part of the launch policy: see adama_tuning. */
int adama_residency(int op, unsigned long long launch_elems);

/* Host-only measurement aid, not for production use and not thread-safe: overrides, until the process
 * ends, the number of workgroups per compute unit for launches of op `op` in size class `size_class`
 * (0: under 2^20 elements, 1: under 2^26, 2: from 2^26 on); wgs_per_cu 0 lifts the bound, -1 restores
 * the library's own choice.  Results never depend on it.  Used to produce the A/B tables of the
 * launch policy. */
void adama_debug_set_residency(int op, int size_class, int wgs_per_cu);

/* Host-only: the chunk size (elements handled by one workgroup) the library uses for a launch of op
 * `op` (numbering as in adama_debug_walk) over tensors totalling `launch_elems` elements; 0 for an
 * unknown op.  For benchmark labels and profile filters. */
int adama_launch_chunk(int op, unsigned long long launch_elems);

/*
 * Host-only check of the launch geometry (no device needed, nothing is dereferenced): walks every
 * (launch, chunk, thread, access) the kernels would issue for `list` and adds 1 to touched[k][e]
 * for each element e of tensor k an access covers (touched[k] is a host array of list[k].n bytes,
 * zero-filled by the caller).  op: 0 decay (m, v), 1 fold (m, v, grad), 2 apply (theta, m, v),
 * 3 fold_first (m, v, grad), 4 fold_last_apply (theta, m, v, grad), 5 rescale_apply (theta, m, v);
 * 6..10 the SGD-with-momentum decay, fold, apply, fold_first, fold_last_apply, whose buffer b is
 * passed in the m field.  Fields an op does not use are ignored.  *vector_accesses and *scalar_accesses count 16-byte and single-element accesses.
 * Returns ADAMA_ERR_INVALID_ARG if an access would leave a tensor or a vector access would be
 * misaligned.  Used by the CPU test-suite.
 */
adama_status adama_debug_walk(const adama_update_tensor *list, int count, int op, adama_dtype gdt,
                              unsigned char *const *touched, unsigned long long *vector_accesses,
                              unsigned long long *scalar_accesses, int *launches);

#ifdef __cplusplus
}
#endif

#endif /* ADAMA_H */
