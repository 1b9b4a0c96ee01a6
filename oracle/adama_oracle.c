/*
 * AdamA (Adam Accumulation) reference oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, single-threaded fp64 implementation of what the AdamA hot path
 * computes, written from the paper's two algorithm boxes (Alg. 1 "Adam vs. AdamA
 * with micro-batches" and Alg. 2 "The training pipeline using AdamA") and the
 * data-parallel state synchronisation of Sec. 3.3 (Eqs. 4-7).  Only tests, the
 * smoke check and the benchmark's CPU-baseline leg may call it.  It shares no
 * code, header, table or helper with the HIP library.
 *
 * Every loop is one statement of the algorithm per element, in the paper's
 * order and notation; nothing is blocked, fused, vectorised by hand or
 * reordered.  Build with -O2 -ffp-contract=off so that a*b+c is two roundings,
 * as written.
 *
 * Pins (tests/test_oracle_pins.py): N=1 equals textbook Adam bit for bit and a
 * library Adam to rounding; m equals Adam's m on the mean gradient; exact
 * rational expansion of the unrolled recurrences on tiny tensors; the constant
 * gradient closed form; v >= 0 and zero handling; sum-of-squares vs
 * square-of-sum relations; the multi-device equivalence of Sec. 3.3; element
 * independence; exhaustive bf16/fp16 widening against library conversions.
 *
 * The last part of the file carries the technique over to the variants the
 * paper's discussion (Sec. 5) points at (any momentum-based optimizer can fold and
 * release gradients the same way): a loss-scale factor on the gradient,
 * decoupled weight decay in the update (AdamW), and SGD with momentum.  The
 * paper gives no formulas for these; each follows the optimizer's textbook
 * definition and is pinned against a library implementation of that optimizer
 * run on the mean gradient, plus closed forms.
 * No function here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* Exact widening of 16-bit storage formats to double.                 */
/* ------------------------------------------------------------------ */

/* bfloat16: the upper half of an IEEE binary32 word. */
double adama_oracle_bf16_to_f64(uint16_t bits)
{
    uint32_t w = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
double adama_oracle_f16_to_f64(uint16_t bits)
{
    int sign = (bits >> 15) & 1;
    int expo = (bits >> 10) & 0x1f;
    int frac = bits & 0x3ff;
    double mag;
    if (expo == 0)
        mag = ldexp((double)frac, -24);               /* zero and subnormals: frac * 2^-24 */
    else if (expo == 31)
        mag = frac ? (double)NAN : (double)INFINITY;
    else
        mag = ldexp((double)(1024 + frac), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
    return sign ? -mag : mag;
}

/* ------------------------------------------------------------------ */
/* Alg. 2, first line of the loop body: once per mini-batch             */
/*   m_t <- beta1 * m_{t-1},  v_t <- beta2 * v_{t-1}                    */
/* (t <- t+1 is the caller's integer).  Sec. 3.3 passes M*beta2 here.   */
/* ------------------------------------------------------------------ */
void adama_oracle_begin_step(double *m, double *v, size_t n, double beta1, double beta2)
{
    for (size_t k = 0; k < n; ++k) {
        m[k] = beta1 * m[k];
        v[k] = beta2 * v[k];
    }
}

/* ------------------------------------------------------------------ */
/* Alg. 2, inner loop body: one layer's gradient of one micro-batch.    */
/*   g <- (1/N) * grad                                                  */
/*   m <- m + (1 - beta1) * g                                           */
/*   v <- v + (1 - beta2) * g^2                                         */
/* `grad` is the raw gradient of the micro-batch loss (not yet / N).    */
/* ------------------------------------------------------------------ */
void adama_oracle_fold(double *m, double *v, const double *grad, size_t n, int N,
                       double beta1, double beta2)
{
    for (size_t k = 0; k < n; ++k) {
        double g = grad[k] / (double)N;
        m[k] = m[k] + (1.0 - beta1) * g;
        v[k] = v[k] + (1.0 - beta2) * (g * g);
    }
}

/* The same fold reading the gradient in its storage format; widening is exact. */
void adama_oracle_fold_f32(double *m, double *v, const float *grad, size_t n, int N,
                           double beta1, double beta2)
{
    for (size_t k = 0; k < n; ++k) {
        double g = (double)grad[k] / (double)N;
        m[k] = m[k] + (1.0 - beta1) * g;
        v[k] = v[k] + (1.0 - beta2) * (g * g);
    }
}

void adama_oracle_fold_bf16(double *m, double *v, const uint16_t *grad, size_t n, int N,
                            double beta1, double beta2)
{
    for (size_t k = 0; k < n; ++k) {
        double g = adama_oracle_bf16_to_f64(grad[k]) / (double)N;
        m[k] = m[k] + (1.0 - beta1) * g;
        v[k] = v[k] + (1.0 - beta2) * (g * g);
    }
}

void adama_oracle_fold_f16(double *m, double *v, const uint16_t *grad, size_t n, int N,
                           double beta1, double beta2)
{
    for (size_t k = 0; k < n; ++k) {
        double g = adama_oracle_f16_to_f64(grad[k]) / (double)N;
        m[k] = m[k] + (1.0 - beta1) * g;
        v[k] = v[k] + (1.0 - beta2) * (g * g);
    }
}

/* ------------------------------------------------------------------ */
/* Alg. 2 "Update" (identical in Alg. 1), with t >= 1 already advanced: */
/*   m_hat <- m / (1 - beta1^t),  v_hat <- v / (1 - beta2^t)            */
/*   theta <- theta - alpha * m_hat / (sqrt(v_hat) + eps)               */
/* eps is added to sqrt(v_hat), i.e. after bias correction and outside  */
/* the square root.                                                     */
/* ------------------------------------------------------------------ */
void adama_oracle_apply(double *theta, const double *m, const double *v, size_t n,
                        double lr, double eps, double beta1, double beta2, long long t)
{
    double bias1 = 1.0 - pow(beta1, (double)t);
    double bias2 = 1.0 - pow(beta2, (double)t);
    for (size_t k = 0; k < n; ++k) {
        double m_hat = m[k] / bias1;
        double v_hat = v[k] / bias2;
        theta[k] = theta[k] - lr * m_hat / (sqrt(v_hat) + eps);
    }
}

/* ------------------------------------------------------------------ */
/* Alg. 1 in its closed (non-streaming) form, both colours: one whole   */
/* mini-batch from the N raw micro-batch gradients grads[i*n + k].      */
/*   g_i <- grad_i / N                                                  */
/*   m <- beta1 m + (1-beta1) sum_i g_i                                 */
/*   v <- beta2 v + (1-beta2) (sum_i g_i)^2        variant 0: Adam      */
/*   v <- beta2 v + (1-beta2) sum_i (g_i^2)        variant 1: AdamA     */
/* followed by the Update with the already advanced t.  Variant 0 is    */
/* Adam with plain gradient accumulation, the comparator of the paper.  */
/* ------------------------------------------------------------------ */
void adama_oracle_alg1_step(double *theta, double *m, double *v, const double *grads,
                            size_t n, int N, int variant, double lr, double eps,
                            double beta1, double beta2, long long t)
{
    for (size_t k = 0; k < n; ++k) {
        double sum_g = 0.0, sum_g2 = 0.0;
        for (int i = 0; i < N; ++i) {
            double g = grads[(size_t)i * n + k] / (double)N;
            sum_g = sum_g + g;
            sum_g2 = sum_g2 + g * g;
        }
        double second = variant ? sum_g2 : sum_g * sum_g;
        m[k] = beta1 * m[k] + (1.0 - beta1) * sum_g;
        v[k] = beta2 * v[k] + (1.0 - beta2) * second;
    }
    adama_oracle_apply(theta, m, v, n, lr, eps, beta1, beta2, t);
}

/* ------------------------------------------------------------------ */
/* Sec. 3.3 (text after Eq. 5): after all-reducing the states of the M  */
/* devices, m is averaged and the summed v is divided by M^2.           */
/* m_ranks / v_ranks hold M device-local states, rank r at [r*n, ...).  */
/* Each rank must have decayed v by M*beta2 (not beta2) in its          */
/* begin_step and folded its own N micro-batches with 1/N.              */
/* ------------------------------------------------------------------ */
void adama_oracle_ddp_combine(double *m_out, double *v_out, const double *m_ranks,
                              const double *v_ranks, size_t n, int M)
{
    for (size_t k = 0; k < n; ++k) {
        double sum_m = 0.0, sum_v = 0.0;
        for (int r = 0; r < M; ++r) {
            sum_m = sum_m + m_ranks[(size_t)r * n + k];
            sum_v = sum_v + v_ranks[(size_t)r * n + k];
        }
        m_out[k] = sum_m / (double)M;
        v_out[k] = sum_v / ((double)M * (double)M);
    }
}

/* ================================================================== */
/* Variants beyond the paper's algorithm boxes (Discussion: the same    */
/* fold-and-release works for any momentum-based optimizer).            */
/* ================================================================== */

/* Exact widening of a stored gradient tensor to double.                */
/* gdt: 0 = binary32, 1 = bfloat16 bits, 2 = binary16 bits.             */
int adama_oracle_widen(double *out, const void *grad, size_t n, int gdt)
{
    for (size_t k = 0; k < n; ++k) {
        if (gdt == 0)
            out[k] = (double)((const float *)grad)[k];
        else if (gdt == 1)
            out[k] = adama_oracle_bf16_to_f64(((const uint16_t *)grad)[k]);
        else if (gdt == 2)
            out[k] = adama_oracle_f16_to_f64(((const uint16_t *)grad)[k]);
        else
            return -1;
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* Fold of a gradient that was computed on a scaled loss (mixed         */
/* precision with loss scaling): the true gradient is grad * grad_scale */
/* with grad_scale = 1 / loss_scale, then Alg. 2's inner body as is.    */
/*   g <- (1/N) * (grad_scale * grad)                                   */
/*   m <- m + (1 - beta1) * g,   v <- v + (1 - beta2) * g^2             */
/* ------------------------------------------------------------------ */
void adama_oracle_fold_scaled(double *m, double *v, const double *grad, size_t n, int N,
                              double beta1, double beta2, double grad_scale)
{
    for (size_t k = 0; k < n; ++k) {
        double g = (grad_scale * grad[k]) / (double)N;
        m[k] = m[k] + (1.0 - beta1) * g;
        v[k] = v[k] + (1.0 - beta2) * (g * g);
    }
}

/* ------------------------------------------------------------------ */
/* Update with decoupled weight decay (AdamW): the decay acts on the    */
/* parameter directly, scaled by the learning rate, and never enters    */
/* m or v:                                                              */
/*   theta <- theta - lr * lambda * theta - lr * m_hat/(sqrt(v_hat)+eps)*/
/* Both terms use the parameter value from before the step.  lambda = 0 */
/* is the paper's plain update: there is no decay term then (library    */
/* optimizers skip it too), so 0 * theta is never formed and an         */
/* infinite parameter stays infinite instead of turning into NaN.       */
/* ------------------------------------------------------------------ */
void adama_oracle_apply_adamw(double *theta, const double *m, const double *v, size_t n,
                              double lr, double eps, double beta1, double beta2, long long t,
                              double weight_decay)
{
    double bias1 = 1.0 - pow(beta1, (double)t);
    double bias2 = 1.0 - pow(beta2, (double)t);
    for (size_t k = 0; k < n; ++k) {
        double m_hat = m[k] / bias1;
        double v_hat = v[k] / bias2;
        double decay = lr * weight_decay * theta[k];
        if (weight_decay == 0.0) decay = 0.0;   /* no decay: the term is absent, also for an infinite theta */
        theta[k] = theta[k] - decay - lr * m_hat / (sqrt(v_hat) + eps);
    }
}

/* ------------------------------------------------------------------ */
/* SGD with momentum, accumulated the AdamA way.  The textbook step on  */
/* the mini-batch gradient g = (1/N) sum_i grad_i is                    */
/*   b <- mu * b + g,   theta <- theta - lr * b.                        */
/* b is linear in g, so it can be built one micro-batch and one layer   */
/* at a time exactly as AdamA builds m:                                 */
/*   once per mini-batch:        b <- mu * b                            */
/*   per layer per micro-batch:  b <- b + (grad_scale * grad) / N       */
/*   once per mini-batch:        theta <- theta - lr*lambda*theta - lr*b*/
/* (lambda: decoupled weight decay, 0 for plain SGD).                   */
/* ------------------------------------------------------------------ */
void adama_oracle_sgdm_begin_step(double *b, size_t n, double mu)
{
    for (size_t k = 0; k < n; ++k)
        b[k] = mu * b[k];
}

void adama_oracle_sgdm_fold(double *b, const double *grad, size_t n, int N, double grad_scale)
{
    for (size_t k = 0; k < n; ++k) {
        double g = (grad_scale * grad[k]) / (double)N;
        b[k] = b[k] + g;
    }
}

void adama_oracle_sgdm_apply(double *theta, const double *b, size_t n, double lr,
                             double weight_decay)
{
    for (size_t k = 0; k < n; ++k) {
        double decay = lr * weight_decay * theta[k];
        if (weight_decay == 0.0) decay = 0.0;   /* no decay: the term is absent, also for an infinite theta */
        theta[k] = theta[k] - decay - lr * b[k];
    }
}
