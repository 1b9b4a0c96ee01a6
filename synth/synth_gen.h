/*
 * Seeded synthetic-input generator shared by the host build (gcc) and the
 * device build (hipcc).  It produces gradient-like and weight-like values only;
 * it contains none of the optimizer's arithmetic.
 *
 * The generator is counter based: element `e` of stream `key` depends on
 * (key, e) alone, so any slice of any tensor can be regenerated anywhere, in
 * any order.  Every floating-point step is an individually rounded IEEE
 * binary32 operation (+, -, *, /, sqrt, fma) written out explicitly, so the
 * host and the device produce the same bits.  Compile both sides with
 * floating-point contraction off.
 *
 * Value classes of one element, chosen by a 32-bit selector s drawn per element:
 *   s <  t_zero                       -> exactly 0
 *   s <  t_zero + t_outlier           -> sigma * outlier_scale * T,  T ~ Student-t(nu = 2)
 *   s <  t_zero + t_outlier + t_sub   -> +-k * 2^-24, k in [1, 1023]  (fp16 subnormal magnitudes)
 *   otherwise                         -> sigma * Z,  Z ~ N(0, 1) by Box-Muller
 * and the result is rounded (nearest even) to the output storage format.
 */
#ifndef SYNTH_GEN_H
#define SYNTH_GEN_H

#include <stdint.h>
#include <string.h>

#ifdef __HIPCC__
#define SYNTH_FN __host__ __device__ static inline
#else
#define SYNTH_FN static inline
#endif

enum { SYNTH_F32 = 0, SYNTH_BF16 = 1, SYNTH_F16 = 2 };

typedef struct {
    uint64_t key;          /* stream key (already mixed from seed / config / step / micro-batch / tensor) */
    float sigma;           /* standard deviation of the Gaussian body */
    float outlier_scale;   /* Student-t draws are multiplied by sigma * outlier_scale */
    uint32_t t_zero;       /* P(exact zero)     = t_zero    / 2^32 */
    uint32_t t_outlier;    /* P(heavy tail)     = t_outlier / 2^32 */
    uint32_t t_sub;        /* P(fp16 subnormal) = t_sub     / 2^32 */
    uint32_t reserved;
} synth_spec;

SYNTH_FN float synth_bits_to_float(uint32_t u)
{
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

SYNTH_FN uint32_t synth_float_to_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return u;
}

/* 64-bit finalizer of the SplitMix64 generator (Steele, Lea, Flood 2014). */
SYNTH_FN uint64_t synth_mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* ln(k * 2^-24) for an integer 1 <= k <= 2^24, in binary32. */
SYNTH_FN float synth_log_u24(uint32_t k)
{
    int e = 31 - __builtin_clz(k);                                 /* floor(log2 k), 0..24 */
    float f = (float)k * synth_bits_to_float((uint32_t)(127 - e) << 23);   /* in [1, 2), exact */
    if (f > 1.41421354f) {
        f = f * 0.5f;
        e += 1;
    }
    /* ln f = 2 atanh(s), s = (f-1)/(f+1), |s| <= 0.1716 */
    float s = (f - 1.0f) / (f + 1.0f);
    float w = s * s;
    float p = 0.111111112f;                    /* 1/9 */
    p = __builtin_fmaf(p, w, 0.142857149f);    /* 1/7 */
    p = __builtin_fmaf(p, w, 0.2f);
    p = __builtin_fmaf(p, w, 0.333333343f);
    p = __builtin_fmaf(p, w, 1.0f);
    float lnf = (s + s) * p;
    return __builtin_fmaf((float)(e - 24), 0.693147182f, lnf);
}

/* cos(2 pi u) for u = w / 2^32: quadrant from the top two bits, the next 24 bits
   give the angle inside the quadrant; Taylor polynomials on [0, pi/2). */
SYNTH_FN float synth_cos_turn(uint32_t w)
{
    uint32_t quadrant = w >> 30;
    float x = (float)((w >> 6) & 0xFFFFFFu) * 5.9604644775390625e-08f;   /* [0,1), exact */
    float a = x * 1.57079637f;
    float a2 = a * a;
    float sp = 1.60590444e-10f;                         /* 1/13! */
    sp = __builtin_fmaf(sp, a2, -2.50521084e-08f);      /* -1/11! */
    sp = __builtin_fmaf(sp, a2, 2.75573188e-06f);       /* 1/9!  */
    sp = __builtin_fmaf(sp, a2, -1.98412701e-04f);      /* -1/7! */
    sp = __builtin_fmaf(sp, a2, 8.33333377e-03f);       /* 1/5!  */
    sp = __builtin_fmaf(sp, a2, -1.66666672e-01f);      /* -1/3! */
    sp = __builtin_fmaf(sp, a2, 1.0f);
    float sin_a = a * sp;
    float cp = -1.14707454e-11f;                        /* -1/14! */
    cp = __builtin_fmaf(cp, a2, 2.08767570e-09f);       /* 1/12! */
    cp = __builtin_fmaf(cp, a2, -2.75573188e-07f);      /* -1/10! */
    cp = __builtin_fmaf(cp, a2, 2.48015876e-05f);       /* 1/8!  */
    cp = __builtin_fmaf(cp, a2, -1.38888892e-03f);      /* -1/6! */
    cp = __builtin_fmaf(cp, a2, 4.16666679e-02f);       /* 1/4!  */
    cp = __builtin_fmaf(cp, a2, -0.5f);
    cp = __builtin_fmaf(cp, a2, 1.0f);
    float cos_a = cp;
    switch (quadrant) {
    case 0: return cos_a;
    case 1: return -sin_a;
    case 2: return -cos_a;
    default: return sin_a;
    }
}

/* The unrounded (binary32) value of element e. */
SYNTH_FN float synth_value(const synth_spec *sp, uint64_t e)
{
    uint64_t z1 = synth_mix64(sp->key + (e + 1u) * 0x9E3779B97F4A7C15ull);
    uint64_t z2 = synth_mix64(z1 ^ 0xD1B54A32D192ED03ull);
    uint32_t sel = (uint32_t)z2;
    uint32_t aux = (uint32_t)(z2 >> 32);
    uint64_t edge = sp->t_zero;
    if (sel < edge) return 0.0f;
    edge += sp->t_outlier;
    if (sel < edge) {
        /* Student-t, nu = 2, by its closed-form inverse CDF  t = (2u-1)/sqrt(2u(1-u)) */
        float u = (float)(2u * (aux >> 9) + 1u) * 5.9604644775390625e-08f;   /* (0,1), exact */
        float num = (u + u) - 1.0f;
        float den = __builtin_sqrtf((u + u) * (1.0f - u));
        return (sp->sigma * sp->outlier_scale) * (num / den);
    }
    edge += sp->t_sub;
    if (sel < edge) {
        float mag = (float)(((aux >> 1) % 1023u) + 1u) * 5.9604644775390625e-08f;
        return (aux & 1u) ? -mag : mag;
    }
    uint32_t k = (uint32_t)(z1 >> 40) + 1u;                 /* 1 .. 2^24 */
    float r = __builtin_sqrtf(-2.0f * synth_log_u24(k));
    return sp->sigma * (r * synth_cos_turn((uint32_t)z1));
}

/* binary32 -> bfloat16 bits, round to nearest even (finite inputs). */
SYNTH_FN uint16_t synth_round_bf16(float f)
{
    uint32_t u = synth_float_to_bits(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* binary32 -> binary16 bits, round to nearest even, with subnormals and overflow to inf. */
SYNTH_FN uint16_t synth_round_f16(float f)
{
    uint32_t u = synth_float_to_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    u &= 0x7FFFFFFFu;
    if (u >= 0x7F800000u)                                   /* inf / nan */
        return (uint16_t)(sign | (u > 0x7F800000u ? 0x7E00u : 0x7C00u));
    if (u >= 0x477FF000u)                                   /* >= 65520 rounds to inf */
        return (uint16_t)(sign | 0x7C00u);
    if (u < 0x38800000u) {                                  /* below 2^-14: subnormal or zero */
        /* adding 0.5 aligns 2^-24 with the last mantissa bit; the add rounds to nearest even */
        float shifted = synth_bits_to_float(u) + 0.5f;
        return (uint16_t)(sign | (synth_float_to_bits(shifted) - 0x3F000000u));
    }
    uint32_t odd = (u >> 13) & 1u;
    u += 0xC8000FFFu + odd;                                 /* rebias exponent by -112, round */
    return (uint16_t)(sign | (u >> 13));
}

/* Write element e of the stream into slot i of `out` in storage format `dtype`. */
SYNTH_FN void synth_store(void *out, int dtype, uint64_t i, float value)
{
    if (dtype == SYNTH_F32)
        ((float *)out)[i] = value;
    else if (dtype == SYNTH_BF16)
        ((uint16_t *)out)[i] = synth_round_bf16(value);
    else
        ((uint16_t *)out)[i] = synth_round_f16(value);
}

#endif /* SYNTH_GEN_H */
