#!/usr/bin/env python3
"""Writes tests/golden/tiny_exact.txt: AdamA on a tiny problem in exact arithmetic.

Independent of the oracle and of the HIP library: it uses only Python's
`fractions` (exact rationals) and `decimal` (80-digit square roots).

What is evaluated (paper: Alg. 1 red variant; the unrolled sums are the ones the
appendix uses in the first line of the proof of Lemma 4, with the inner sum over
micro-batches that Alg. 1 adds):

    ghat_{k,i} = grad_{k,i} / N
    m_T = (1-b1) * sum_{k=1..T} b1^(T-k) * sum_i ghat_{k,i}
    v_T = (1-b2) * sum_{k=1..T} b2^(T-k) * sum_i ghat_{k,i}^2
    theta_T = theta_0 - sum_{t=1..T} lr * (m_t/(1-b1^t)) / (sqrt(v_t/(1-b2^t)) + eps)

Hyper-parameters are the exact binary values of the doubles 0.9, 0.999, 1e-3,
1e-8, because that is what a double-typed interface receives.  Gradients are
small dyadic rationals (multiples of 2^-7 with at most 3 significant bits) so
that they are exactly representable in fp64, fp32, bf16 and fp16 alike.

File format, one record per line:
    hyper  beta1 beta2 lr eps            (repr of the doubles)
    shape  T N n
    theta0 <n values>
    grad   t i <n values>                 (t = 1..T, i = 0..N-1), decimal, exact
    m      t <n values>                   40 significant digits
    v      t <n values>
    theta  t <n values>
"""
from __future__ import annotations

import os
from decimal import Decimal, getcontext
from fractions import Fraction

getcontext().prec = 80

BETA1, BETA2, LR, EPS = 0.9, 0.999, 1e-3, 1e-8
T, N, n = 3, 4, 5

# numerators over 128: includes an exact zero column entry, sign changes, and a
# column (index 4) that is zero in every micro-batch of every step.
NUM = {
    (1, 0): [3, -5, 0, 96, 0], (1, 1): [-1, 7, 2, -80, 0], (1, 2): [6, 6, -4, 112, 0], (1, 3): [-2, -3, 1, 64, 0],
    (2, 0): [5, 1, -7, -48, 0], (2, 1): [4, -6, 3, 40, 0], (2, 2): [-3, 2, 2, 56, 0], (2, 3): [1, 1, -1, -96, 0],
    (3, 0): [-6, 4, 5, 24, 0], (3, 1): [2, -2, -2, 28, 0], (3, 2): [7, 3, 6, -20, 0], (3, 3): [-4, -7, 1, 12, 0],
}
THETA0_NUM = [64, -32, 16, 8, -128]   # over 1024


def dec(fr: Fraction) -> Decimal:
    return Decimal(fr.numerator) / Decimal(fr.denominator)


def fmt(values) -> str:
    return " ".join(f"{(v if isinstance(v, Decimal) else dec(v)):.40E}" for v in values)


def main() -> None:
    b1, b2, lr, eps = (Fraction(x) for x in (BETA1, BETA2, LR, EPS))
    grad = {key: [Fraction(a, 128) for a in row] for key, row in NUM.items()}
    theta = [dec(Fraction(a, 1024)) for a in THETA0_NUM]
    lines = [
        "# AdamA on a tiny problem in exact rational arithmetic; written by make_tiny_exact.py",
        "# Source: Alg. 1 (AdamA variant) unrolled as in the appendix proof of Lemma 4.",
        f"hyper {BETA1!r} {BETA2!r} {LR!r} {EPS!r}",
        f"shape {T} {N} {n}",
        "theta0 " + fmt(Fraction(a, 1024) for a in THETA0_NUM),
    ]
    for (t, i), row in sorted(grad.items()):
        lines.append(f"grad {t} {i} " + fmt(row))
    for t in range(1, T + 1):
        m_t, v_t = [], []
        for e in range(n):
            m_e = Fraction(0)
            v_e = Fraction(0)
            for k in range(1, t + 1):
                s1 = sum(grad[(k, i)][e] / N for i in range(N))
                s2 = sum((grad[(k, i)][e] / N) ** 2 for i in range(N))
                m_e += b1 ** (t - k) * s1
                v_e += b2 ** (t - k) * s2
            m_t.append((1 - b1) * m_e)
            v_t.append((1 - b2) * v_e)
        for e in range(n):
            m_hat = dec(m_t[e] / (1 - b1 ** t))
            v_hat = dec(v_t[e] / (1 - b2 ** t))
            theta[e] = theta[e] - dec(lr) * m_hat / (v_hat.sqrt() + dec(eps))
        lines.append(f"m {t} " + fmt(m_t))
        lines.append(f"v {t} " + fmt(v_t))
        lines.append(f"theta {t} " + fmt(theta))
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_exact.txt")
    with open(out, "w") as fh:
        fh.write("\n".join(lines) + "\n")
    print("wrote", out)


if __name__ == "__main__":
    main()
