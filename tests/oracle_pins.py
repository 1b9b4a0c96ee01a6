"""Pins for the fp64 oracle: each function checks one fact that the paper or the
mathematics fixes, against something other than the oracle itself, and raises
AssertionError when the oracle library `lib` violates it.

They take the loaded oracle library as an argument so that the same checks run
against the real oracle (test_oracle_pins.py) and against deliberately broken
copies of its source (test_oracle_mutants.py), which every one of the planted
mistakes must fail.
"""
from __future__ import annotations

import math
import os
from decimal import Decimal

import numpy as np

import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
B1, B2, LR, EPS = 0.9, 0.999, 1e-3, 1e-8
GRAD_KINDS = ("f64", "f32", "bf16", "f16")


def encode_grad(g64: np.ndarray, kind: str):
    """Storage encoding of a gradient; returns (array, gdtype, exact fp64 value of what was stored).

    Uses library conversions only (numpy float16, torch bfloat16)."""
    g64 = np.ascontiguousarray(g64, dtype=np.float64)
    if kind == "f64":
        return g64, None, g64
    if kind == "f32":
        a = g64.astype(np.float32)
        return a, None, a.astype(np.float64)
    if kind == "f16":
        a = g64.astype(np.float16)
        return a.view(np.uint16), "f16", a.astype(np.float64)
    if kind == "bf16":
        import torch

        tb = torch.from_numpy(g64).to(torch.bfloat16)
        bits = tb.view(torch.int16).numpy().view(np.uint16).copy()
        return bits, "bf16", tb.to(torch.float64).numpy()
    raise ValueError(kind)


def rel_close(a, b, rtol, what=""):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    err = np.abs(a - b)
    bound = rtol * np.abs(b)
    assert np.all(err <= bound), f"{what}: max rel err {np.max(err / np.maximum(np.abs(b), 1e-300)):.3e} > {rtol}"


# --------------------------------------------------------------------------
# widening of the 16-bit storage formats (all 65536 patterns, library routine)
# --------------------------------------------------------------------------
def pin_widening(lib):
    import torch

    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref16 = bits.view(np.float16).astype(np.float64)
    refbf = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    for b in range(65536):
        got16 = oracle.f16_to_f64(b, lib=lib)
        gotbf = oracle.bf16_to_f64(b, lib=lib)
        for got, ref in ((got16, ref16[b]), (gotbf, refbf[b])):
            if math.isnan(ref):
                assert math.isnan(got), f"pattern {b:#06x}: expected NaN"
            else:
                assert got == ref and math.copysign(1.0, got) == math.copysign(1.0, ref), \
                    f"pattern {b:#06x}: {got!r} != {ref!r}"
    # and the typed folds really go through them: one fold of every finite pattern
    for kind, ref in (("f16", ref16), ("bf16", refbf)):
        fin = np.isfinite(ref) & (np.abs(ref) < 1e150)
        m = np.zeros(int(fin.sum()))
        v = np.zeros_like(m)
        oracle.fold(m, v, bits[fin].copy(), 1, 0.0, 0.0, gdtype=kind, lib=lib)
        assert np.array_equal(m, ref[fin]), f"{kind} fold: m != widened gradient"
        assert np.array_equal(v, ref[fin] * ref[fin]), f"{kind} fold: v != widened gradient squared"


# --------------------------------------------------------------------------
# exact rational expansion (tests/golden/tiny_exact.txt)
# --------------------------------------------------------------------------
def load_tiny_exact():
    rec = {"grad": {}, "m": {}, "v": {}, "theta": {}}
    with open(os.path.join(GOLDEN, "tiny_exact.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            tok = line.split()
            if tok[0] == "hyper":
                rec["hyper"] = tuple(float(x) for x in tok[1:])
            elif tok[0] == "shape":
                rec["shape"] = tuple(int(x) for x in tok[1:])
            elif tok[0] == "theta0":
                rec["theta0"] = np.array([float(Decimal(x)) for x in tok[1:]])
            elif tok[0] == "grad":
                rec["grad"][(int(tok[1]), int(tok[2]))] = np.array([float(Decimal(x)) for x in tok[3:]])
            else:
                rec[tok[0]][int(tok[1])] = np.array([float(Decimal(x)) for x in tok[2:]])
    return rec


def pin_tiny_exact(lib, kinds=GRAD_KINDS):
    """Streaming Alg. 2 through the oracle == exact unrolled sums, for every gradient dtype."""
    rec = load_tiny_exact()
    b1, b2, lr, eps = rec["hyper"]
    T, N, n = rec["shape"]
    for kind in kinds:
        st = oracle.OracleState([rec["theta0"]], lib=lib)
        for t in range(1, T + 1):
            st.begin_step(b1, b2)
            for i in range(N):
                arr, gdt, exact = encode_grad(rec["grad"][(t, i)], kind)
                assert np.array_equal(exact, rec["grad"][(t, i)]), "fixture gradient not exact in " + kind
                st.fold(0, arr, N, b1, b2, gdtype=gdt)
            st.apply(lr, eps, b1, b2)
            assert st.t == t
            rel_close(st.m[0], rec["m"][t], 1e-14, f"tiny exact m t={t} {kind}")
            rel_close(st.v[0], rec["v"][t], 1e-14, f"tiny exact v t={t} {kind}")
            rel_close(st.theta[0], rec["theta"][t], 1e-14, f"tiny exact theta t={t} {kind}")
            # the all-zero column: v stays exactly 0 and theta exactly unchanged
            assert st.v[0][4] == 0.0 and st.m[0][4] == 0.0 and st.theta[0][4] == rec["theta0"][4]
        # Alg. 1 closed form (AdamA colour) reaches the same numbers
        th = rec["theta0"].copy()
        m = np.zeros(n)
        v = np.zeros(n)
        for t in range(1, T + 1):
            grads = np.stack([rec["grad"][(t, i)] for i in range(N)])
            oracle.alg1_step(th, m, v, grads, "adama", lr, eps, b1, b2, t, lib=lib)
            rel_close(m, rec["m"][t], 1e-14, f"alg1 m t={t}")
            rel_close(v, rec["v"][t], 1e-14, f"alg1 v t={t}")
            rel_close(th, rec["theta"][t], 1e-14, f"alg1 theta t={t}")


# --------------------------------------------------------------------------
# N = 1: AdamA is Adam
# --------------------------------------------------------------------------
def _rand_grads(rng, shape, sigma=1e-2):
    return rng.standard_normal(shape) * sigma


def pin_n1_textbook_bitwise(lib):
    """With one micro-batch the streaming form has the same roundings as
    m = b1 m + (1-b1) g, v = b2 v + (1-b2) g^2 followed by the usual update."""
    rng = np.random.default_rng(11)
    n, T = 4099, 4
    theta0 = rng.standard_normal(n) * 0.02
    st = oracle.OracleState([theta0], lib=lib)
    th, m, v = theta0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, T + 1):
        g = _rand_grads(rng, n)
        g[rng.random(n) < 0.01] = 0.0
        st.begin_step(B1, B2)
        st.fold(0, g, 1, B1, B2)
        st.apply(LR, EPS, B1, B2)
        m = B1 * m + (1.0 - B1) * g
        v = B2 * v + (1.0 - B2) * (g * g)
        m_hat = m / (1.0 - B1 ** t)
        v_hat = v / (1.0 - B2 ** t)
        th = th - LR * m_hat / (np.sqrt(v_hat) + EPS)
        assert np.array_equal(st.m[0], m), f"N=1 m differs from textbook Adam at t={t}"
        assert np.array_equal(st.v[0], v), f"N=1 v differs from textbook Adam at t={t}"
        assert np.array_equal(st.theta[0], th), f"N=1 theta differs from textbook Adam at t={t}"
    # with one micro-batch Alg. 1's two colours coincide, bit for bit
    tha, ma, va = theta0.copy(), np.zeros(n), np.zeros(n)
    thb, mb, vb = theta0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, T + 1):
        g = _rand_grads(rng, (1, n))
        oracle.alg1_step(tha, ma, va, g, "adam", LR, EPS, B1, B2, t, lib=lib)
        oracle.alg1_step(thb, mb, vb, g, "adama", LR, EPS, B1, B2, t, lib=lib)
        assert np.array_equal(tha, thb) and np.array_equal(va, vb) and np.array_equal(ma, mb)


def pin_n1_library_adam(lib):
    """N=1 against torch.optim.Adam in fp64 on the CPU (an independent library routine)."""
    import torch

    rng = np.random.default_rng(5)
    n, T = 1537, 6
    theta0 = rng.standard_normal(n) * 0.02
    p = torch.nn.Parameter(torch.from_numpy(theta0.copy()))
    opt = torch.optim.Adam([p], lr=LR, betas=(B1, B2), eps=EPS, weight_decay=0.0, amsgrad=False,
                           foreach=False, fused=False)
    st = oracle.OracleState([theta0], lib=lib)
    for t in range(1, T + 1):
        g = _rand_grads(rng, n, sigma=3e-3)
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        st.begin_step(B1, B2)
        st.fold(0, g, 1, B1, B2)
        st.apply(LR, EPS, B1, B2)
        state = opt.state[p]
        # the library forms m by lerp (m + (g-m)(1-b1)), so compare on the tensor's scale
        ref_m = state["exp_avg"].numpy()
        assert np.max(np.abs(st.m[0] - ref_m)) <= 1e-14 * np.sqrt(np.mean(ref_m ** 2)), f"library Adam m t={t}"
        rel_close(st.v[0], state["exp_avg_sq"].numpy(), 1e-12, f"library Adam v t={t}")
        rel_close(st.theta[0], p.detach().numpy(), 1e-12, f"library Adam theta t={t}")


def pin_m_is_adam_on_mean_gradient(lib, kinds=("f64", "f32")):
    """m after a mini-batch equals library Adam's first moment on the mean of the
    micro-batch gradients (m is linear in the gradients)."""
    import torch

    rng = np.random.default_rng(17)
    n, T, N = 1025, 3, 8
    for kind in kinds:
        theta0 = rng.standard_normal(n) * 0.02
        p = torch.nn.Parameter(torch.from_numpy(theta0.copy()))
        opt = torch.optim.Adam([p], lr=LR, betas=(B1, B2), eps=EPS, foreach=False)
        st = oracle.OracleState([theta0], lib=lib)
        for t in range(1, T + 1):
            st.begin_step(B1, B2)
            mean = np.zeros(n)
            for i in range(N):
                arr, gdt, exact = encode_grad(_rand_grads(rng, n), kind)
                st.fold(0, arr, N, B1, B2, gdtype=gdt)
                mean += exact / N
            st.apply(LR, EPS, B1, B2)
            p.grad = torch.from_numpy(mean.copy())
            opt.step()
            ref = opt.state[p]["exp_avg"].numpy()
            err = np.max(np.abs(st.m[0] - ref))
            assert err <= 1e-13 * np.sqrt(np.mean(ref ** 2)), f"m vs Adam(mean grad) t={t}: {err:.3e}"


# --------------------------------------------------------------------------
# constant gradient: closed form of the whole trajectory
# --------------------------------------------------------------------------
def pin_constant_gradient(lib, kinds=GRAD_KINDS):
    """grad = c in every micro-batch of every step  =>  m_hat = c, v_hat = c^2/N,
    theta_T = theta_0 - T*lr*c/(|c|/sqrt(N) + eps)."""
    c = np.array([0.5, -0.25, 0.0078125, -3.0, 0.0, 6.103515625e-05])   # exact in all four dtypes
    theta0 = np.array([1.0, -2.0, 0.5, 0.25, 0.125, -0.75])
    for kind in kinds:
        for N in (1, 4, 7):
            for (b1, b2, lr, eps) in ((B1, B2, LR, EPS), (0.5, 0.75, 0.125, 1e-3)):
                st = oracle.OracleState([theta0], lib=lib)
                arr, gdt, exact = encode_grad(c, kind)
                assert np.array_equal(exact, c)
                for t in range(1, 6):
                    st.begin_step(b1, b2)
                    for _ in range(N):
                        st.fold(0, arr, N, b1, b2, gdtype=gdt)
                    st.apply(lr, eps, b1, b2)
                    m_hat = st.m[0] / (1.0 - b1 ** t)
                    v_hat = st.v[0] / (1.0 - b2 ** t)
                    rel_close(m_hat, c, 1e-13, f"const grad m_hat N={N} t={t} {kind}")
                    rel_close(v_hat, c * c / N, 1e-13, f"const grad v_hat N={N} t={t} {kind}")
                    want = theta0 - t * lr * c / (np.abs(c) / math.sqrt(N) + eps)
                    rel_close(st.theta[0], want, 1e-13, f"const grad theta N={N} t={t} {kind}")


# --------------------------------------------------------------------------
# sign / zero structure
# --------------------------------------------------------------------------
def pin_v_nonnegative_and_zeros(lib, kinds=GRAD_KINDS):
    rng = np.random.default_rng(3)
    n, T, N = 2048, 3, 4
    for kind in kinds:
        theta0 = rng.standard_normal(n) * 0.02
        st = oracle.OracleState([theta0], lib=lib)
        never = rng.random(n) < 0.05             # elements whose gradient is always exactly 0
        any_nonzero = np.zeros(n, dtype=bool)
        for t in range(1, T + 1):
            st.begin_step(B1, B2)
            for i in range(N):
                g = _rand_grads(rng, n)
                g[rng.random(n) < 0.01] = 0.0
                g[never] = 0.0
                arr, gdt, exact = encode_grad(g, kind)
                any_nonzero |= exact != 0.0
                st.fold(0, arr, N, B1, B2, gdtype=gdt)
            st.apply(LR, EPS, B1, B2)
            assert np.all(st.v[0] >= 0.0), "v went negative"
            assert np.array_equal(st.v[0] == 0.0, ~any_nonzero), "v == 0 must mean: every gradient so far was 0"
            assert np.all(st.theta[0][~any_nonzero] == theta0[~any_nonzero]), "zero gradients moved theta"
            assert np.all(st.m[0][~any_nonzero] == 0.0)
            moved = st.theta[0][any_nonzero] != theta0[any_nonzero]
            assert moved.mean() > 0.99


# --------------------------------------------------------------------------
# sum of squares vs. square of sum (Alg. 1, the two colours)
# --------------------------------------------------------------------------
def pin_adam_vs_adama_second_moment(lib):
    rng = np.random.default_rng(23)
    n, N = 4096, 8
    zeros = lambda: (np.zeros(n), np.zeros(n), np.zeros(n))   # noqa: E731
    # (a) identical micro-gradients: AdamA's v increment is Adam's divided by N
    g = _rand_grads(rng, n)
    grads = np.repeat(g[None, :], N, axis=0)
    th_a, m_a, v_a = zeros()
    th_b, m_b, v_b = zeros()
    oracle.alg1_step(th_a, m_a, v_a, grads, "adam", LR, EPS, B1, B2, 1, lib=lib)
    oracle.alg1_step(th_b, m_b, v_b, grads, "adama", LR, EPS, B1, B2, 1, lib=lib)
    rel_close(v_b * N, v_a, 1e-13, "identical micro-gradients")
    rel_close(v_a, (1.0 - B2) * g * g, 1e-13, "Adam increment is (1-b2) g^2")
    assert np.array_equal(m_a, m_b)
    # (b) disjoint supports: the two second moments coincide
    grads = np.zeros((N, n))
    owner = rng.integers(0, N, n)
    grads[owner, np.arange(n)] = _rand_grads(rng, n)
    th_a, m_a, v_a = zeros()
    th_b, m_b, v_b = zeros()
    oracle.alg1_step(th_a, m_a, v_a, grads, "adam", LR, EPS, B1, B2, 1, lib=lib)
    oracle.alg1_step(th_b, m_b, v_b, grads, "adama", LR, EPS, B1, B2, 1, lib=lib)
    rel_close(v_b, v_a, 1e-13, "disjoint supports")
    rel_close(th_b, th_a, 1e-13, "disjoint supports theta")
    # (c) Cauchy-Schwarz: (sum g)^2 <= N sum g^2, and for iid zero-mean micro-gradients
    # the ratio sqrt(v_adama)/sqrt(v_adam') of Fig. 6's kind concentrates: E[v_adam] = E[v_adama]
    grads = _rand_grads(rng, (N, n))
    th_a, m_a, v_a = zeros()
    th_b, m_b, v_b = zeros()
    oracle.alg1_step(th_a, m_a, v_a, grads, "adam", LR, EPS, B1, B2, 1, lib=lib)
    oracle.alg1_step(th_b, m_b, v_b, grads, "adama", LR, EPS, B1, B2, 1, lib=lib)
    assert np.all(v_a <= N * v_b * (1 + 1e-12)), "Cauchy-Schwarz violated"
    ratio = v_a.mean() / v_b.mean()
    assert 0.9 < ratio < 1.1, f"mean second moments should agree for iid micro-gradients, ratio {ratio}"
    # streaming Alg. 2 equals closed-form Alg. 1 (AdamA colour) to rounding
    st = oracle.OracleState([np.zeros(n)], lib=lib)
    st.begin_step(B1, B2)
    for i in range(N):
        st.fold(0, grads[i], N, B1, B2)
    st.apply(LR, EPS, B1, B2)
    rel_close(st.v[0], v_b, 1e-13, "Alg. 2 vs Alg. 1 v")
    assert np.max(np.abs(st.m[0] - m_b)) <= 1e-14 * np.sqrt(np.mean(m_b ** 2)) * N
    rel_close(st.theta[0], th_b, 1e-9, "Alg. 2 vs Alg. 1 theta")


# --------------------------------------------------------------------------
# Sec. 3.3: M devices x N micro-batches == one device x N*M micro-batches
# --------------------------------------------------------------------------
def pin_ddp_equivalence(lib):
    rng = np.random.default_rng(29)
    n, T = 777, 3
    for M, N in ((2, 4), (4, 2), (3, 5)):
        theta0 = rng.standard_normal(n) * 0.02
        single = oracle.OracleState([theta0], lib=lib)
        m_sync, v_sync = np.zeros(n), np.zeros(n)
        theta_ddp = theta0.copy()
        for t in range(1, T + 1):
            grads = _rand_grads(rng, (M, N, n))
            # one device, N*M micro-batches
            single.begin_step(B1, B2)
            for r in range(M):
                for i in range(N):
                    single.fold(0, grads[r, i], N * M, B1, B2)
            single.apply(LR, EPS, B1, B2)
            # M devices: decay v by M*beta2, fold own micro-batches with 1/N, combine
            m_r = np.repeat(m_sync[None, :], M, axis=0)
            v_r = np.repeat(v_sync[None, :], M, axis=0)
            for r in range(M):
                oracle.begin_step(m_r[r], v_r[r], B1, M * B2, lib=lib)
                for i in range(N):
                    oracle.fold(m_r[r], v_r[r], grads[r, i], N, B1, B2, lib=lib)
            m_sync, v_sync = oracle.ddp_combine(m_r, v_r, lib=lib)
            oracle.apply(theta_ddp, m_sync, v_sync, LR, EPS, B1, B2, t, lib=lib)
            assert np.max(np.abs(m_sync - single.m[0])) <= 1e-13 * np.sqrt(np.mean(single.m[0] ** 2))
            rel_close(v_sync, single.v[0], 1e-13, f"ddp v M={M} N={N} t={t}")
            rel_close(theta_ddp, single.theta[0], 1e-10, f"ddp theta M={M} N={N} t={t}")


# --------------------------------------------------------------------------
# element independence
# --------------------------------------------------------------------------
def pin_element_independence(lib, kinds=GRAD_KINDS):
    rng = np.random.default_rng(31)
    n, N = 3001, 4
    perm = rng.permutation(n)
    cut = 1234
    for kind in kinds:
        theta0 = rng.standard_normal(n) * 0.02
        whole = oracle.OracleState([theta0], lib=lib)
        permuted = oracle.OracleState([theta0[perm]], lib=lib)
        pieces = oracle.OracleState([theta0[:cut], theta0[cut:]], lib=lib)
        for t in (1, 2):
            for st in (whole, permuted, pieces):
                st.begin_step(B1, B2)
            for i in range(N):
                arr, gdt, _ = encode_grad(_rand_grads(rng, n), kind)
                whole.fold(0, arr, N, B1, B2, gdtype=gdt)
                permuted.fold(0, arr[perm], N, B1, B2, gdtype=gdt)
                pieces.fold(1, arr[cut:], N, B1, B2, gdtype=gdt)
                pieces.fold(0, arr[:cut], N, B1, B2, gdtype=gdt)
            for st in (whole, permuted, pieces):
                st.apply(LR, EPS, B1, B2)
        for name in ("theta", "m", "v"):
            w = getattr(whole, name)[0]
            assert np.array_equal(getattr(permuted, name)[0], w[perm])
            assert np.array_equal(np.concatenate(getattr(pieces, name)), w)


# --------------------------------------------------------------------------
# variants beyond the paper's algorithm boxes: loss-scale factor, AdamW, momentum SGD
# --------------------------------------------------------------------------
def pin_widen_tensor(lib):
    """The tensor widening used by the variant folds: all 16-bit patterns and random float32,
    against library conversions."""
    import torch

    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref16 = bits.view(np.float16).astype(np.float64)
    refbf = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    for kind, ref in (("f16", ref16), ("bf16", refbf)):
        got = oracle.widen(bits.copy(), kind, lib=lib)
        nan = np.isnan(ref)
        assert np.array_equal(np.isnan(got), nan), f"{kind}: NaN patterns differ"
        assert np.array_equal(got[~nan], ref[~nan]) and np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan])), kind
    f = np.random.default_rng(3).standard_normal(4099).astype(np.float32)
    assert np.array_equal(oracle.widen(f, lib=lib), f.astype(np.float64))


def pin_fold_scaled_exact(lib, kinds=GRAD_KINDS):
    """One scaled fold from known state against exact rational arithmetic, and the scaling
    invariant: a gradient stored 2^k times too large with grad_scale = 2^-k folds to the very
    bits of the plain fold of the true gradient."""
    from fractions import Fraction

    N, b1, b2, s = 3, 0.875, 0.96875, 1.0 / 1024.0
    g = np.array([0.5, -1.25, 3.0, 0.0, -0.0078125, 24.0])
    m0 = np.array([0.25, -0.5, 0.0, 1.0, 2.0, -3.0])
    v0 = np.array([0.125, 0.5, 0.0, 0.25, 4.0, 9.0])
    for kind in kinds:
        arr, gdt, exact = encode_grad(g * 1024.0, kind)
        assert np.array_equal(exact, g * 1024.0)
        m, v = m0.copy(), v0.copy()
        oracle.fold_scaled(m, v, arr, N, b1, b2, s, gdtype=gdt, lib=lib)
        for k in range(g.size):
            gk = Fraction(float(g[k])) / N
            em = Fraction(float(m0[k])) + (1 - Fraction(b1)) * gk
            ev = Fraction(float(v0[k])) + (1 - Fraction(b2)) * gk * gk
            assert abs(Fraction(float(m[k])) - em) <= abs(em) * Fraction(1, 10 ** 15), f"scaled fold m[{k}] {kind}"
            assert abs(Fraction(float(v[k])) - ev) <= abs(ev) * Fraction(1, 10 ** 15), f"scaled fold v[{k}] {kind}"
    rng = np.random.default_rng(23)
    g = _rand_grads(rng, 777)
    m1, v1 = rng.standard_normal(777) * 1e-3, rng.random(777) * 1e-6
    m2, v2 = m1.copy(), v1.copy()
    oracle.fold(m1, v1, g, 4, B1, B2, lib=lib)
    oracle.fold_scaled(m2, v2, g * 4096.0, 4, B1, B2, 1.0 / 4096.0, lib=lib)
    assert np.array_equal(m1, m2) and np.array_equal(v1, v2), "power-of-two loss scale must cancel exactly"


def pin_adamw_library(lib):
    """N=1 with decoupled weight decay against torch.optim.AdamW in fp64 on the CPU; the moments
    must not see the decay (they equal plain Adam's)."""
    import torch

    rng = np.random.default_rng(29)
    n, T, wd, lr = 1283, 7, 0.1, 2e-3
    theta0 = rng.standard_normal(n) * 0.5
    p = torch.nn.Parameter(torch.from_numpy(theta0.copy()))
    opt = torch.optim.AdamW([p], lr=lr, betas=(B1, B2), eps=EPS, weight_decay=wd, amsgrad=False, foreach=False,
                            fused=False)
    q = torch.nn.Parameter(torch.from_numpy(theta0.copy()))
    plain = torch.optim.Adam([q], lr=lr, betas=(B1, B2), eps=EPS, foreach=False, fused=False)
    theta, m, v = theta0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, T + 1):
        g = _rand_grads(rng, n, sigma=3e-3)
        p.grad = torch.from_numpy(g.copy())
        q.grad = torch.from_numpy(g.copy())
        opt.step()
        plain.step()
        oracle.begin_step(m, v, B1, B2, lib=lib)
        oracle.fold(m, v, g, 1, B1, B2, lib=lib)
        oracle.apply_adamw(theta, m, v, lr, EPS, B1, B2, t, wd, lib=lib)
        rel_close(theta, p.detach().numpy(), 1e-12, f"library AdamW theta t={t}")
        rel_close(v, plain.state[q]["exp_avg_sq"].numpy(), 1e-12, f"AdamW v == Adam v t={t}")
    assert np.max(np.abs(theta - q.detach().numpy())) > 1e-4, "weight decay had no effect"


def pin_adamw_closed_forms(lib):
    """Zero moments: theta_T = theta_0 (1 - lr*lambda)^T exactly as a product.  lambda = 0: the
    very bits of the plain update.  One step from given state against exact rationals up to the
    square root."""
    rng = np.random.default_rng(31)
    n, lr, wd = 257, 0.05, 0.3
    theta0 = rng.standard_normal(n)
    theta = theta0.copy()
    z = np.zeros(n)
    for t in range(1, 6):
        oracle.apply_adamw(theta, z, z, lr, EPS, B1, B2, t, wd, lib=lib)
        rel_close(theta, theta0 * (1.0 - lr * wd) ** t, 1e-14, f"pure decay t={t}")
    m, v = rng.standard_normal(n) * 1e-2, rng.random(n) * 1e-4
    a, b = theta0.copy(), theta0.copy()
    oracle.apply(a, m, v, LR, EPS, B1, B2, 3, lib=lib)
    oracle.apply_adamw(b, m, v, LR, EPS, B1, B2, 3, 0.0, lib=lib)
    assert np.array_equal(a, b), "lambda = 0 must reproduce the plain update"
    # decay and Adam step are additive: theta_w - theta_plain = -lr*lambda*theta_0
    c = theta0.copy()
    oracle.apply_adamw(c, m, v, LR, EPS, B1, B2, 3, wd, lib=lib)
    err = np.abs((c - a) + LR * wd * theta0)
    assert np.all(err <= 4e-16 * np.abs(theta0) + 1e-300), "decay term is not -lr*lambda*theta_0"


def pin_sgdm_library(lib, kinds=GRAD_KINDS):
    """Momentum SGD accumulated per micro-batch against torch.optim.SGD(momentum) in fp64 on the
    mean gradient: the buffer and the parameters agree to rounding."""
    import torch

    rng = np.random.default_rng(37)
    n, T, N, mu, lr = 1031, 5, 4, 0.9, 0.05
    for kind in kinds:
        theta0 = rng.standard_normal(n) * 0.1
        p = torch.nn.Parameter(torch.from_numpy(theta0.copy()))
        opt = torch.optim.SGD([p], lr=lr, momentum=mu, dampening=0.0, weight_decay=0.0, nesterov=False, foreach=False)
        theta, b = theta0.copy(), np.zeros(n)
        for t in range(1, T + 1):
            oracle.sgdm_begin_step(b, mu, lib=lib)
            mean = np.zeros(n)
            for i in range(N):
                arr, gdt, exact = encode_grad(_rand_grads(rng, n), kind)
                oracle.sgdm_fold(b, arr, N, 1.0, gdtype=gdt, lib=lib)
                mean += exact / N
            oracle.sgdm_apply(theta, b, lr, 0.0, lib=lib)
            p.grad = torch.from_numpy(mean.copy())
            opt.step()
            ref_b = opt.state[p]["momentum_buffer"].numpy()
            scale = np.sqrt(np.mean(ref_b ** 2))
            assert np.max(np.abs(b - ref_b)) <= 1e-13 * scale, f"SGD momentum buffer t={t} {kind}"
            assert np.max(np.abs(theta - p.detach().numpy())) <= 1e-13 * np.max(np.abs(theta0)), f"SGD theta t={t} {kind}"


def pin_sgdm_closed_forms(lib):
    """Constant gradient c: b_T = c (1 - mu^T)/(1 - mu), theta_T = theta_0 - lr * sum_t b_t.
    Zero gradient with decay: theta_T = theta_0 (1 - lr*lambda)^T.  Loss scale: exact rationals."""
    from fractions import Fraction

    n, N, mu, lr, T = 65, 4, 0.75, 0.125, 6
    c = np.linspace(-2.0, 2.0, n)
    theta0 = np.linspace(1.0, 3.0, n)
    theta, b = theta0.copy(), np.zeros(n)
    acc = np.zeros(n)
    for t in range(1, T + 1):
        oracle.sgdm_begin_step(b, mu, lib=lib)
        for i in range(N):
            oracle.sgdm_fold(b, c, N, 1.0, lib=lib)
        oracle.sgdm_apply(theta, b, lr, 0.0, lib=lib)
        bt = c * (1.0 - mu ** t) / (1.0 - mu)
        acc += bt
        assert np.max(np.abs(b - bt)) <= 1e-14 * np.max(np.abs(bt)), f"constant gradient buffer t={t}"
        assert np.max(np.abs(theta - (theta0 - lr * acc))) <= 1e-14 * np.max(np.abs(theta0)), f"constant gradient theta t={t}"
    theta = theta0.copy()
    z = np.zeros(n)
    for t in range(1, 5):
        oracle.sgdm_apply(theta, z, lr, 0.5, lib=lib)
        rel_close(theta, theta0 * (1.0 - lr * 0.5) ** t, 1e-14, f"SGD pure decay t={t}")
    g = np.array([3.0, -0.375, 640.0])
    b0 = np.array([1.0, -2.0, 0.5])
    b = b0.copy()
    oracle.sgdm_fold(b, g, 3, 1.0 / 64.0, lib=lib)
    for k in range(3):
        eb = Fraction(float(b0[k])) + Fraction(float(g[k])) / 64 / 3
        assert abs(Fraction(float(b[k])) - eb) <= abs(eb) * Fraction(1, 10 ** 15), f"scaled SGD fold [{k}]"
    th = np.array([2.0, -4.0, 8.0])
    th0 = th.copy()
    oracle.sgdm_apply(th, b0, 0.25, 0.5, lib=lib)
    for k in range(3):
        e = Fraction(float(th0[k])) * (1 - Fraction(1, 8)) - Fraction(1, 4) * Fraction(float(b0[k]))
        assert Fraction(float(th[k])) == e, f"SGD apply [{k}]"


def pin_non_finite_values(lib):
    """IEEE special cases worked out by hand (beta > 0, lr > 0): an infinite moment decays to the same
    infinity; an infinite gradient makes m infinite of its sign and v +inf; the update leaves theta alone
    when only v is infinite (finite / inf = 0), sends it to -/+inf when only m is +/-inf, and gives NaN
    for inf / inf; NaN stays NaN.  Momentum SGD with an infinite gradient, two steps, against
    torch.optim.SGD (which forms no decay term for weight_decay = 0): buffer and parameter keep their
    infinities.  lambda = 0 reproduces the plain update bit for bit on infinite parameters too."""
    import torch

    inf, nan = np.inf, np.nan
    m = np.array([1.0, inf, -inf, nan, 2.0, 0.5])
    v = np.array([inf, 3.0, inf, 1.0, nan, 0.25])
    oracle.begin_step(m, v, 0.9, 0.999, lib=lib)
    assert m[1] == inf and m[2] == -inf and np.isnan(m[3]) and v[0] == inf and v[2] == inf and np.isnan(v[4])
    assert m[0] == 0.9 and v[5] == 0.999 * 0.25
    m, v = np.zeros(4), np.zeros(4)
    for kind in ("f64", "f32", "bf16", "f16"):
        arr, gdt, _ = encode_grad(np.array([inf, -inf, 1.0, 0.0]), kind)
        if kind == "f64":
            arr = np.array([inf, -inf, nan, 0.0])
        mm, vv = m.copy(), v.copy()
        oracle.fold(mm, vv, arr, 4, 0.9, 0.999, gdtype=gdt, lib=lib)
        assert mm[0] == inf and mm[1] == -inf and vv[0] == inf and vv[1] == inf and mm[3] == 0 and vv[3] == 0, kind
        if kind == "f64":
            assert np.isnan(mm[2]) and np.isnan(vv[2])
    theta0 = np.array([1.5, -2.5, 3.5, 4.5, 5.5, inf, -inf])
    theta = theta0.copy()
    m = np.array([1e-3, inf, -inf, inf, nan, 1e-3, 1e-3])
    v = np.array([inf, 1e-6, 1e-6, inf, 1e-6, 1e-6, 1e-6])
    oracle.apply(theta, m, v, 1e-3, 1e-8, 0.9, 0.999, 2, lib=lib)
    assert theta[0] == 1.5 and theta[1] == -inf and theta[2] == inf and np.isnan(theta[3]) and np.isnan(theta[4])
    assert theta[5] == inf and theta[6] == -inf
    plain = theta.copy()
    theta = theta0.copy()
    oracle.apply_adamw(theta, m, v, 1e-3, 1e-8, 0.9, 0.999, 2, 0.0, lib=lib)
    assert np.array_equal(theta, plain, equal_nan=True), "lambda = 0 must be the plain update, infinite parameters included"
    # momentum SGD against the library over two steps
    n, mu, lr = 6, 0.8, 0.05
    g1 = np.array([inf, -inf, 1.0, -2.0, nan, 0.5])
    g2 = np.array([1.0, 1.0, 1.0, inf, 1.0, -0.5])
    th0 = np.linspace(-1.0, 1.0, n)
    p = torch.nn.Parameter(torch.from_numpy(th0.copy()))
    opt = torch.optim.SGD([p], lr=lr, momentum=mu, dampening=0.0, weight_decay=0.0, nesterov=False, foreach=False)
    theta, b = th0.copy(), np.zeros(n)
    for g in (g1, g2):
        oracle.sgdm_begin_step(b, mu, lib=lib)
        oracle.sgdm_fold(b, g, 1, 1.0, lib=lib)
        oracle.sgdm_apply(theta, b, lr, 0.0, lib=lib)
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        assert np.array_equal(b, opt.state[p]["momentum_buffer"].numpy(), equal_nan=True), "SGD buffer with non-finite gradients"
        assert np.array_equal(theta, p.detach().numpy(), equal_nan=True), "SGD parameters with non-finite gradients"
    assert theta[0] == -inf and theta[1] == inf and theta[3] == -inf and np.isnan(theta[4]) and np.isfinite(theta[2])


ALL_PINS = (
    pin_widening,
    pin_tiny_exact,
    pin_n1_textbook_bitwise,
    pin_n1_library_adam,
    pin_m_is_adam_on_mean_gradient,
    pin_constant_gradient,
    pin_v_nonnegative_and_zeros,
    pin_adam_vs_adama_second_moment,
    pin_ddp_equivalence,
    pin_element_independence,
    pin_widen_tensor,
    pin_fold_scaled_exact,
    pin_adamw_library,
    pin_adamw_closed_forms,
    pin_sgdm_library,
    pin_sgdm_closed_forms,
    pin_non_finite_values,
)
