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
)
