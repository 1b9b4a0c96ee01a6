"""GPU parity on non-finite values across mini-batches: an infinite or NaN moment left behind by one
mini-batch goes through the next decay, the next folds and the next update exactly as in the fp64
oracle (the method has no skip logic: Alg. 2 applies IEEE arithmetic to whatever arrives).

The decay factor is applied on the device as a float32 pair hi + lo.  For beta = 0.999, 0.99, 0.8 and
for 1/3, 1/9 the low part is negative, which is the case where a careless hi*x + lo*x turns an
infinite moment into inf - inf = NaN; beta = 0.9, 0.9999 have a positive low part.  Both signs, the
separate and the fused entry points, the data-parallel rescale and the SGD buffer are covered, over
two mini-batches so that the second decay meets the first one's leftovers."""
import numpy as np
import pytest

import oracle
import synth
from parity import check_close

pytestmark = pytest.mark.gpu

LR, EPS = 1e-3, 1e-8
POS, NEG, NAN = np.inf, -np.inf, np.nan


@pytest.fixture(scope="module")
def torch_cuda():
    import torch

    assert torch.cuda.is_available()
    from paper_2305_19982_amd import binding

    binding.load()
    return torch


def _plant(g_host: np.ndarray, gdt: str, where: dict) -> np.ndarray:
    """Overwrite elements of a host gradient array (float32 values or 16-bit patterns) with specials."""
    for idx, val in where.items():
        if gdt == "f32":
            g_host[idx] = val
        elif gdt == "bf16":
            g_host[idx] = np.array([val], dtype=np.float32).view(np.uint32)[0] >> 16
        else:
            g_host[idx] = np.array([val], dtype=np.float16).view(np.uint16)[0]
    return g_host


def _upload(torch, g_host: np.ndarray):
    return torch.from_numpy(g_host.view(np.int16) if g_host.dtype == np.uint16 else g_host).cuda()


def _same_specials(name: str, kind: str, gpu: np.ndarray, ref: np.ndarray) -> int:
    """NaN, +inf and -inf sit at the same elements on both sides; everything else is within tolerance.
    Returns the number of non-finite elements."""
    assert np.array_equal(np.isnan(gpu), np.isnan(ref)), \
        f"{name} {kind}: NaN at {np.flatnonzero(np.isnan(gpu) != np.isnan(ref))[:8]} differs from the oracle"
    assert np.array_equal(np.isposinf(gpu), np.isposinf(ref)), \
        f"{name} {kind}: +inf at {np.flatnonzero(np.isposinf(gpu) != np.isposinf(ref))[:8]} differs from the oracle"
    assert np.array_equal(np.isneginf(gpu), np.isneginf(ref)), \
        f"{name} {kind}: -inf at {np.flatnonzero(np.isneginf(gpu) != np.isneginf(ref))[:8]} differs from the oracle"
    fin = np.isfinite(ref)
    check_close(name + " (finite part)", kind, gpu[fin], ref[fin])
    return int((~fin).sum())


# beta pairs: float32(beta) above beta for 0.999, 0.99, 0.8 (negative low part), below for 0.9, 0.9999
BETAS = [(0.9, 0.999), (0.8, 0.99), (0.9, 0.9999)]


@pytest.mark.parametrize("gdt", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("fused", [False, True], ids=["separate", "fused"])
@pytest.mark.parametrize("b1,b2", BETAS)
def test_non_finite_moments_through_the_next_mini_batch(torch_cuda, b1, b2, fused, gdt):
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    n, N, steps = 9001, 3, 2
    th0 = synth.fill_host(synth.Spec(key=synth.stream_key(91, 0), sigma=0.02), "f32", n)
    # moments the run starts from: finite almost everywhere, plus every combination the update can meet
    rng = np.random.default_rng(17)
    m0 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    v0 = (np.abs(rng.standard_normal(n)) * 1e-6).astype(np.float32)
    m0[100], v0[100] = 1e-3, POS          # v infinite alone: the step is m / inf = 0, theta stays
    m0[101], v0[101] = POS, 1e-6          # m infinite alone: theta goes to -inf
    m0[102], v0[102] = NEG, 1e-6
    m0[103], v0[103] = POS, POS           # both: inf / inf = NaN
    m0[104], v0[104] = NAN, 1e-6
    m0[105], v0[105] = 1e-3, NAN
    m0[8999], v0[8999] = NEG, POS
    theta, m, v = (torch.from_numpy(x.copy()).cuda() for x in (th0, m0, v0))
    ref = oracle.OracleState([th0])
    ref.m[0][:] = m0
    ref.v[0][:] = v0
    # gradients: specials arrive in step 1 (micro-batches 0, 1 and 2) and one more in step 2
    planted = {(1, 0): {7: POS, 8: NEG, 4097: POS}, (1, 1): {9: NAN, 5000: NEG}, (1, 2): {10: POS, 7: NEG},
               (2, 1): {11: POS}}
    gd = None if gdt == "f32" else gdt
    total_bad = 0
    for t in range(1, steps + 1):
        ref.begin_step(b1, b2)
        if not fused:
            binding.adama_begin_step(m, v, n, b1, b2)
        for i in range(N):
            g_host = synth.fill_host(synth.Spec(key=synth.stream_key(91, t, i), sigma=1e-2, p_zero=0.01), gdt, n)
            g_host = _plant(g_host, gdt, planted.get((t, i), {}))
            g = _upload(torch, g_host)
            if fused and i == 0:
                binding.adama_fold_first(m, v, g, gdt, n, N, b1, b2)
            elif fused and i == N - 1:
                binding.adama_fold_last_apply(theta, m, v, g, gdt, n, N, LR, EPS, b1, b2, t)
            else:
                binding.adama_fold(m, v, g, gdt, n, N, b1, b2)
            ref.fold(0, g_host, N, b1, b2, gdtype=gd)
        if not fused:
            binding.adama_apply(theta, m, v, n, LR, EPS, b1, b2, t)
        ref.apply(LR, EPS, b1, b2)
        torch.cuda.synchronize()
        name = f"b1={b1} b2={b2} {'fused' if fused else 'separate'} {gdt} t={t}"
        with np.errstate(invalid="ignore"):
            total_bad += _same_specials(name, "m", m.cpu().numpy(), ref.m[0])
            total_bad += _same_specials(name, "v", v.cpu().numpy(), ref.v[0])
            total_bad += _same_specials(name, "theta", theta.cpu().numpy(), ref.theta[0])
    hv, hm, ht = v.cpu().numpy(), m.cpu().numpy(), theta.cpu().numpy()
    # the point of the exercise: infinite moments are still infinite after two decays (not NaN), and
    # an infinite second moment alone leaves its parameter where it was
    assert hv[100] == POS and hv[7] == POS and hv[4097] == POS and hm[4097] == POS and hm[8] == NEG
    assert ht[100] == th0[100], "theta must not move while its second moment is infinite and its first finite"
    assert total_bad >= 30


@pytest.mark.parametrize("M", [3, 2, 7])
def test_non_finite_moments_through_the_data_parallel_rescale(torch_cuda, M):
    """Sec. 3.3: the summed moments are scaled by 1/M and 1/M^2 (float32 pairs with a negative low part
    for M = 3) before the update; an infinite sum stays infinite."""
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    n, b1, b2, t = 6007, 0.9, 0.999, 4
    th0 = synth.fill_host(synth.Spec(key=synth.stream_key(92, M), sigma=0.02), "f32", n)
    rng = np.random.default_rng(M)
    m_r = rng.standard_normal((M, n)) * 1e-3
    v_r = np.abs(rng.standard_normal((M, n))) * 1e-6
    m_r, v_r = m_r.astype(np.float32).astype(np.float64), v_r.astype(np.float32).astype(np.float64)
    v_r[0, 50] = POS
    m_r[1, 51] = POS
    m_r[0, 52] = NEG
    m_r[0, 53], v_r[0, 53] = POS, POS
    m_r[0, 54], m_r[1, 54] = POS, NEG          # inf - inf in the sum itself: NaN on both sides
    v_r[1, 55] = NAN
    m_r[M - 1, 6006], v_r[M - 1, 6006] = NEG, POS
    with np.errstate(invalid="ignore"):
        m_sum = torch.from_numpy(m_r.astype(np.float32)).cuda().sum(dim=0)     # stand-in for the all-reduce
        v_sum = torch.from_numpy(v_r.astype(np.float32)).cuda().sum(dim=0)
        theta = torch.from_numpy(th0.copy()).cuda()
        rm, rv = oracle.ddp_combine(m_r, v_r)          # fp64: sum over devices, / M and / M^2
        rth = th0.astype(np.float64)
        oracle.apply(rth, rm, rv, LR, EPS, b1, b2, t)
        binding.adama_rescale_apply(theta, m_sum, v_sum, n, 1.0 / M, 1.0 / (M * M), LR, EPS, b1, b2, t)
        torch.cuda.synchronize()
        name = f"rescale M={M}"
        bad = _same_specials(name, "m", m_sum.cpu().numpy(), rm)
        bad += _same_specials(name, "v", v_sum.cpu().numpy(), rv)
        bad += _same_specials(name, "theta", theta.cpu().numpy(), rth)
    assert v_sum.cpu().numpy()[50] == POS and theta.cpu().numpy()[50] == th0[50]
    assert bad >= 12


@pytest.mark.parametrize("fused", [False, True], ids=["separate", "fused"])
@pytest.mark.parametrize("mu", [0.8, 0.9, 0.99])
def test_non_finite_momentum_buffer_through_the_next_mini_batch(torch_cuda, mu, fused):
    """SGD with momentum: an infinite buffer element stays infinite through the next decay
    (float32(0.8) and float32(0.99) are above the factor: negative low part)."""
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    n, N, steps, lr, gdt = 7001, 2, 2, 0.05, "bf16"
    th0 = synth.fill_host(synth.Spec(key=synth.stream_key(93, 0), sigma=0.02), "f32", n)
    theta = torch.from_numpy(th0.copy()).cuda()
    b = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    rth, rb = th0.astype(np.float64), np.zeros(n)
    planted = {(1, 0): {3: POS, 4: NEG, 4100: NAN}, (1, 1): {5: POS, 3: POS}, (2, 0): {6: NEG}}
    bad = 0
    for t in range(1, steps + 1):
        oracle.sgdm_begin_step(rb, mu)
        if not fused:
            binding.adama_sgdm_begin_step_multi([(None, b, None, n)], None, mu)
        for i in range(N):
            g_host = _plant(synth.fill_host(synth.Spec(key=synth.stream_key(93, t, i), sigma=1e-2), gdt, n), gdt,
                            planted.get((t, i), {}))
            g = _upload(torch, g_host)
            if fused and i == 0:
                binding.adama_sgdm_fold_first_multi([(None, b, g, n)], None, gdt, N, mu)
            elif fused and i == N - 1:
                binding.adama_sgdm_fold_last_apply_multi([(theta, b, g, n)], None, gdt, N, lr)
            else:
                binding.adama_sgdm_fold_multi([(None, b, g, n)], None, gdt, N)
            oracle.sgdm_fold(rb, g_host, N, 1.0, gdtype=gdt)
        if not fused:
            binding.adama_sgdm_apply_multi([(theta, b, None, n)], None, lr)
        oracle.sgdm_apply(rth, rb, lr, 0.0)
        torch.cuda.synchronize()
        name = f"sgdm mu={mu} {'fused' if fused else 'separate'} t={t}"
        with np.errstate(invalid="ignore"):
            bad += _same_specials(name, "m", b.cpu().numpy(), rb)
            bad += _same_specials(name, "theta", theta.cpu().numpy(), rth)
    hb = b.cpu().numpy()
    assert hb[3] == POS and hb[4] == NEG and hb[5] == POS and hb[6] == NEG and np.isnan(hb[4100])
    assert bad >= 12
