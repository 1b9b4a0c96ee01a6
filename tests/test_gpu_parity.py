"""GPU parity: libadama (through its C ABI) against the fp64 oracle, element by element."""
import numpy as np
import pytest

import oracle
import synth
from parity import WorkloadRun, check_close
from synth import configs

pytestmark = pytest.mark.gpu

B1, B2, LR, EPS = 0.9, 0.999, 1e-3, 1e-8


@pytest.fixture(scope="module")
def torch_cuda():
    import torch

    assert torch.cuda.is_available()
    from paper_2305_19982_amd import binding

    binding.load()
    return torch


def _log(msg):
    print(msg, flush=True)


# ---------------------------------------------------------------------------
# the synthetic-input generator writes the same bits on the device and on the host
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_device_and_host_generators_agree(torch_cuda, dtype):
    torch = torch_cuda
    n = 3_000_001
    spec = synth.Spec(key=synth.stream_key(7, 1, 2, 3), sigma=3e-3, p_zero=0.01, p_outlier=0.002, p_sub=0.01)
    buf = torch.empty(n * 4, dtype=torch.uint8, device="cuda:0")
    synth.fill_device(buf.data_ptr(), spec, dtype, n, 0, first=12345)
    torch.cuda.synchronize()
    nbytes = n * synth.gen.DTYPE_BYTES[dtype]
    dev = buf[:nbytes].cpu().numpy().view(np.float32 if dtype == "f32" else np.uint16)
    host = synth.fill_host(spec, dtype, n, first=12345)
    assert np.array_equal(dev, host)


# ---------------------------------------------------------------------------
# single calls on awkward shapes: lengths around chunk boundaries, misaligned starts
# ---------------------------------------------------------------------------
LENGTHS = [1, 2, 3, 4, 5, 7, 63, 64, 255, 1023, 1024, 1025, 4095, 4096, 4097, 8191, 12289, 1 << 16,
           (1 << 22) + 5, (1 << 22) + 4096 * 3 + 1]


def _fold_case(torch, gdt, n, pre_state, pre_grad, N, kind="fold"):
    """One begin_step + fold(s) + apply on a tensor placed `pre` elements past an aligned address."""
    from paper_2305_19982_amd import binding

    gbytes = synth.gen.DTYPE_BYTES[gdt]
    pad = 64
    theta = torch.zeros(n + pad, dtype=torch.float32, device="cuda:0")
    m = torch.zeros(n + pad, dtype=torch.float32, device="cuda:0")
    v = torch.zeros(n + pad, dtype=torch.float32, device="cuda:0")
    g = torch.zeros((n + pad) * gbytes, dtype=torch.uint8, device="cuda:0")
    key = synth.stream_key(11, n, pre_state, pre_grad, N)
    th0 = synth.fill_host(synth.Spec(key=key, sigma=0.02), "f32", n)
    m0 = synth.fill_host(synth.Spec(key=key + 1, sigma=1e-3), "f32", n)
    v0 = np.abs(synth.fill_host(synth.Spec(key=key + 2, sigma=1e-5), "f32", n))
    sl = slice(pre_state, pre_state + n)
    theta[sl] = torch.from_numpy(th0).cuda()
    m[sl] = torch.from_numpy(m0).cuda()
    v[sl] = torch.from_numpy(v0).cuda()
    p_t, p_m, p_v = (x.data_ptr() + 4 * pre_state for x in (theta, m, v))
    p_g = g.data_ptr() + gbytes * pre_grad
    ref = oracle.OracleState([th0])
    ref.m[0][:] = m0
    ref.v[0][:] = v0
    ref.t = 2
    binding.adama_begin_step(p_m, p_v, n, B1, B2)
    ref.begin_step(B1, B2)
    gd = None if gdt == "f32" else gdt
    for i in range(N):
        spec = synth.Spec(key=key + 10 + i, sigma=1e-2, p_zero=0.02, p_sub=0.02 if gdt == "f16" else 0.0,
                          p_outlier=0.001)
        synth.fill_device(p_g, spec, gdt, n, 0)
        binding.adama_fold(p_m, p_v, p_g, gdt, n, N, B1, B2)
        ref.fold(0, synth.fill_host(spec, gdt, n), N, B1, B2, gdtype=gd)
    binding.adama_apply(p_t, p_m, p_v, n, LR, EPS, B1, B2, ref.t)
    ref.apply(LR, EPS, B1, B2)
    torch.cuda.synchronize()
    name = f"{gdt} n={n} pre={pre_state}/{pre_grad} N={N}"
    check_close(name, "m", m[sl].cpu().numpy(), ref.m[0])
    check_close(name, "v", v[sl].cpu().numpy(), ref.v[0])
    check_close(name, "theta", theta[sl].cpu().numpy(), ref.theta[0], th0, th0.astype(np.float64))
    # nothing outside the tensor was written
    for arr in (theta, m, v):
        assert float(arr[:pre_state].abs().sum()) == 0.0 and float(arr[pre_state + n:].abs().sum()) == 0.0, name


@pytest.mark.parametrize("gdt", ["f32", "bf16", "f16"])
def test_fold_lengths_aligned(torch_cuda, gdt):
    for n in LENGTHS:
        _log(f"case {gdt} n={n} aligned")
        _fold_case(torch_cuda, gdt, n, 0, 0, N=3)


@pytest.mark.parametrize("gdt", ["f32", "bf16", "f16"])
def test_fold_misaligned_starts(torch_cuda, gdt):
    for n in (1, 6, 1021, 4099, 70001, (1 << 22) + 11):
        for pre_state, pre_grad in ((1, 1), (2, 2), (3, 3), (1, 0), (0, 3), (2, 5), (3, 7)):
            _log(f"case {gdt} n={n} pre={pre_state}/{pre_grad}")
            _fold_case(torch_cuda, gdt, n, pre_state, pre_grad, N=2)


def test_fold_n1_and_large_N(torch_cuda):
    _fold_case(torch_cuda, "bf16", 50001, 0, 0, N=1)
    _fold_case(torch_cuda, "f16", 50001, 0, 0, N=64)


def test_fp16_every_finite_pattern_including_subnormals(torch_cuda):
    """All 63488 finite fp16 patterns through one fold: widening happens before scaling and squaring."""
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    bits = bits[np.isfinite(bits.view(np.float16))]
    n = bits.size
    g = torch.from_numpy(bits.view(np.int16).copy()).cuda()
    m = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    v = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    N = 4
    binding.adama_fold(m, v, g, "f16", n, N, B1, B2)
    torch.cuda.synchronize()
    rm, rv = np.zeros(n), np.zeros(n)
    oracle.fold(rm, rv, bits, N, B1, B2, gdtype="f16")
    gm, gv = m.cpu().numpy().astype(np.float64), v.cpu().numpy().astype(np.float64)
    nz = rm != 0
    assert np.all(gm[~nz] == 0) and np.all(gv[~nz] == 0)
    assert np.max(np.abs(gm[nz] - rm[nz]) / np.abs(rm[nz])) <= 2.0 ** -22
    assert np.max(np.abs(gv[nz] - rv[nz]) / rv[nz]) <= 2.0 ** -22
    assert np.all(gv[nz] > 0), "a non-zero fp16 gradient (subnormals included) must leave v > 0"


def test_bf16_pattern_sweep(torch_cuda):
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    val = (bits.astype(np.uint32) << 16).view(np.float32)
    keep = np.isfinite(val) & (np.abs(val) < 1e15) & ((np.abs(val) > 1e-15) | (val == 0))
    bits = bits[keep]
    n = bits.size
    g = torch.from_numpy(bits.view(np.int16).copy()).cuda()
    m = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    v = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    binding.adama_fold(m, v, g, "bf16", n, 2, B1, B2)
    torch.cuda.synchronize()
    rm, rv = np.zeros(n), np.zeros(n)
    oracle.fold(rm, rv, bits, 2, B1, B2, gdtype="bf16")
    gm, gv = m.cpu().numpy().astype(np.float64), v.cpu().numpy().astype(np.float64)
    nz = rm != 0
    assert np.all(gm[~nz] == 0) and np.all(gv[~nz] == 0)
    assert np.max(np.abs(gm[nz] - rm[nz]) / np.abs(rm[nz])) <= 2.0 ** -22
    assert np.max(np.abs(gv[nz] - rv[nz]) / rv[nz]) <= 2.0 ** -22


# ---------------------------------------------------------------------------
# fold_multi == repeated fold, bit for bit; lists longer than one launch's table
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("gdt", ["f32", "bf16", "f16"])
def test_fold_multi_bitwise_equals_fold(torch_cuda, gdt):
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    rng = np.random.default_rng(5)
    cap = binding.adama_max_tensors_per_launch()
    sizes = [int(x) for x in rng.integers(0, 9000, 2 * cap + 9)] + [300001, (1 << 22) + 77, 0, 1]
    gbytes = synth.gen.DTYPE_BYTES[gdt]
    total = sum(sizes)
    arena = {k: torch.zeros(total + 8, dtype=torch.float32, device="cuda:0") for k in ("m1", "v1", "m2", "v2")}
    g = torch.zeros((total + 8) * gbytes, dtype=torch.uint8, device="cuda:0")
    synth.fill_device(g.data_ptr(), synth.Spec(key=99, sigma=1e-2, p_zero=0.01), gdt, total, 0)
    for k in ("m1", "m2"):
        synth.fill_device(arena[k].data_ptr(), synth.Spec(key=5, sigma=1e-3), "f32", total, 0)
    for k in ("v1", "v2"):
        synth.fill_device(arena[k].data_ptr(), synth.Spec(key=6, sigma=1e-4), "f32", total, 0)
        arena[k].abs_()
    entries1, entries2, off = [], [], 0
    for n in sizes:                      # packed back to back: every misalignment occurs
        entries1.append((arena["m1"].data_ptr() + 4 * off, arena["v1"].data_ptr() + 4 * off, g.data_ptr() + gbytes * off, n))
        entries2.append((arena["m2"].data_ptr() + 4 * off, arena["v2"].data_ptr() + 4 * off, g.data_ptr() + gbytes * off, n))
        off += n
    binding.adama_fold_multi(entries1, None, gdt, 4, B1, B2)
    for (pm, pv, pg, n) in entries2:
        binding.adama_fold(pm, pv, pg, gdt, n, 4, B1, B2)
    torch.cuda.synchronize()
    assert torch.equal(arena["m1"], arena["m2"]) and torch.equal(arena["v1"], arena["v2"])
    assert float(arena["m1"][total:].abs().sum()) == 0.0


def test_state_multi_bitwise_equals_single(torch_cuda):
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    rng = np.random.default_rng(6)
    sizes = [int(x) for x in rng.integers(0, 5000, 150)] + [(1 << 22) + 3]
    total = sum(sizes)
    a = {k: torch.zeros(total, dtype=torch.float32, device="cuda:0") for k in ("t1", "m1", "v1", "t2", "m2", "v2")}
    for s, (kt, km, kv) in enumerate((("t1", "m1", "v1"), ("t2", "m2", "v2"))):
        synth.fill_device(a[kt].data_ptr(), synth.Spec(key=1, sigma=0.02), "f32", total, 0)
        synth.fill_device(a[km].data_ptr(), synth.Spec(key=2, sigma=1e-3), "f32", total, 0)
        synth.fill_device(a[kv].data_ptr(), synth.Spec(key=3, sigma=1e-5), "f32", total, 0)
        a[kv].abs_()
    l1, l2, off = [], [], 0
    for n in sizes:
        l1.append((a["t1"].data_ptr() + 4 * off, a["m1"].data_ptr() + 4 * off, a["v1"].data_ptr() + 4 * off, n))
        l2.append((a["t2"].data_ptr() + 4 * off, a["m2"].data_ptr() + 4 * off, a["v2"].data_ptr() + 4 * off, n))
        off += n
    binding.adama_begin_step_multi(l1, None, B1, B2)
    binding.adama_apply_multi(l1, None, LR, EPS, B1, B2, 3)
    for (pt, pm, pv, n) in l2:
        binding.adama_begin_step(pm, pv, n, B1, B2)
    for (pt, pm, pv, n) in l2:
        binding.adama_apply(pt, pm, pv, n, LR, EPS, B1, B2, 3)
    torch.cuda.synchronize()
    for k in ("t", "m", "v"):
        assert torch.equal(a[k + "1"], a[k + "2"]), k


def test_begin_step_accepts_ddp_decay(torch_cuda):
    """Sec. 3.3: devices decay v by M*beta2 (> 1 allowed)."""
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    n = 10007
    m = torch.full((n,), 0.5, dtype=torch.float32, device="cuda:0")
    v = torch.full((n,), 0.25, dtype=torch.float32, device="cuda:0")
    binding.adama_begin_step(m, v, n, 0.9, 8 * 0.999)
    torch.cuda.synchronize()
    assert np.allclose(m.cpu().numpy(), np.float32(0.9) * np.float32(0.5), rtol=0, atol=0)
    assert np.allclose(v.cpu().numpy(), np.float32(8 * 0.999) * np.float32(0.25), rtol=0, atol=0)


# ---------------------------------------------------------------------------
# the five workloads at reduced size: every element, every step
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5"])
@pytest.mark.parametrize("pack", ["aligned", "tight"])
def test_reduced_workload_full_parity(torch_cuda, name, pack):
    w = configs.reduced(name)
    run = WorkloadRun(w, pack=pack, sampled=False)
    for step in range(1, w.steps + 1):
        stats = run.run_step(step, check_grad_bits=(step == 1 and pack == "aligned"))
        _log(f"{w.name} [{pack}] step {step}: {stats}")
    assert run.hb.peak_grad_bytes <= (w.largest_layer_elems + 128 * 32) * w.grad_bytes
    assert run.hb.peak_grad_bytes < run.hb.whole_model_grad_bytes


# ---------------------------------------------------------------------------
# fused edge forms: decay inside the first fold, update inside the last fold
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("gdt", ["f32", "bf16", "f16"])
def test_fused_edges_bitwise_equal_separate_calls(torch_cuda, gdt):
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    rng = np.random.default_rng(8)
    sizes = [int(x) for x in rng.integers(0, 9000, 100)] + [300001, (1 << 22) + 77, 0, 1, 5]
    gbytes = synth.gen.DTYPE_BYTES[gdt]
    total = sum(sizes)
    names = ("t", "m", "v")
    a = {k + s: torch.zeros(total + 8, dtype=torch.float32, device="cuda:0") for k in names for s in "12"}
    g = torch.zeros((total + 8) * gbytes, dtype=torch.uint8, device="cuda:0")
    synth.fill_device(g.data_ptr(), synth.Spec(key=77, sigma=1e-2, p_zero=0.01, p_outlier=0.001), gdt, total, 0)
    for s in "12":
        synth.fill_device(a["t" + s].data_ptr(), synth.Spec(key=1, sigma=0.02), "f32", total, 0)
        synth.fill_device(a["m" + s].data_ptr(), synth.Spec(key=2, sigma=1e-3), "f32", total, 0)
        synth.fill_device(a["v" + s].data_ptr(), synth.Spec(key=3, sigma=1e-5), "f32", total, 0)
        a["v" + s].abs_()
    fold1, fold2, upd1, st2, off = [], [], [], [], 0
    for n in sizes:                      # packed back to back: every misalignment occurs
        p = {k: a[k].data_ptr() + 4 * off for k in a}
        pg = g.data_ptr() + gbytes * off
        fold1.append((p["m1"], p["v1"], pg, n))
        upd1.append((p["t1"], p["m1"], p["v1"], pg, n))
        fold2.append((p["m2"], p["v2"], pg, n))
        st2.append((p["t2"], p["m2"], p["v2"], n))
        off += n
    N, t = 4, 3
    # fused: first fold carries the decay, last fold carries the update
    binding.adama_fold_first_multi(fold1, None, gdt, N, B1, B2)
    binding.adama_fold_multi(fold1, None, gdt, N, B1, B2)
    binding.adama_fold_last_apply_multi(upd1, None, gdt, N, LR, EPS, B1, B2, t)
    # separate calls
    binding.adama_begin_step_multi(st2, None, B1, B2)
    binding.adama_fold_multi(fold2, None, gdt, N, B1, B2)
    binding.adama_fold_multi(fold2, None, gdt, N, B1, B2)
    binding.adama_fold_multi(fold2, None, gdt, N, B1, B2)
    binding.adama_apply_multi(st2, None, LR, EPS, B1, B2, t)
    torch.cuda.synchronize()
    for k in names:
        assert torch.equal(a[k + "1"], a[k + "2"]), f"{k}: fused and separate paths differ"
    # single-tensor forms agree with the list forms
    b = {k: torch.zeros(70001, dtype=torch.float32, device="cuda:0") for k in ("t1", "m1", "v1", "t2", "m2", "v2")}
    for s in "12":
        synth.fill_device(b["t" + s].data_ptr(), synth.Spec(key=4, sigma=0.02), "f32", 70001, 0)
        synth.fill_device(b["m" + s].data_ptr(), synth.Spec(key=5, sigma=1e-3), "f32", 70001, 0)
    binding.adama_fold_first(b["m1"], b["v1"], g, gdt, 70001, N, B1, B2)
    binding.adama_fold_last_apply(b["t1"], b["m1"], b["v1"], g, gdt, 70001, N, LR, EPS, B1, B2, 1)
    binding.adama_begin_step(b["m2"], b["v2"], 70001, B1, B2)
    binding.adama_fold(b["m2"], b["v2"], g, gdt, 70001, N, B1, B2)
    binding.adama_fold(b["m2"], b["v2"], g, gdt, 70001, N, B1, B2)
    binding.adama_apply(b["t2"], b["m2"], b["v2"], 70001, LR, EPS, B1, B2, 1)
    torch.cuda.synchronize()
    for k in names:
        assert torch.equal(b[k + "1"], b[k + "2"]), f"{k}: single-tensor fused and separate paths differ"


@pytest.mark.parametrize("name", ["c1", "c3", "c4"])
def test_reduced_workload_fused_parity(torch_cuda, name):
    w = configs.reduced(name)
    run = WorkloadRun(w, pack="tight", sampled=False, fused=True)
    for step in range(1, w.steps + 1):
        stats = run.run_step(step)
        _log(f"{w.name} [fused] step {step}: {stats}")


@pytest.mark.parametrize("name,fused", [("c4", False), ("c3", True), ("c2", False)])
def test_folds_spread_over_streams_give_the_same_bits(torch_cuda, name, fused):
    """fold_streams > 1: layer l is produced and folded on stream l mod k with a gradient buffer per stream;
    the arithmetic and its order per element are unchanged, so two and three streams give the single
    stream's bits, and the oracle agrees; peak gradient memory is k layers."""
    torch = torch_cuda
    w = configs.reduced(name)
    outs, peaks = [], []
    for k in (1, 2, 3):
        run = WorkloadRun(w, pack="tight", sampled=False, fused=fused, fold_streams=k)
        for step in range(1, w.steps + 1):
            stats = run.run_step(step, check_grad_bits=(k == 2 and step == 1))
        _log(f"{w.name} fold_streams={k}: {stats}")
        run.hb.synchronize()
        outs.append([x.clone() for x in (run.hb.theta, run.hb.m, run.hb.v)])
        peaks.append(run.hb.peak_grad_bytes)
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert torch.equal(a, b)
    assert peaks[0] < peaks[1] <= 2 * peaks[0] + 1024 and peaks[1] < peaks[2] <= 3 * peaks[0] + 2048


# ---------------------------------------------------------------------------
# Sec. 3.3: M simulated devices on one GPU == one device with N*M micro-batches
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("M,N", [(2, 4), (4, 2), (3, 3)])
def test_data_parallel_state_sync_arithmetic(torch_cuda, M, N):
    """Each simulated device decays v by M*beta2 and folds its own N micro-batches with 1/N; the summed
    states (a torch add stands in for the all-reduce) go through adama_rescale_apply(1/M, 1/M^2).  The
    result must match the oracle's multi-device combine AND the oracle's single-device N*M run."""
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    n, T, gdt = 100003, 2, "bf16"
    theta0 = synth.fill_host(synth.Spec(key=41, sigma=0.02), "f32", n)
    theta = torch.from_numpy(theta0).cuda()
    m_sync = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    v_sync = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    g = torch.zeros(n * 2, dtype=torch.uint8, device="cuda:0")
    single = oracle.OracleState([theta0])                  # one device, N*M micro-batches
    ddp_theta = theta0.astype(np.float64)
    ddp_m, ddp_v = np.zeros(n), np.zeros(n)
    prev_gpu, prev_ref = theta0.copy(), theta0.astype(np.float64)
    for t in range(1, T + 1):
        single.begin_step(B1, B2)
        m_r = np.repeat(ddp_m[None, :], M, axis=0)
        v_r = np.repeat(ddp_v[None, :], M, axis=0)
        m_sum = torch.zeros_like(m_sync)
        v_sum = torch.zeros_like(v_sync)
        for r in range(M):
            m_dev, v_dev = m_sync.clone(), v_sync.clone()
            binding.adama_begin_step(m_dev, v_dev, n, B1, M * B2)
            oracle.begin_step(m_r[r], v_r[r], B1, M * B2)
            for i in range(N):
                spec = synth.Spec(key=synth.stream_key(43, t, r, i), sigma=3e-3, p_outlier=1e-3)
                synth.fill_device(g.data_ptr(), spec, gdt, n, 0)
                binding.adama_fold(m_dev, v_dev, g, gdt, n, N, B1, B2)
                host = synth.fill_host(spec, gdt, n)
                oracle.fold(m_r[r], v_r[r], host, N, B1, B2, gdtype=gdt)
                single.fold(0, host, N * M, B1, B2, gdtype=gdt)
            m_sum += m_dev                                   # stand-in for the all-reduce (sum)
            v_sum += v_dev
        binding.adama_rescale_apply(theta, m_sum, v_sum, n, 1.0 / M, 1.0 / (M * M), LR, EPS, B1, B2, t)
        m_sync, v_sync = m_sum, v_sum
        ddp_m, ddp_v = oracle.ddp_combine(m_r, v_r)
        oracle.apply(ddp_theta, ddp_m, ddp_v, LR, EPS, B1, B2, t)
        single.apply(LR, EPS, B1, B2)
        torch.cuda.synchronize()
        th = theta.cpu().numpy()
        for label, rm, rv, rt in (("vs oracle combine", ddp_m, ddp_v, ddp_theta),
                                  ("vs single device N*M", single.m[0], single.v[0], single.theta[0])):
            name = f"ddp M={M} N={N} t={t} {label}"
            check_close(name, "m", m_sync.cpu().numpy(), rm)
            check_close(name, "v", v_sync.cpu().numpy(), rv)
            check_close(name, "theta", th, rt, prev_gpu, prev_ref)
        prev_gpu, prev_ref = th.copy(), ddp_theta.copy()


# ---------------------------------------------------------------------------
# HIP graph of a launch-bound sweep (many small tensors): replays equal eager launches bit for bit
# ---------------------------------------------------------------------------
def test_graph_replay_of_ragged_sweep_equals_eager(torch_cuda):
    torch = torch_cuda
    from paper_2305_19982_amd.harness import SimulatedBackward

    w = configs.reduced("c4")
    runs = {}
    for mode in ("eager", "graph"):
        hb = SimulatedBackward([t.n for t in w.tensors], w.layers, w.gdtype, grad_buffer="model")
        for t in w.tensors:
            synth.fill_device(hb.theta_ptr(t.index), w.theta_spec(t.index), "f32", t.n, hb.stream_handle)

        def sweep(hb=hb):
            for li in w.backward_layers():
                hb.fold_layer(li, w.N, w.beta1, w.beta2)

        graph = hb.capture(sweep) if mode == "graph" else None
        if graph is not None:           # capture does not execute: state is still untouched
            hb.synchronize()
            assert float(hb.m.abs().sum()) == 0.0
        for step in range(1, 3):
            hb.begin_step(w.beta1, w.beta2)
            for i in range(w.N):
                for t in w.tensors:     # new gradients before every replay, by eager launches between replays
                    synth.fill_device(hb.grad_ptr(t.index), w.grad_spec(step, i, t.index), w.gdtype, t.n, hb.stream_handle)
                if graph is not None:
                    with torch.cuda.stream(hb.stream):
                        graph.replay()
                else:
                    sweep()
                hb.synchronize()        # host synchronisation between replays
            hb.apply(w.lr, w.eps, w.beta1, w.beta2)
        hb.synchronize()
        runs[mode] = (hb.theta.clone(), hb.m.clone(), hb.v.clone())
    for a, b, name in zip(runs["eager"], runs["graph"], ("theta", "m", "v")):
        assert torch.equal(a, b), f"{name}: graph replay differs from eager launches"
    assert float(runs["graph"][2].sum()) > 0.0


# ---------------------------------------------------------------------------
# degenerate hyper-parameters and special values
# ---------------------------------------------------------------------------
def _one_step_against_oracle(torch, n, N, b1, b2, lr, eps, t, gdt="f32", grad_values=None, m0=None, v0=None):
    from paper_2305_19982_amd import binding

    key = synth.stream_key(77, n, N, t)
    th0 = synth.fill_host(synth.Spec(key=key, sigma=0.02), "f32", n)
    m0 = np.zeros(n, dtype=np.float32) if m0 is None else m0.astype(np.float32)
    v0 = np.zeros(n, dtype=np.float32) if v0 is None else v0.astype(np.float32)
    theta, m, v = (torch.from_numpy(x.copy()).cuda() for x in (th0, m0, v0))
    ref = oracle.OracleState([th0])
    ref.m[0][:] = m0
    ref.v[0][:] = v0
    ref.t = t - 1
    binding.adama_begin_step(m, v, n, b1, b2)
    ref.begin_step(b1, b2)
    for i in range(N):
        if grad_values is None:
            g_host = synth.fill_host(synth.Spec(key=key + 1 + i, sigma=1e-2), gdt, n)
        else:
            g_host = grad_values[i]
        g = torch.from_numpy(g_host.view(np.int16) if g_host.dtype == np.uint16 else g_host).cuda()
        binding.adama_fold(m, v, g, gdt, n, N, b1, b2)
        ref.fold(0, g_host, N, b1, b2, gdtype=None if gdt == "f32" else gdt)
    binding.adama_apply(theta, m, v, n, lr, eps, b1, b2, t)
    ref.apply(lr, eps, b1, b2)
    torch.cuda.synchronize()
    return (theta.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy()), ref, th0


@pytest.mark.parametrize("b1,b2,lr,eps,t", [(0.0, 0.999, 1e-3, 1e-8, 1), (0.9, 0.0, 1e-3, 1e-8, 1), (0.0, 0.0, 1e-2, 1e-6, 3),
                                            (0.9, 0.999, 0.0, 1e-8, 2), (0.9, 0.999, 1e-3, 0.0, 5), (0.9, 0.999, 1e-3, 1e-8, 1000),
                                            (0.99, 0.9999, 3e-4, 1e-12, 100000), (0.5, 0.5, -1e-3, 1e-3, 7)])
def test_degenerate_hyper_parameters(torch_cuda, b1, b2, lr, eps, t):
    n, N = 40961, 3
    rng = np.random.default_rng(t)
    m0 = rng.standard_normal(n) * 1e-3
    v0 = np.abs(rng.standard_normal(n)) * 1e-5 + 1e-12          # v > 0 so that eps = 0 is well defined
    (th, m, v), ref, th0 = _one_step_against_oracle(torch_cuda, n, N, b1, b2, lr, eps, t, m0=m0, v0=v0)
    name = f"b1={b1} b2={b2} lr={lr} eps={eps} t={t}"
    check_close(name, "m", m, ref.m[0])
    check_close(name, "v", v, ref.v[0])
    check_close(name, "theta", th, ref.theta[0], th0, th0.astype(np.float64))
    if lr == 0.0:
        assert np.array_equal(th, th0), "lr = 0 must leave theta untouched, bit for bit"


def test_non_finite_gradients_propagate_by_ieee_rules(torch_cuda):
    """No skip logic: an inf or nan gradient poisons exactly its own element, as in the oracle."""
    n, N = 5000, 2
    g0 = synth.fill_host(synth.Spec(key=5, sigma=1e-2), "f32", n)
    g1 = synth.fill_host(synth.Spec(key=6, sigma=1e-2), "f32", n)
    g0[7], g0[8], g1[9], g0[4097] = np.inf, -np.inf, np.nan, np.inf
    (th, m, v), ref, th0 = _one_step_against_oracle(torch_cuda, n, N, B1, B2, LR, EPS, 1, grad_values=[g0, g1])
    bad = np.zeros(n, dtype=bool)
    bad[[7, 8, 9, 4097]] = True
    with np.errstate(invalid="ignore"):
        assert np.array_equal(np.isnan(th), np.isnan(ref.theta[0])) and np.array_equal(np.isnan(th), bad)
        assert np.array_equal(np.isinf(m), np.isinf(ref.m[0])) and np.array_equal(np.isnan(m), np.isnan(ref.m[0]))
        assert np.array_equal(np.isinf(v), np.isinf(ref.v[0])) and np.array_equal(np.isnan(v), np.isnan(ref.v[0]))
    ok = ~bad
    check_close("finite part", "m", m[ok], ref.m[0][ok])
    check_close("finite part", "v", v[ok], ref.v[0][ok])
    check_close("finite part", "theta", th[ok], ref.theta[0][ok])


def test_float32_subnormal_moments_are_kept(torch_cuda):
    """Denormal m and v are not flushed to zero by the decay or the fold."""
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    n = 4099
    tiny = np.float32(1e-41)
    m = torch.full((n,), float(tiny), dtype=torch.float32, device="cuda:0")
    v = torch.full((n,), float(tiny), dtype=torch.float32, device="cuda:0")
    g = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    binding.adama_begin_step(m, v, n, 0.5, 0.5)
    binding.adama_fold(m, v, g, "f32", n, 4, 0.9, 0.999)
    torch.cuda.synchronize()
    want = np.float32(tiny * np.float32(0.5))
    assert want > 0
    assert np.all(m.cpu().numpy() == want) and np.all(v.cpu().numpy() == want)


def test_concurrent_host_threads_on_their_own_streams(torch_cuda):
    """No shared mutable state in the library: two host threads drive independent tensors at once."""
    import threading

    torch = torch_cuda
    from paper_2305_19982_amd import binding

    n, N, rounds = 300007, 4, 20
    results, errors = {}, []

    def worker(idx):
        try:
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                m = torch.zeros(n, dtype=torch.float32, device="cuda:0")
                v = torch.zeros(n, dtype=torch.float32, device="cuda:0")
                g = torch.zeros(n * 2, dtype=torch.uint8, device="cuda:0")
            stream.synchronize()
            for r in range(rounds):
                synth.fill_device(g.data_ptr(), synth.Spec(key=1000 + r, sigma=1e-2), "bf16", n, stream.cuda_stream)
                binding.adama_fold(m, v, g, "bf16", n, N, B1, B2, stream.cuda_stream)
                try:
                    binding.adama_fold(m, None, g, "bf16", n, N, B1, B2, stream.cuda_stream)   # errors stay thread-local
                except binding.AdamaError as e:
                    assert "v is NULL" in e.message
            stream.synchronize()
            results[idx] = (m.cpu().numpy(), v.cpu().numpy())
        except Exception as e:   # noqa: BLE001
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    assert np.array_equal(results[0][0], results[1][0]) and np.array_equal(results[0][1], results[1][1])
    rm, rv = np.zeros(n), np.zeros(n)
    for r in range(rounds):
        oracle.fold(rm, rv, synth.fill_host(synth.Spec(key=1000 + r, sigma=1e-2), "bf16", n), N, B1, B2, gdtype="bf16")
    check_close("threads", "m", results[0][0], rm)
    check_close("threads", "v", results[0][1], rv)


@pytest.mark.parametrize("optimizer", ["adam", "sgdm"])
def test_arena_placement_does_not_change_results(torch_cuda, optimizer):
    """Where the state lives does not change the results: separate allocations, one slab with the arenas a chosen
    multiple of 2 MiB apart and staggered against each other, or the fastest of the placements the harness tried
    (placement_tries allocations x pitch_tries pitches inside each slab: it times decay, folds and update on each
    candidate with scratch contents, keeps the best and hands it over zeroed); bit-identical state after a
    mini-batch."""
    torch = torch_cuda
    from paper_2305_19982_amd.harness import SimulatedBackward

    w = configs.reduced("c3")
    outs = []
    for layout, stagger, extra, tries, pitches in (("separate", 0, 0, 1, 1), ("slab", 0, 0, 1, 1), ("slab", 4096, 0, 1, 1),
                                                   ("slab", 0, 1, 1, 1), ("separate", 0, 0, 3, 1), ("slab", 4096, 2, 2, 3),
                                                   ("slab", 0, 0, 1, 4)):
        hb = SimulatedBackward([t.n for t in w.tensors], w.layers, w.gdtype, pack="tight", arena_layout=layout,
                               arena_stagger_bytes=stagger, arena_pitch_extra=extra, optimizer=optimizer,
                               placement_tries=tries, pitch_tries=pitches, placement_micro_batches=w.N)
        hb.synchronize()
        pl = hb.placement
        assert pl["tries"] == tries and pl["pitch_tries"] == pitches
        searched = tries > 1 or pitches > 1
        assert [len(row) for row in pl["step_ms"]] == ([pitches] * tries if searched else [])
        assert 0 <= pl["chosen"][0] < tries and 0 <= pl["chosen"][1] < pitches
        if searched:
            assert pl["step_ms"][pl["chosen"][0]][pl["chosen"][1]] == min(min(row) for row in pl["step_ms"])
        for arena in (hb.theta, hb.m, hb.v):
            assert arena is None or not bool(arena.any())            # handed over zeroed
        for t in w.tensors:
            synth.fill_device(hb.theta_ptr(t.index), w.theta_spec(t.index), "f32", t.n, hb.stream_handle)

        def produce(i, li, hb=hb):
            for ti in w.layers[li]:
                synth.fill_device(hb.grad_ptr(ti), w.grad_spec(1, i, ti), w.gdtype, w.tensors[ti].n, hb.stream_handle)

        hb.mini_batch(produce, w.N, w.lr, w.eps, w.beta1, w.beta2)
        hb.synchronize()
        kinds = ("theta", "m", "v") if optimizer == "adam" else ("theta", "b")
        outs.append([torch.cat([hb.tensor_view(k, t.index) for t in w.tensors]).clone() for k in kinds])
        if layout == "slab":           # consecutive arenas: the reported pitch (a multiple of 2 MiB) plus the stagger apart
            other = hb.v if optimizer == "adam" else hb.theta
            first = -(-(hb.arena_elems * 4 + 2 * stagger) // (1 << 21)) + extra
            assert pl["pitch_extras_2mib"][:2] == [0, 1][:pitches] and len(pl["pitch_extras_2mib"]) == pitches
            assert pl["pitch_2mib"] == first + pl["pitch_extras_2mib"][pl["chosen"][1]]
            assert all((first + x) % 128 in (0, 1) for x in pl["pitch_extras_2mib"][2:])
            assert other.data_ptr() - hb.m.data_ptr() == pl["pitch_2mib"] * (1 << 21) + stagger
            assert hb.m.data_ptr() % (1 << 21) == 0
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert torch.equal(a, b)


def test_three_hundred_mini_batches_stay_within_tolerance(torch_cuda):
    """Rounding errors of the float32 state do not build up beyond the tolerance over a long run: 300
    mini-batches of 2 micro-batches (the second moment averages over about 1000 steps, so this is a third
    of its memory), compared with the oracle after every 50th update."""
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    n, N, steps = 8191, 2, 300
    th = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    m = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    v = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    g = torch.zeros(n, dtype=torch.bfloat16, device="cuda:0")
    th0 = synth.fill_host(synth.Spec(key=synth.stream_key(83, 0), sigma=0.02), "f32", n)
    th.copy_(torch.from_numpy(th0))
    ref = oracle.OracleState([th0])
    prev_gpu, prev_ref = th0.copy(), ref.theta[0].copy()
    for t in range(1, steps + 1):
        ref.begin_step(B1, B2)
        for i in range(N):
            spec = synth.Spec(key=synth.stream_key(83, t, i), sigma=3e-3, p_zero=0.01, p_outlier=0.001)
            synth.fill_device(g.data_ptr(), spec, "bf16", n, 0)
            if i == 0:
                binding.adama_fold_first(m, v, g, "bf16", n, N, B1, B2)
            else:
                binding.adama_fold_last_apply(th, m, v, g, "bf16", n, N, LR, EPS, B1, B2, t)
            ref.fold(0, synth.fill_host(spec, "bf16", n), N, B1, B2, gdtype="bf16")
        ref.apply(LR, EPS, B1, B2)
        if t % 50 == 0:
            torch.cuda.synchronize()
            name = f"long run t={t}"
            sm = check_close(name, "m", m.cpu().numpy(), ref.m[0])
            sv = check_close(name, "v", v.cpu().numpy(), ref.v[0])
            got = th.cpu().numpy()
            # theta itself: the binding criterion; its change over the last 50 steps on the change's own scale
            err = np.abs(got.astype(np.float64) - ref.theta[0])
            assert np.all(err <= np.maximum(1e-5 * np.abs(ref.theta[0]), 1e-6)), f"{name}: theta off by {err.max():.3e}"
            d_gpu, d_ref = got.astype(np.float64) - prev_gpu, ref.theta[0] - prev_ref
            scale = np.sqrt(np.mean(d_ref ** 2))
            assert np.max(np.abs(d_gpu - d_ref)) <= 1e-5 * scale * 50 + 50 * 2.0 ** -24 * np.max(np.abs(got))
            prev_gpu, prev_ref = got.astype(np.float64), ref.theta[0].copy()
            _log(f"{name}: m {sm} v {sv} theta max abs err {err.max():.3e}")
