"""GPU parity of the variant calls (decoupled weight decay, gradient scale, SGD with momentum) against
the fp64 oracle, and their bit-for-bit relations to the plain calls."""
import numpy as np
import pytest

import oracle
import synth
from parity import WorkloadRun, check_close
from synth import configs

pytestmark = pytest.mark.gpu

B1, B2, LR, EPS = 0.9, 0.999, 1e-3, 1e-8
# two ragged lists packed back to back (every misalignment occurs): one short enough for the
# 1024-element chunks, one long enough for the larger chunks of long launches
SMALL = [0, 1, 2, 3, 5, 64, 1023, 1024, 1025, 4097, 12289, 0, 70001]
BIG = [7, 300001, (1 << 22) + 77, 0, 4096 * 3 + 1, 65536, 9]


@pytest.fixture(scope="module")
def torch_cuda():
    import torch

    assert torch.cuda.is_available()
    from paper_2305_19982_amd import binding

    binding.load()
    return torch


class Packed:
    """float32 arrays `names` and one gradient buffer over a ragged list of tensors packed back to back."""

    def __init__(self, torch, sizes, gdt, names, seed):
        self.torch, self.sizes, self.gdt, self.names = torch, sizes, gdt, names
        self.gbytes = synth.gen.DTYPE_BYTES[gdt]
        self.total = sum(sizes)
        self.offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
        self.dev = {k: torch.zeros(self.total + 8, dtype=torch.float32, device="cuda:0") for k in names}
        self.g = torch.zeros((self.total + 8) * self.gbytes, dtype=torch.uint8, device="cuda:0")
        self.seed = seed

    def fill(self, name, key, sigma, absolute=False):
        spec = synth.Spec(key=synth.stream_key(self.seed, key), sigma=sigma)
        synth.fill_device(self.dev[name].data_ptr(), spec, "f32", self.total, 0)
        host = synth.fill_host(spec, "f32", self.total)
        if absolute:
            self.dev[name].abs_()
            host = np.abs(host)
        return host

    def fill_grad(self, key, sigma):
        # heavy-tailed outliers stay inside float16's range also when the stream is scaled up
        spec = synth.Spec(key=synth.stream_key(self.seed, 1000 + key), sigma=sigma, p_zero=0.02, p_outlier=0.001,
                          outlier_scale=10.0 if sigma < 1.0 else 2.0, p_sub=0.02 if self.gdt == "f16" else 0.0)
        synth.fill_device(self.g.data_ptr(), spec, self.gdt, self.total, 0)
        return synth.fill_host(spec, self.gdt, self.total)

    def entries(self, *fields):
        """Tuples of per-tensor device addresses; field "g" is the gradient, "n" the length, None stays None."""
        out = []
        for i, n in enumerate(self.sizes):
            off = int(self.offs[i])
            row = []
            for f in fields:
                if f is None:
                    row.append(None)
                elif f == "n":
                    row.append(n)
                elif f == "g":
                    row.append(self.g.data_ptr() + self.gbytes * off)
                else:
                    row.append(self.dev[f].data_ptr() + 4 * off)
            out.append(tuple(row))
        return out

    def host(self, name):
        self.torch.cuda.synchronize()
        return self.dev[name][: self.total].cpu().numpy()

    def untouched_tail(self):
        self.torch.cuda.synchronize()
        return all(float(x[self.total:].abs().sum()) == 0.0 for x in self.dev.values())


# ---------------------------------------------------------------------------
# options that say "nothing" change no bit
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("gdt", ["f32", "bf16", "f16"])
def test_default_options_are_bitwise_the_plain_calls(torch_cuda, gdt):
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    for sizes in (SMALL, BIG):
        p = Packed(torch, sizes, gdt, ("t1", "m1", "v1", "t2", "m2", "v2"), seed=41)
        for s in "12":
            p.fill("t" + s, 1, 0.02)
            p.fill("m" + s, 2, 1e-3)
            p.fill("v" + s, 3, 1e-5, absolute=True)
        p.fill_grad(0, 1e-2)
        N, t = 4, 3
        f1, u1, s1 = p.entries("m1", "v1", "g", "n"), p.entries("t1", "m1", "v1", "g", "n"), p.entries("t1", "m1", "v1", "n")
        f2, u2, s2 = p.entries("m2", "v2", "g", "n"), p.entries("t2", "m2", "v2", "g", "n"), p.entries("t2", "m2", "v2", "n")
        for opt in (None, (0.0, 1.0), binding.options()):
            binding.adama_fold_first_opt_multi(f1, None, gdt, N, B1, B2, opt)
            binding.adama_fold_opt_multi(f1, None, gdt, N, B1, B2, opt)
            binding.adama_fold_last_apply_opt_multi(u1, None, gdt, N, LR, EPS, B1, B2, t, opt)
            binding.adama_apply_opt_multi(s1, None, LR, EPS, B1, B2, t + 1, opt)
            binding.adama_rescale_apply_opt_multi(s1, None, 0.5, 0.25, LR, EPS, B1, B2, t + 2, opt)
            binding.adama_fold_first_multi(f2, None, gdt, N, B1, B2)
            binding.adama_fold_multi(f2, None, gdt, N, B1, B2)
            binding.adama_fold_last_apply_multi(u2, None, gdt, N, LR, EPS, B1, B2, t)
            binding.adama_apply_multi(s2, None, LR, EPS, B1, B2, t + 1)
            binding.adama_rescale_apply_multi(s2, None, 0.5, 0.25, LR, EPS, B1, B2, t + 2)
            torch.cuda.synchronize()
            for k in "tmv":
                assert torch.equal(p.dev[k + "1"], p.dev[k + "2"]), f"{k}: default options changed bits ({opt})"


# ---------------------------------------------------------------------------
# AdamW + loss scale against the oracle, separate and fused call sequences
# ---------------------------------------------------------------------------
def _adam_variant_steps(torch, sizes, gdt, fused, wd, scale, steps=3, N=4, lr=LR):
    from paper_2305_19982_amd import binding

    p = Packed(torch, sizes, gdt, ("t", "m", "v"), seed=43)
    th = p.fill("t", 1, 0.05).astype(np.float64)
    m = np.zeros(p.total)
    v = np.zeros(p.total)
    fold, upd, st = p.entries("m", "v", "g", "n"), p.entries("t", "m", "v", "g", "n"), p.entries("t", "m", "v", "n")
    opt = binding.options(wd, scale)
    gd = None if gdt == "f32" else gdt
    prev_gpu, prev_ref = p.host("t"), th.copy()
    for t in range(1, steps + 1):
        if not fused:
            binding.adama_begin_step_multi(st, None, B1, B2)
        oracle.begin_step(m, v, B1, B2)
        for i in range(N):
            # gradients are stored 1/scale times too large, as a scaled loss produces them
            g = p.fill_grad(100 * t + i, 1e-2 / scale)
            if fused and i == 0 and N > 1:
                binding.adama_fold_first_opt_multi(fold, None, gdt, N, B1, B2, opt)
            elif fused and i == N - 1:
                if N == 1:
                    binding.adama_begin_step_multi(st, None, B1, B2)
                binding.adama_fold_last_apply_opt_multi(upd, None, gdt, N, lr, EPS, B1, B2, t, opt)
            else:
                binding.adama_fold_opt_multi(fold, None, gdt, N, B1, B2, opt)
            oracle.fold_scaled(m, v, g, N, B1, B2, scale, gdtype=gd)
        if not fused:
            binding.adama_apply_opt_multi(st, None, lr, EPS, B1, B2, t, opt)
        oracle.apply_adamw(th, m, v, lr, EPS, B1, B2, t, wd)
        name = f"adamw {gdt} fused={fused} wd={wd} scale={scale} t={t}"
        check_close(name, "m", p.host("m"), m)
        check_close(name, "v", p.host("v"), v)
        gpu_t = p.host("t")
        check_close(name, "theta", gpu_t, th, prev_gpu, prev_ref)
        prev_gpu, prev_ref = gpu_t, th.copy()
    assert p.untouched_tail()
    return p


@pytest.mark.parametrize("gdt,scale", [("f32", 1.0), ("bf16", 1.0 / 128.0), ("f16", 1.0 / 1024.0), ("f16", 1.0 / 3.0)])
@pytest.mark.parametrize("fused", [False, True])
def test_adamw_with_loss_scale_parity(torch_cuda, gdt, scale, fused):
    for sizes in (SMALL, BIG):
        _adam_variant_steps(torch_cuda, sizes, gdt, fused, wd=0.1, scale=scale)


def test_adamw_fused_bitwise_equals_separate(torch_cuda):
    a = _adam_variant_steps(torch_cuda, BIG, "bf16", False, wd=0.05, scale=0.25, steps=2)
    b = _adam_variant_steps(torch_cuda, BIG, "bf16", True, wd=0.05, scale=0.25, steps=2)
    for k in "tmv":
        assert torch_cuda.equal(a.dev[k], b.dev[k]), f"{k}: fused and separate AdamW paths differ"


def test_weight_decay_alone_shrinks_parameters(torch_cuda):
    """Zero moments: theta_T = theta_0 (1 - lr*lambda)^T up to one float32 rounding per step."""
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    p = Packed(torch, SMALL, "f32", ("t", "m", "v"), seed=47)
    th0 = p.fill("t", 1, 1.0).astype(np.float64)
    st = p.entries("t", "m", "v", "n")
    lr, wd, T = 0.05, 0.3, 5
    for t in range(1, T + 1):
        binding.adama_apply_opt_multi(st, None, lr, EPS, B1, B2, t, (wd, 1.0))
    got = p.host("t").astype(np.float64)
    ref = th0 * (1.0 - lr * wd) ** T
    assert np.all(np.abs(got - ref) <= T * 2.0 ** -23 * np.abs(ref))
    assert float(p.dev["m"].abs().sum()) == 0.0 and float(p.dev["v"].abs().sum()) == 0.0


def test_rescale_apply_with_weight_decay_parity(torch_cuda):
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    p = Packed(torch, BIG, "f32", ("t", "m", "v"), seed=53)
    th = p.fill("t", 1, 0.05).astype(np.float64)
    m = p.fill("m", 2, 4e-3).astype(np.float64)
    v = p.fill("v", 3, 16e-6, absolute=True).astype(np.float64)
    M, t, wd = 4, 7, 0.1
    prev = p.host("t")
    binding.adama_rescale_apply_opt_multi(p.entries("t", "m", "v", "n"), None, 1.0 / M, 1.0 / (M * M), LR, EPS, B1, B2, t,
                                          (wd, 1.0))
    th0 = th.copy()
    m, v = m / M, v / (M * M)
    oracle.apply_adamw(th, m, v, LR, EPS, B1, B2, t, wd)
    check_close("rescale wd", "m", p.host("m"), m)
    check_close("rescale wd", "v", p.host("v"), v)
    check_close("rescale wd", "theta", p.host("t"), th, prev, th0)


# ---------------------------------------------------------------------------
# SGD with momentum
# ---------------------------------------------------------------------------
def _sgdm_steps(torch, sizes, gdt, fused, wd, scale, mu=0.9, lr=0.05, steps=3, N=4):
    from paper_2305_19982_amd import binding

    p = Packed(torch, sizes, gdt, ("t", "b"), seed=59)
    th = p.fill("t", 1, 0.05).astype(np.float64)
    b = np.zeros(p.total)
    lst = p.entries("t", "b", "g", "n")
    opt = binding.options(wd, scale)
    gd = None if gdt == "f32" else gdt
    prev_gpu, prev_ref = p.host("t"), th.copy()
    for t in range(1, steps + 1):
        if not fused:
            binding.adama_sgdm_begin_step_multi(lst, None, mu)
        oracle.sgdm_begin_step(b, mu)
        for i in range(N):
            g = p.fill_grad(100 * t + i, 1e-2 / scale)
            if fused and i == 0 and N > 1:
                binding.adama_sgdm_fold_first_multi(lst, None, gdt, N, mu, opt)
            elif fused and i == N - 1:
                if N == 1:
                    binding.adama_sgdm_begin_step_multi(lst, None, mu)
                binding.adama_sgdm_fold_last_apply_multi(lst, None, gdt, N, lr, opt)
            else:
                binding.adama_sgdm_fold_multi(lst, None, gdt, N, opt)
            oracle.sgdm_fold(b, g, N, scale, gdtype=gd)
        if not fused:
            binding.adama_sgdm_apply_multi(lst, None, lr, opt)
        oracle.sgdm_apply(th, b, lr, wd)
        name = f"sgdm {gdt} fused={fused} wd={wd} scale={scale} t={t}"
        check_close(name, "m", p.host("b"), b)
        gpu_t = p.host("t")
        check_close(name, "theta", gpu_t, th, prev_gpu, prev_ref)
        prev_gpu, prev_ref = gpu_t, th.copy()
    assert p.untouched_tail()
    return p


@pytest.mark.parametrize("gdt,scale", [("f32", 1.0), ("bf16", 1.0), ("f16", 1.0 / 1024.0)])
@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("wd", [0.0, 0.1])
def test_sgdm_parity(torch_cuda, gdt, scale, fused, wd):
    for sizes in (SMALL, BIG):
        _sgdm_steps(torch_cuda, sizes, gdt, fused, wd, scale)


@pytest.mark.parametrize("gdt", ["f32", "bf16", "f16"])
def test_sgdm_fused_bitwise_equals_separate(torch_cuda, gdt):
    for sizes in (SMALL, BIG):
        a = _sgdm_steps(torch_cuda, sizes, gdt, False, 0.05, 0.5, steps=2)
        b = _sgdm_steps(torch_cuda, sizes, gdt, True, 0.05, 0.5, steps=2)
        for k in "tb":
            assert torch_cuda.equal(a.dev[k], b.dev[k]), f"{k}: fused and separate SGD paths differ"


def test_sgdm_single_micro_batch_and_zero_momentum(torch_cuda):
    _sgdm_steps(torch_cuda, SMALL, "f32", False, 0.0, 1.0, mu=0.0, N=1)
    _sgdm_steps(torch_cuda, SMALL, "bf16", True, 0.0, 1.0, mu=0.0, N=1)
    _sgdm_steps(torch_cuda, BIG, "f16", True, 0.0, 1.0, mu=0.99, N=2)


def test_sgdm_matches_library_sgd_on_mean_gradient(torch_cuda):
    """The accumulated buffer is the library's momentum buffer on the mean gradient (float32 on the GPU
    against torch.optim.SGD in float64 on the CPU)."""
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    n, N, mu, lr, T = 50001, 4, 0.9, 0.05, 3
    p = Packed(torch, [n], "f32", ("t", "b"), seed=61)
    th0 = p.fill("t", 1, 0.05).astype(np.float64)
    q = torch.nn.Parameter(torch.from_numpy(th0.copy()))
    opt = torch.optim.SGD([q], lr=lr, momentum=mu)
    lst = p.entries("t", "b", "g", "n")
    for t in range(1, T + 1):
        binding.adama_sgdm_begin_step_multi(lst, None, mu)
        mean = np.zeros(n)
        for i in range(N):
            mean += p.fill_grad(10 * t + i, 1e-2).astype(np.float64) / N
            binding.adama_sgdm_fold_multi(lst, None, "f32", N)
        binding.adama_sgdm_apply_multi(lst, None, lr)
        q.grad = torch.from_numpy(mean.copy())
        opt.step()
    check_close("library SGD", "m", p.host("b"), opt.state[q]["momentum_buffer"].numpy())
    check_close("library SGD", "theta", p.host("t"), q.detach().numpy())


# ---------------------------------------------------------------------------
# the variants on the benchmark workloads (harness, one reusable gradient buffer), reduced and full size
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["c1", "c3", "c4"])
@pytest.mark.parametrize("fused", [False, True])
def test_reduced_workload_momentum_sgd(torch_cuda, name, fused):
    w = configs.reduced(name)
    run = WorkloadRun(w, pack="tight", fused=fused, optimizer="sgdm", momentum=0.9, weight_decay=0.01)
    for step in range(1, w.steps + 1):
        stats = run.run_step(step)
        print(f"{w.name} [sgdm fused={fused}] step {step}: {stats}", flush=True)


@pytest.mark.parametrize("name", ["c1", "c3", "c4"])
@pytest.mark.parametrize("fused", [False, True])
def test_reduced_workload_adamw_scaled(torch_cuda, name, fused):
    w = configs.reduced(name)
    run = WorkloadRun(w, pack="aligned", fused=fused, weight_decay=0.01, grad_scale=1.0 / 64.0)
    for step in range(1, w.steps + 1):
        stats = run.run_step(step)
        print(f"{w.name} [adamw scaled fused={fused}] step {step}: {stats}", flush=True)


@pytest.mark.parametrize("optimizer", ["sgdm", "adamw"])
def test_full_size_c3_variants_sampled(torch_cuda, optimizer):
    """The GPT-2-1.5B-shaped workload at full size through the variant entry points (fused edges, as
    bench.py --optimizer runs them), compared on sampled slices of every tensor."""
    w = configs.FULL["c3"]()
    kw = dict(optimizer="sgdm", momentum=0.9) if optimizer == "sgdm" else dict(weight_decay=0.01)
    run = WorkloadRun(w, pack="aligned", sampled=True, fused=True, **kw)
    stats = run.run_step(1)
    print(f"{w.name} [full size, {optimizer}] step 1: {stats}", flush=True)
    run.close()
    del run
    import gc

    gc.collect()
    torch_cuda.cuda.empty_cache()


# ---------------------------------------------------------------------------
# 16-bit gradient patterns and non-finite values through the SGD fold and the scaled Adam fold
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("gdt", ["f16", "bf16"])
def test_sgdm_fold_every_16_bit_pattern(torch_cuda, gdt):
    """Every finite pattern (fp16 subnormals included; bf16 within a range whose sums stay normal)
    through one SGD fold from a zero buffer: b = s * g / N up to one float32 rounding."""
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    if gdt == "f16":
        val = bits.view(np.float16).astype(np.float64)
        keep = np.isfinite(val)
    else:
        with np.errstate(invalid="ignore"):            # signalling-NaN patterns are filtered out just below
            val = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        keep = np.isfinite(val) & (np.abs(val) < 1e30) & ((np.abs(val) > 1e-30) | (val == 0))
    bits, val = bits[keep], val[keep]
    n = bits.size
    g = torch.from_numpy(bits.view(np.int16).copy()).cuda()
    b = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    N, scale = 3, 0.5
    binding.adama_sgdm_fold_multi([(None, b, g, n)], None, gdt, N, (0.0, scale))
    torch.cuda.synchronize()
    ref = np.zeros(n)
    oracle.sgdm_fold(ref, bits, N, scale, gdtype=gdt)
    got = b.cpu().numpy().astype(np.float64)
    nz = ref != 0
    assert np.all(got[~nz] == 0)
    assert np.all(np.sign(got[nz]) == np.sign(ref[nz]))
    assert np.max(np.abs(got[nz] - ref[nz]) / np.abs(ref[nz])) <= 2.0 ** -22


def test_non_finite_gradients_propagate_through_the_variants(torch_cuda):
    """inf and NaN gradients follow IEEE rules in the SGD buffer and in the scaled Adam fold; finite
    neighbours are untouched."""
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    n = 4099
    g = torch.full((n,), 0.25, dtype=torch.float32, device="cuda:0")
    g[5], g[1000], g[4098] = float("inf"), float("-inf"), float("nan")
    b = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    th = torch.ones(n, dtype=torch.float32, device="cuda:0")
    binding.adama_sgdm_fold_multi([(None, b, g, n)], None, "f32", 2)
    binding.adama_sgdm_apply_multi([(th, b, None, n)], None, 0.5)
    m = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    v = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    binding.adama_fold_opt_multi([(m, v, g, n)], None, "f32", 2, B1, B2, (0.0, 0.5))
    torch.cuda.synchronize()
    hb, ht, hm, hv = (x.cpu().numpy() for x in (b, th, m, v))
    assert hb[5] == np.inf and hb[1000] == -np.inf and np.isnan(hb[4098])
    assert ht[5] == -np.inf and ht[1000] == np.inf and np.isnan(ht[4098])
    assert hm[5] == np.inf and hm[1000] == -np.inf and np.isnan(hm[4098])
    assert hv[5] == np.inf and hv[1000] == np.inf and np.isnan(hv[4098])
    fin = np.ones(n, dtype=bool)
    fin[[5, 1000, 4098]] = False
    assert np.all(hb[fin] == 0.125) and np.all(ht[fin] == 1.0 - 0.5 * 0.125)
    assert np.allclose(hm[fin], (1 - B1) * 0.25 * 0.5 / 2, rtol=1e-6) and np.allclose(hv[fin], (1 - B2) * (0.25 * 0.5 / 2) ** 2, rtol=1e-6)


@pytest.mark.parametrize("gdt", ["f32", "bf16"])
def test_sgdm_arrays_with_different_misalignments(torch_cuda, gdt):
    """theta, b and the gradient each start a different number of elements past a 16-byte boundary, so
    no 16-byte access is possible and every element goes through the element-wise path; long enough for
    the large-launch shapes."""
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    gbytes = synth.gen.DTYPE_BYTES[gdt]
    for n in (5, 1023, 70001, (1 << 20) + 77):
        pad = 16
        th = torch.zeros(n + pad, dtype=torch.float32, device="cuda:0")
        b = torch.zeros(n + pad, dtype=torch.float32, device="cuda:0")
        g = torch.zeros((n + pad) * gbytes, dtype=torch.uint8, device="cuda:0")
        o_t, o_b, o_g = 1, 2, 3
        th0 = synth.fill_host(synth.Spec(key=synth.stream_key(67, n), sigma=0.05), "f32", n)
        th[o_t:o_t + n] = torch.from_numpy(th0).cuda()
        spec = synth.Spec(key=synth.stream_key(67, n, 1), sigma=1e-2, p_zero=0.02)
        synth.fill_device(g.data_ptr() + gbytes * o_g, spec, gdt, n, 0)
        lst = [(th.data_ptr() + 4 * o_t, b.data_ptr() + 4 * o_b, g.data_ptr() + gbytes * o_g, n)]
        N, mu, lr, wd = 2, 0.9, 0.05, 0.1
        binding.adama_sgdm_fold_first_multi(lst, None, gdt, N, mu)
        binding.adama_sgdm_fold_last_apply_multi(lst, None, gdt, N, lr, (wd, 1.0))
        torch.cuda.synchronize()
        rb, rt = np.zeros(n), th0.astype(np.float64)
        gh = synth.fill_host(spec, gdt, n)
        gd = None if gdt == "f32" else gdt
        oracle.sgdm_begin_step(rb, mu)
        oracle.sgdm_fold(rb, gh, N, 1.0, gdtype=gd)
        oracle.sgdm_fold(rb, gh, N, 1.0, gdtype=gd)
        oracle.sgdm_apply(rt, rb, lr, wd)
        name = f"sgdm misaligned {gdt} n={n}"
        check_close(name, "m", b[o_b:o_b + n].cpu().numpy(), rb)
        check_close(name, "theta", th[o_t:o_t + n].cpu().numpy(), rt, th0, th0.astype(np.float64))
        for arr, o in ((th, o_t), (b, o_b)):
            assert float(arr[:o].abs().sum()) == 0.0 and float(arr[o + n:].abs().sum()) == 0.0, name


def test_long_run_of_the_variants_stays_within_tolerance(torch_cuda):
    """300 mini-batches of AdamW with a gradient scale and of momentum SGD with weight decay: rounding
    does not build up beyond the tolerance (the decay factors are applied as float32 pairs)."""
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    n, N, steps = 4099, 2, 300
    for which in ("adamw", "sgdm"):
        th = torch.zeros(n, dtype=torch.float32, device="cuda:0")
        a = torch.zeros(n, dtype=torch.float32, device="cuda:0")      # m or the momentum buffer
        v = torch.zeros(n, dtype=torch.float32, device="cuda:0")
        g = torch.zeros(n, dtype=torch.float16, device="cuda:0")
        th0 = synth.fill_host(synth.Spec(key=synth.stream_key(89, 0), sigma=0.05), "f32", n)
        th.copy_(torch.from_numpy(th0))
        rt, ra, rv = th0.astype(np.float64), np.zeros(n), np.zeros(n)
        scale, wd, lr, mu = 1.0 / 256.0, 0.05, 1e-3, 0.99
        opt = (wd, scale)
        for t in range(1, steps + 1):
            if which == "adamw":
                oracle.begin_step(ra, rv, B1, B2)
            else:
                oracle.sgdm_begin_step(ra, mu)
            for i in range(N):
                spec = synth.Spec(key=synth.stream_key(89, t, i), sigma=3e-3 / scale, outlier_scale=2.0, p_outlier=0.001)
                synth.fill_device(g.data_ptr(), spec, "f16", n, 0)
                gh = synth.fill_host(spec, "f16", n)
                if which == "adamw":
                    if i == 0:
                        binding.adama_fold_first_opt_multi([(a, v, g, n)], None, "f16", N, B1, B2, opt)
                    else:
                        binding.adama_fold_last_apply_opt_multi([(th, a, v, g, n)], None, "f16", N, lr, EPS, B1, B2, t, opt)
                    oracle.fold_scaled(ra, rv, gh, N, B1, B2, scale, gdtype="f16")
                else:
                    if i == 0:
                        binding.adama_sgdm_fold_first_multi([(th, a, g, n)], None, "f16", N, mu, opt)
                    else:
                        binding.adama_sgdm_fold_last_apply_multi([(th, a, g, n)], None, "f16", N, lr, opt)
                    oracle.sgdm_fold(ra, gh, N, scale, gdtype="f16")
            if which == "adamw":
                oracle.apply_adamw(rt, ra, rv, lr, EPS, B1, B2, t, wd)
            else:
                oracle.sgdm_apply(rt, ra, lr, wd)
            if t % 100 == 0:
                torch.cuda.synchronize()
                name = f"long run {which} t={t}"
                stats = [check_close(name, "m", a.cpu().numpy(), ra)]
                if which == "adamw":
                    stats.append(check_close(name, "v", v.cpu().numpy(), rv))
                err = np.abs(th.cpu().numpy().astype(np.float64) - rt)
                assert np.all(err <= np.maximum(1e-5 * np.abs(rt), 1e-6)), f"{name}: theta off by {err.max():.3e}"
                print(name, stats, f"theta max abs err {err.max():.3e}", flush=True)
