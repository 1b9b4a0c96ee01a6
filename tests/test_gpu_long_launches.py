"""Launches of 2^23 and of 2^26 elements and more take their own launch policy (a bound on the workgroups a compute
unit holds, streaming stores with the scope bit, for some ops another workgroup shape).  Every step is elementwise,
so one long launch must give, bit for bit, what the same call gives when the tensor is cut into pieces short enough
for the plain policy; checked for every op, with the state and the gradient at misaligned starts (which selects the
element-aligned form of the wide accesses) and with nothing written outside the tensor."""
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

pytestmark = pytest.mark.gpu

B1, B2, LR, EPS, MU, T, N = 0.9, 0.999, 1e-3, 1e-8, 0.9, 3, 4
PIECE = 3_000_001                      # under 2^23 elements: the plain policy
GBYTES = {"f32": 4, "bf16": 2, "f16": 2}


@pytest.fixture(scope="module")
def torch_cuda():
    import torch

    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch


def _ops(binding):
    """name -> (gradient dtype or None, call(theta, m, v, g, e0, n) on element range [e0, e0 + n))."""
    def at(p, e0, size=4):
        return p + size * e0

    ops = {"decay": (None, lambda th, m, v, g, e0, n: binding.adama_begin_step(at(m, e0), at(v, e0), n, B1, B2)),
           "apply": (None, lambda th, m, v, g, e0, n: binding.adama_apply(at(th, e0), at(m, e0), at(v, e0), n, LR, EPS, B1, B2, T)),
           "rescale_apply": (None, lambda th, m, v, g, e0, n: binding.adama_rescale_apply(
               at(th, e0), at(m, e0), at(v, e0), n, 1.0 / 3, 1.0 / 9, LR, EPS, B1, B2, T))}
    for gdt in ("f32", "bf16", "f16"):
        gb = GBYTES[gdt]
        ops[f"fold_{gdt}"] = (gdt, lambda th, m, v, g, e0, n, gdt=gdt, gb=gb: binding.adama_fold(
            at(m, e0), at(v, e0), at(g, e0, gb), gdt, n, N, B1, B2))
    ops["fold_first_bf16"] = ("bf16", lambda th, m, v, g, e0, n: binding.adama_fold_first(
        at(m, e0), at(v, e0), at(g, e0, 2), "bf16", n, N, B1, B2))
    ops["fold_last_apply_f16"] = ("f16", lambda th, m, v, g, e0, n: binding.adama_fold_last_apply(
        at(th, e0), at(m, e0), at(v, e0), at(g, e0, 2), "f16", n, N, LR, EPS, B1, B2, T))
    sg = lambda th, m, g, e0, n, gb: binding.sgdm_list([(at(th, e0), at(m, e0), at(g, e0, gb), n)])   # noqa: E731
    ops["sgd_decay"] = (None, lambda th, m, v, g, e0, n: binding.adama_sgdm_begin_step_multi(sg(th, m, g, e0, n, 2), None, MU))
    ops["sgd_fold_bf16"] = ("bf16", lambda th, m, v, g, e0, n: binding.adama_sgdm_fold_multi(sg(th, m, g, e0, n, 2), None, "bf16", N))
    ops["sgd_fold_first_f32"] = ("f32", lambda th, m, v, g, e0, n: binding.adama_sgdm_fold_first_multi(
        sg(th, m, g, e0, n, 4), None, "f32", N, MU))
    ops["sgd_apply"] = (None, lambda th, m, v, g, e0, n: binding.adama_sgdm_apply_multi(sg(th, m, g, e0, n, 2), None, LR))
    ops["sgd_fold_last_apply_bf16"] = ("bf16", lambda th, m, v, g, e0, n: binding.adama_sgdm_fold_last_apply_multi(
        sg(th, m, g, e0, n, 2), None, "bf16", N, LR))
    return ops


@pytest.mark.parametrize("n,pre_state,pre_grad", [((1 << 23) + 4099, 0, 0), ((1 << 23) + 4099, 1, 1), ((1 << 23) + 4098, 3, 2),
                                                  ((1 << 23) + 517, 2, 5), ((1 << 26) + 517, 0, 0), ((1 << 26) + 4099, 3, 1)])
def test_long_launch_equals_short_launches(torch_cuda, n, pre_state, pre_grad):
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    pad = 64
    gen = torch.Generator(device="cuda:0").manual_seed(n + 17 * pre_state + pre_grad)
    theta0 = torch.empty(n + pad, dtype=torch.float32, device="cuda:0").normal_(0.0, 0.02, generator=gen)
    m0 = torch.empty(n + pad, dtype=torch.float32, device="cuda:0").normal_(0.0, 1e-3, generator=gen)
    v0 = torch.empty(n + pad, dtype=torch.float32, device="cuda:0").uniform_(1e-9, 1e-5, generator=gen)
    grads = {"f32": torch.empty(n + pad, dtype=torch.float32, device="cuda:0").normal_(0.0, 1e-2, generator=gen)}
    grads["bf16"] = grads["f32"].to(torch.bfloat16)
    grads["f16"] = grads["f32"].to(torch.float16)
    assert binding.adama_residency("fold", n) > 0 and binding.adama_tuning("fold", n)["policy_bits"] & 8
    assert binding.adama_residency("fold", PIECE) == 0 and binding.adama_tuning("fold", PIECE)["policy_bits"] & 8 == 0
    for name, (gdt, call) in _ops(binding).items():
        print(f"case {name} n={n} pre={pre_state}/{pre_grad}", flush=True)
        out = []
        for pieces in (False, True):
            th, m, v = theta0.clone(), m0.clone(), v0.clone()
            g = grads[gdt or "bf16"]
            gb = GBYTES[gdt or "bf16"]
            p = [x.data_ptr() + 4 * pre_state for x in (th, m, v)] + [g.data_ptr() + gb * pre_grad]
            if pieces:
                for e0 in range(0, n, PIECE):
                    call(*p, e0, min(PIECE, n - e0))
            else:
                call(*p, 0, n)
            torch.cuda.synchronize()
            out.append((th, m, v))
        for a, b, base, what in zip(out[0], out[1], (theta0, m0, v0), ("theta", "m", "v")):
            assert torch.equal(a, b), f"{name}: {what} of one long launch differs from short launches"
            assert torch.equal(a[:pre_state], base[:pre_state]) and torch.equal(a[pre_state + n:], base[pre_state + n:]), \
                f"{name}: {what} written outside the tensor"
        changed = [not torch.equal(a, base) for a, base in zip(out[0], (theta0, m0, v0))]
        assert any(changed), f"{name} changed nothing"


@pytest.mark.parametrize("gdt", ["f32", "bf16", "f16"])
def test_long_multi_tensor_launch_equals_single_tensor_calls(torch_cuda, gdt):
    """Seven tensors packed back to back (so most starts are misaligned), none long on its own, together past 2^23
    elements: the one multi-tensor launch runs under the long-launch policy, the per-tensor calls under the plain one."""
    torch = torch_cuda
    from paper_2305_19982_amd import binding

    sizes = [3_000_001, 17, 2_500_003, 999_999, 1_888_889, 5, 1_000_003]
    total = sum(sizes)
    assert total >= 1 << 23 and max(sizes) < 1 << 23
    gb = GBYTES[gdt]
    gen = torch.Generator(device="cuda:0").manual_seed(total)
    m0 = torch.empty(total + 8, dtype=torch.float32, device="cuda:0").normal_(0.0, 1e-3, generator=gen)
    v0 = torch.empty(total + 8, dtype=torch.float32, device="cuda:0").uniform_(1e-9, 1e-5, generator=gen)
    th0 = torch.empty(total + 8, dtype=torch.float32, device="cuda:0").normal_(0.0, 0.02, generator=gen)
    g32 = torch.empty(total + 8, dtype=torch.float32, device="cuda:0").normal_(0.0, 1e-2, generator=gen)
    g = {"f32": g32, "bf16": g32.to(torch.bfloat16), "f16": g32.to(torch.float16)}[gdt]
    out = []
    for multi in (True, False):
        th, m, v = th0.clone(), m0.clone(), v0.clone()
        fold, upd, off = [], [], 1                    # first tensor one element past an aligned address
        for n in sizes:
            fold.append((m.data_ptr() + 4 * off, v.data_ptr() + 4 * off, g.data_ptr() + gb * off, n))
            upd.append((th.data_ptr() + 4 * off, m.data_ptr() + 4 * off, v.data_ptr() + 4 * off, g.data_ptr() + gb * off, n))
            off += n
        if multi:
            binding.adama_fold_first_multi(fold, None, gdt, N, B1, B2)
            binding.adama_fold_multi(fold, None, gdt, N, B1, B2)
            binding.adama_fold_last_apply_multi(upd, None, gdt, N, LR, EPS, B1, B2, T)
        else:
            for f, u in zip(fold, upd):
                binding.adama_fold_first(f[0], f[1], f[2], gdt, f[3], N, B1, B2)
                binding.adama_fold(f[0], f[1], f[2], gdt, f[3], N, B1, B2)
                binding.adama_fold_last_apply(u[0], u[1], u[2], u[3], gdt, u[4], N, LR, EPS, B1, B2, T)
        torch.cuda.synchronize()
        out.append((th, m, v))
    for a, b, base in zip(out[0], out[1], (th0, m0, v0)):
        assert torch.equal(a, b) and not torch.equal(a, base)
        assert torch.equal(a[:1], base[:1]) and torch.equal(a[1 + total:], base[1 + total:])
