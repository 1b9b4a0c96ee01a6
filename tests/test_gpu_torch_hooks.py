"""AdamA attached to a real PyTorch backward pass through hooks (the paper's single-device system
design): parameters after a mini-batch match the fp64 oracle fed with the very gradients autograd
produced, and at most one layer's gradients are alive at any time."""
import copy

import numpy as np
import pytest

import oracle
from parity import check_close

pytestmark = pytest.mark.gpu


def _model(torch):
    torch.manual_seed(0)
    nn = torch.nn
    return nn.Sequential(nn.Linear(131, 517), nn.GELU(), nn.LayerNorm(517), nn.Linear(517, 389), nn.GELU(),
                         nn.Linear(389, 389), nn.LayerNorm(389), nn.Linear(389, 67)).cuda()


def _batches(torch, n_micro, steps):
    g = torch.Generator(device="cuda").manual_seed(1)
    return [[(torch.randn(32, 131, device="cuda", generator=g), torch.randn(32, 67, device="cuda", generator=g))
             for _ in range(n_micro)] for _ in range(steps)]


@pytest.mark.parametrize("fused", [False, True])
def test_hooks_match_oracle_and_release_gradients(fused):
    import torch

    from paper_2305_19982_amd.torch_hooks import AdamAccumulation, leaf_layers

    torch.backends.cuda.matmul.allow_tf32 = False
    N, steps, lr, b1, b2, eps = 4, 2, 1e-3, 0.9, 0.999, 1e-8
    ref_model = _model(torch)
    model = copy.deepcopy(ref_model)
    data = _batches(torch, N, steps)
    loss_fn = torch.nn.MSELoss()

    layers = leaf_layers(model)
    opt = AdamAccumulation(layers, lr=lr, betas=(b1, b2), eps=eps, N=N, fused_edges=fused)
    ref_params = list(ref_model.parameters())
    params = [p for ps in layers for p in ps]
    assert len(params) == len(ref_params)
    ref = oracle.OracleState([p.detach().cpu().numpy() for p in ref_params])
    prev_gpu = [p.detach().cpu().numpy().ravel().copy() for p in params]
    prev_ref = [x.copy() for x in ref.theta]
    largest_layer = max(sum(p.numel() * 4 for p in ps) for ps in layers)
    total = sum(p.numel() * 4 for p in params)
    for step in range(steps):
        # reference gradients: plain autograd on a twin model holding the same parameter values
        with torch.no_grad():
            for rp, p in zip(ref_params, params):
                rp.copy_(p)
        ref.begin_step(b1, b2)
        opt.begin_mini_batch()
        for (x, y) in data[step]:
            ref_model.zero_grad(set_to_none=True)
            loss_fn(ref_model(x), y).backward()
            for i, rp in enumerate(ref_params):
                ref.fold(i, rp.grad.detach().cpu().numpy().ravel(), N, b1, b2)
            loss_fn(model(x), y).backward()
            opt.micro_batch_done()
            assert all(p.grad is None for p in params), "gradients must be released inside the backward pass"
        opt.step()
        ref.apply(lr, eps, b1, b2)
        torch.cuda.synchronize()
        for i, p in enumerate(params):
            name = f"hooks fused={fused} step {step + 1} param {i}"
            th = p.detach().cpu().numpy().ravel()
            if step == 0:
                # same parameters => same gradients: full parity against the oracle
                check_close(name, "m", opt.m[p].cpu().numpy().ravel(), ref.m[i])
                check_close(name, "v", opt.v[p].cpu().numpy().ravel(), ref.v[i])
                check_close(name, "theta", th, ref.theta[i], prev_gpu[i], prev_ref[i])
            else:
                # the oracle's gradients came from the GPU-updated parameters, its own theta differs by rounding
                assert np.max(np.abs(th - ref.theta[i])) <= 1e-6 + 1e-5 * np.max(np.abs(ref.theta[i]))
            prev_gpu[i], prev_ref[i] = th.copy(), ref.theta[i].copy()
            ref.theta[i][:] = th            # keep the twin and the oracle on the GPU trajectory
    assert opt.peak_live_grad_bytes <= largest_layer
    assert opt.peak_live_grad_bytes < total / 2
    opt.remove_hooks()


def test_hook_path_peak_memory_below_gradient_accumulation():
    """Peak allocated memory of a backward pass: whole-model gradients (accumulation) vs one layer (AdamA)."""
    import torch

    from paper_2305_19982_amd.torch_hooks import AdamAccumulation

    def build():
        torch.manual_seed(0)
        return torch.nn.Sequential(*[torch.nn.Linear(2048, 2048) for _ in range(24)]).cuda()

    x = torch.randn(8, 2048, device="cuda")
    grad_bytes = 24 * (2048 * 2048 + 2048) * 4

    model = build()
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    base = torch.cuda.memory_allocated()
    for _ in range(2):
        model(x).sum().backward()             # plain accumulation into p.grad
    torch.cuda.synchronize()
    peak_accum = torch.cuda.max_memory_allocated() - base
    del model
    torch.cuda.empty_cache()

    model = build()
    opt = AdamAccumulation([list(l.parameters()) for l in model], N=2)
    torch.cuda.synchronize()
    torch.cuda.reset_peak_memory_stats()
    base = torch.cuda.memory_allocated()
    opt.begin_mini_batch()
    for _ in range(2):
        model(x).sum().backward()
        opt.micro_batch_done()
    opt.step()
    torch.cuda.synchronize()
    peak_adama = torch.cuda.max_memory_allocated() - base
    print(f"peak extra memory during backward: accumulation {peak_accum / 2**20:.1f} MiB, AdamA hooks "
          f"{peak_adama / 2**20:.1f} MiB (whole-model gradients {grad_bytes / 2**20:.1f} MiB)", flush=True)
    assert peak_accum >= grad_bytes
    assert peak_adama < 0.15 * grad_bytes
    opt.remove_hooks()


@pytest.mark.parametrize("fused", [False, True])
def test_hooks_adamw_with_scaled_loss_match_oracle(fused):
    """AdamW with a loss scaled by 1024 (as float16 training does): one mini-batch against the oracle's
    scaled fold and decoupled-decay update, fed with the gradients autograd produced."""
    import torch

    from paper_2305_19982_amd.torch_hooks import AdamAccumulation, leaf_layers

    torch.backends.cuda.matmul.allow_tf32 = False
    N, lr, b1, b2, eps, wd, S = 3, 1e-3, 0.9, 0.999, 1e-8, 0.1, 1024.0
    ref_model = _model(torch)
    model = copy.deepcopy(ref_model)
    data = _batches(torch, N, 1)[0]
    loss_fn = torch.nn.MSELoss()
    layers = leaf_layers(model)
    opt = AdamAccumulation(layers, lr=lr, betas=(b1, b2), eps=eps, N=N, fused_edges=fused, weight_decay=wd,
                           grad_scale=1.0 / S)
    params = [p for ps in layers for p in ps]
    ref_params = list(ref_model.parameters())
    theta = [p.detach().cpu().numpy().ravel().astype(np.float64) for p in params]
    theta0 = [x.copy() for x in theta]
    m = [np.zeros_like(x) for x in theta]
    v = [np.zeros_like(x) for x in theta]
    opt.begin_mini_batch()
    for (x, y) in data:
        ref_model.zero_grad(set_to_none=True)
        (loss_fn(ref_model(x), y) * S).backward()
        for i, rp in enumerate(ref_params):
            oracle.fold_scaled(m[i], v[i], rp.grad.detach().cpu().numpy().ravel(), N, b1, b2, 1.0 / S)
        (loss_fn(model(x), y) * S).backward()
        opt.micro_batch_done()
        assert all(p.grad is None for p in params)
    opt.step()
    torch.cuda.synchronize()
    for i, p in enumerate(params):
        oracle.apply_adamw(theta[i], m[i], v[i], lr, eps, b1, b2, 1, wd)
        name = f"adamw hooks fused={fused} param {i}"
        check_close(name, "m", opt.m[p].cpu().numpy().ravel(), m[i])
        check_close(name, "v", opt.v[p].cpu().numpy().ravel(), v[i])
        check_close(name, "theta", p.detach().cpu().numpy().ravel(), theta[i], theta0[i].astype(np.float32), theta0[i])
    opt.remove_hooks()


@pytest.mark.parametrize("fused", [False, True])
def test_hooks_momentum_sgd_match_oracle_and_library(fused):
    """Momentum SGD through the hooks: against the oracle (same micro-batch gradients) and against
    torch.optim.SGD stepping a twin model on the mean loss."""
    import torch

    from paper_2305_19982_amd.torch_hooks import MomentumAccumulation, leaf_layers

    torch.backends.cuda.matmul.allow_tf32 = False
    N, lr, mu, steps = 4, 0.05, 0.9, 2
    twin = _model(torch)
    model = copy.deepcopy(twin)
    ref_model = copy.deepcopy(twin)
    data = _batches(torch, N, steps)
    loss_fn = torch.nn.MSELoss()
    layers = leaf_layers(model)
    opt = MomentumAccumulation(layers, lr=lr, momentum=mu, N=N, fused_edges=fused)
    lib = torch.optim.SGD(twin.parameters(), lr=lr, momentum=mu)
    params = [p for ps in layers for p in ps]
    ref_params = list(ref_model.parameters())
    theta = [p.detach().cpu().numpy().ravel().astype(np.float64) for p in params]
    b = [np.zeros_like(x) for x in theta]
    for step in range(steps):
        with torch.no_grad():
            for rp, p in zip(ref_params, params):
                rp.copy_(p)
        for i, p in enumerate(params):
            theta[i][:] = p.detach().cpu().numpy().ravel()
        prev = [x.copy() for x in theta]
        opt.begin_mini_batch()
        lib.zero_grad(set_to_none=True)
        for i in range(len(b)):
            oracle.sgdm_begin_step(b[i], mu)
        for (x, y) in data[step]:
            ref_model.zero_grad(set_to_none=True)
            loss_fn(ref_model(x), y).backward()
            for i, rp in enumerate(ref_params):
                oracle.sgdm_fold(b[i], rp.grad.detach().cpu().numpy().ravel(), N)
            loss_fn(model(x), y).backward()
            opt.micro_batch_done()
            (loss_fn(twin(x), y) / N).backward()          # the library accumulates the mean gradient
            assert all(p.grad is None for p in params)
        opt.step()
        lib.step()
        torch.cuda.synchronize()
        for i, p in enumerate(params):
            oracle.sgdm_apply(theta[i], b[i], lr, 0.0)
            name = f"sgdm hooks fused={fused} step {step + 1} param {i}"
            check_close(name, "m", opt.b[p].cpu().numpy().ravel(), b[i])
            check_close(name, "theta", p.detach().cpu().numpy().ravel(), theta[i], prev[i].astype(np.float32), prev[i])
            b[i][:] = opt.b[p].cpu().numpy().ravel()      # keep the oracle on the GPU trajectory
    # the library's trajectory (float32 autograd on its own parameters) stays within float32 noise of ours
    for p, q in zip(params, twin.parameters()):
        assert float((p.detach() - q.detach()).abs().max()) <= 1e-5 * max(1.0, float(q.detach().abs().max()))
    opt.remove_hooks()


def test_transformer_demo_saves_the_gradient_memory():
    """The end-to-end demonstration at a small size: AdamA through hooks reaches the same loss as
    gradient accumulation + library Adam (AdamA's v differs from Adam's, so only closely) and its peak
    memory is lower by most of the whole-model gradient size."""
    import argparse

    import bench_hooks as hook_demo

    args = argparse.Namespace(layers=4, hidden=512, heads=8, vocab=4000, seq=256, micro_batch=2, N=4, steps=2)
    out = hook_demo.compare(args)
    grad_bytes = out["model"]["params"] * 4
    a, b = out["gradient_accumulation_adam"], out["adama_hooks"]
    assert abs(a["final_loss"] - b["final_loss"]) < 0.05 * a["final_loss"]
    assert out["peak_memory_saved_bytes"] > 0.6 * grad_bytes
    assert b["peak_live_grad_bytes"] < 0.5 * grad_bytes
    print(out, flush=True)


def test_side_stream_folds_give_the_same_bits():
    """overlap=True moves every optimizer launch to a side stream ordered by events; the arithmetic and
    its order per element are unchanged, so parameters and moments are bit-identical."""
    import torch

    from paper_2305_19982_amd.torch_hooks import AdamAccumulation, MomentumAccumulation, leaf_layers

    torch.backends.cuda.matmul.allow_tf32 = False
    N, steps = 3, 3
    data = _batches(torch, N, steps)
    loss_fn = torch.nn.MSELoss()
    for cls, kw, state in ((AdamAccumulation, dict(lr=1e-3, weight_decay=0.01), ("m", "v")),
                           (MomentumAccumulation, dict(lr=0.05, momentum=0.9), ("b",))):
        for fused in (False, True):
            results = []
            for overlap in (False, True):
                model = _model(torch)
                opt = cls(leaf_layers(model), N=N, fused_edges=fused, overlap=overlap, **kw)
                for step in range(steps):
                    opt.begin_mini_batch()
                    for (x, y) in data[step]:
                        loss_fn(model(x), y).backward()
                        opt.micro_batch_done()
                    opt.step()
                torch.cuda.synchronize()
                params = [p.detach().clone() for p in model.parameters()]
                moments = [getattr(opt, k)[p].clone() for k in state for p in model.parameters()]
                results.append(params + moments)
                opt.remove_hooks()
            for a, b in zip(*results):
                assert torch.equal(a, b), f"{cls.__name__} fused={fused}: side-stream result differs"


@pytest.mark.parametrize("fused", [False, True])
def test_hooks_with_bfloat16_parameters_and_float32_master_weights(fused):
    """A bfloat16 model: autograd produces bfloat16 gradients, the optimizer keeps float32 master
    weights, m and v; after the mini-batch the master weights match the oracle fed with the very
    gradient bits, and every parameter is the rounded value of its master weight."""
    import torch

    from paper_2305_19982_amd.torch_hooks import AdamAccumulation, leaf_layers

    N, lr, b1, b2, eps = 3, 1e-3, 0.9, 0.999, 1e-8
    ref_model = _model(torch).bfloat16()
    model = copy.deepcopy(ref_model)
    data = [(x.bfloat16(), y.bfloat16()) for (x, y) in _batches(torch, N, 1)[0]]
    loss_fn = torch.nn.MSELoss()
    layers = leaf_layers(model)
    opt = AdamAccumulation(layers, lr=lr, betas=(b1, b2), eps=eps, N=N, fused_edges=fused)
    params = [p for ps in layers for p in ps]
    ref_params = list(ref_model.parameters())
    assert all(p in opt.master and opt.master[p].dtype == torch.float32 for p in params)
    ref = oracle.OracleState([p.detach().float().cpu().numpy() for p in params])
    theta0 = [x.copy() for x in ref.theta]
    ref.begin_step(b1, b2)
    opt.begin_mini_batch()
    for (x, y) in data:
        ref_model.zero_grad(set_to_none=True)
        loss_fn(ref_model(x), y).backward()
        for i, rp in enumerate(ref_params):
            assert rp.grad.dtype == torch.bfloat16
            bits = rp.grad.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16).ravel()
            ref.fold(i, bits, N, b1, b2, gdtype="bf16")
        loss_fn(model(x), y).backward()
        opt.micro_batch_done()
        assert all(p.grad is None for p in params)
    opt.step()
    ref.apply(lr, eps, b1, b2)
    torch.cuda.synchronize()
    for i, p in enumerate(params):
        name = f"bf16 hooks fused={fused} param {i}"
        check_close(name, "m", opt.m[p].cpu().numpy().ravel(), ref.m[i])
        check_close(name, "v", opt.v[p].cpu().numpy().ravel(), ref.v[i])
        master = opt.master[p]
        check_close(name, "theta", master.cpu().numpy().ravel(), ref.theta[i], theta0[i].astype(np.float32), theta0[i])
        assert torch.equal(p.detach(), master.bfloat16()), f"{name}: parameter is not the rounded master weight"
    opt.remove_hooks()
