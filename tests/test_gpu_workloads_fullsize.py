"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times (one
adama_fold_multi launch per layer, backward order, every micro-batch), on sampled element ranges the
oracle can afford: every tensor of at most 2^20 elements in full; for longer tensors the first and
last 65536 elements plus sixteen random 65536-element blocks (about 230 M compared elements of the
GPT-2-shaped workload, 290 M of the 12.75 B-parameter one).  The host regenerates exactly the bits the
device generator wrote (checked bit for bit in test_gpu_parity.py), so no data flows from the GPU path
into the oracle; the oracle is called from 16 host threads, each on its own compared range.

Two whole-arena checks cover what sampling cannot:
* every second moment of every tensor is positive after the run (a gradient element is never exactly 0
  in all micro-batches here) and every padding element between tensors is still 0: no chunk skipped,
  nothing written outside a tensor;
* where HBM allows (all but the 12.75 B-parameter workload), a shadow copy of the state goes through a
  different launch geometry (single-tensor folds, flat whole-arena decay and update) and must end
  bit-identical over all of theta, m and v."""
import gc
import time

import pytest

from parity import WorkloadRun
from synth import configs

pytestmark = pytest.mark.gpu


def _count_positive(x, piece=1 << 28) -> int:
    return sum(int((x[a:a + piece] > 0).sum()) for a in range(0, x.numel(), piece))


def _run_full(name, shadow=True):
    import torch

    w = configs.FULL[name]()
    t0 = time.time()
    print(f"{w.name}: P={w.P} tensors={len(w.tensors)} layers={len(w.layers)} N={w.N} steps={w.steps}", flush=True)
    run = WorkloadRun(w, pack="aligned", sampled=True, shadow=shadow)
    sampled = sum(b - a for (_, a, b) in run.key)
    print(f"  state resident, {len(run.key)} compared ranges, {sampled} elements = {100.0 * sampled / w.P:.2f} % "
          f"({time.time() - t0:.1f} s)", flush=True)
    for step in range(1, w.steps + 1):
        stats = run.run_step(step)
        print(f"  step {step} ok after {time.time() - t0:.1f} s: {stats}", flush=True)
    # whole-arena coverage: v > 0 on every element of every tensor, 0 on the padding between tensors
    run.hb.synchronize()
    positive = _count_positive(run.hb.v)
    zero_prob = w.p_zero ** (w.N * w.steps)          # an element whose every gradient was exactly 0
    assert positive <= w.P, f"{positive} positive second moments but only {w.P} parameters: a write outside a tensor"
    assert positive >= w.P * (1.0 - zero_prob) - 64, f"only {positive} of {w.P} second moments are positive: a chunk was skipped"
    print(f"  coverage: {positive} of {w.P} second moments positive, {run.hb.arena_elems - w.P} padding elements still 0",
          flush=True)
    if shadow:
        n = run.assert_shadow_identical()
        print(f"  shadow geometry (single-tensor folds, flat decay / update): {n} state elements bit-identical "
              f"({time.time() - t0:.1f} s)", flush=True)
    peak, whole = run.hb.peak_grad_bytes, run.hb.whole_model_grad_bytes
    print(f"  peak gradient memory {peak} B (largest layer) vs {whole} B for whole-model gradients: 1/{whole / peak:.1f}",
          flush=True)
    assert peak < (w.largest_layer_elems + 128 * 32) * w.grad_bytes
    if len(w.layers) > 2:
        assert peak < whole
    run.close()
    del run
    gc.collect()
    torch.cuda.empty_cache()
    return peak, whole


def test_c2_bert_large_full_size():
    _run_full("c2")


def test_c3_gpt2_xl_full_size():
    peak, whole = _run_full("c3")
    assert peak < whole / 15          # the embedding layer (160.8 MB of bf16) vs 3.1 GB


def test_c4_ragged_small_full_size():
    _run_full("c4")


def test_c5_decoder_10b_full_size():
    import torch

    free, total = torch.cuda.mem_get_info()
    if free < 170 * (1 << 30):
        pytest.skip(f"needs ~155 GB of free HBM, {free >> 30} GB available")
    peak, whole = _run_full("c5", shadow=False)      # a second copy of 153 GB of state does not fit
    assert peak < whole / 40          # one block (629 MB) vs 25.5 GB


def test_single_tensor_longer_than_2_32_elements():
    """One tensor of 2^32 + 4099 elements (60 GB of theta, m, v and bf16 gradients) through the fused
    sequence fold_first, fold, fold_last_apply: element indices and byte offsets beyond 32 bits.
    Compared with the oracle on slices at the start, across the 2^32 boundary, at random places and
    at the ragged end."""
    import numpy as np
    import torch

    import oracle
    import synth
    from parity import check_close
    from paper_2305_19982_amd import binding

    n = (1 << 32) + 4099
    free, _ = torch.cuda.mem_get_info()
    if free < 70 * (1 << 30):
        pytest.skip(f"needs ~61 GB of free HBM, {free >> 30} GB available")
    t0 = time.time()
    theta = torch.empty(n, dtype=torch.float32, device="cuda:0")
    m = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    v = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    g = torch.empty(n, dtype=torch.bfloat16, device="cuda:0")
    th_spec = synth.Spec(key=synth.stream_key(71, 0), sigma=0.02)
    synth.fill_device(theta.data_ptr(), th_spec, "f32", n, 0)
    rng = np.random.default_rng(5)
    starts = [0, (1 << 32) - 2048, n - 4099] + [int(x) for x in rng.integers(4096, n - 8192, 5)]
    slices = [(a, min(a + 4099, n)) for a in starts]
    ref = oracle.OracleState([synth.fill_host(th_spec, "f32", b - a, first=a) for a, b in slices])
    th0 = [x.copy() for x in ref.theta]
    N, b1, b2, lr, eps = 3, 0.9, 0.999, 1e-3, 1e-8
    ref.begin_step(b1, b2)
    for i in range(N):
        spec = synth.Spec(key=synth.stream_key(71, 1 + i), sigma=1e-2, p_zero=0.01, p_outlier=0.001)
        synth.fill_device(g.data_ptr(), spec, "bf16", n, 0)
        if i == 0:
            binding.adama_fold_first(m, v, g, "bf16", n, N, b1, b2)
        elif i == N - 1:
            binding.adama_fold_last_apply(theta, m, v, g, "bf16", n, N, lr, eps, b1, b2, 1)
        else:
            binding.adama_fold(m, v, g, "bf16", n, N, b1, b2)
        for r, (a, b) in enumerate(slices):
            ref.fold(r, synth.fill_host(spec, "bf16", b - a, first=a), N, b1, b2, gdtype="bf16")
    ref.apply(lr, eps, b1, b2)
    torch.cuda.synchronize()
    print(f"  2^32+4099 elements: three passes queued and finished after {time.time() - t0:.1f} s", flush=True)
    for r, (a, b) in enumerate(slices):
        name = f"long tensor [{a}:{b}]"
        check_close(name, "m", m[a:b].cpu().numpy(), ref.m[r])
        check_close(name, "v", v[a:b].cpu().numpy(), ref.v[r])
        check_close(name, "theta", theta[a:b].cpu().numpy(), ref.theta[r], th0[r].astype(np.float32), th0[r])
    # every element was reached: v is positive wherever a gradient was non-zero, which is ~99 % of all
    # elements; count in pieces to keep temporaries small
    touched = 0
    for a in range(0, n, 1 << 28):
        touched += int((v[a:a + (1 << 28)] > 0).sum())
    assert touched > 0.95 * n, f"only {touched} of {n} second moments are non-zero"
    del theta, m, v, g
    gc.collect()
    torch.cuda.empty_cache()
