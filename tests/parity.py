"""Shared machinery of the GPU parity tests: run a synthetic workload through libadama (via the
simulated-backward harness) and through the fp64 oracle on the same seeded inputs, and compare.

Tolerance (stated by the benchmark spec: max elementwise relative error 1e-5 with a 1e-6 absolute floor on
theta, m and v for fp32 state), read as
    |gpu - ref| <= max(1e-5 * |ref|, 1e-6)                                   (binding criterion)
and, because m and v are far below 1e-6-relevant magnitudes at the configured gradient scales, the
scale-aware criteria derived from the arithmetic are gated as well:
    v      : |gpu - ref| <= 1e-5 * ref wherever ref > 0, and gpu == 0 exactly where ref == 0
             (all terms are non-negative: error <= (N+2) * 2^-24 per mini-batch)
    m      : |gpu - ref| <= 1e-5 * max(|ref|, rms(ref)) with the rms over the compared elements of the
             tensor (m is a signed sum: cancellation can leave |m| far below the terms that formed it,
             so the tensor's own scale replaces the fixed 1e-6 floor)
    dtheta : the same bound on the parameter change of the step, plus the half ulp (2^-24 |theta|) that
             storing theta in fp32 costs whatever the arithmetic
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

import oracle
import synth
from synth import configs

RTOL, ATOL = 1e-5, 1e-6
# Sampling of full-size workloads: every tensor of at most FULL_BELOW elements is compared in full; a
# longer one on its first and last SLICE elements plus BLOCKS random SLICE-element blocks.
FULL_BELOW = 1 << 20
SLICE = 65536
BLOCKS = 16


def host_threads() -> int:
    """Threads for the oracle side of a sampled full-size run: the GPU machine grants 16 cores per GPU."""
    return max(1, min(16, len(os.sched_getaffinity(0))))


def check_close(name: str, kind: str, gpu: np.ndarray, ref: np.ndarray, prev_gpu=None, prev_ref=None) -> dict:
    gpu64 = gpu.astype(np.float64)
    err = np.abs(gpu64 - ref)
    assert np.all(np.isfinite(gpu64)), f"{name} {kind}: non-finite GPU values"
    bound = np.maximum(RTOL * np.abs(ref), ATOL)
    worst = int(np.argmax(err - bound))
    assert np.all(err <= bound), (f"{name} {kind}: |gpu-ref| = {err[worst]:.3e} at {worst} "
                                  f"(gpu {gpu64[worst]!r}, ref {ref[worst]!r})")
    stats = {"max_abs": float(err.max(initial=0.0))}
    if kind == "v":
        pos = ref > 0
        assert np.all(gpu64[~pos] == 0.0), f"{name} v: must be exactly 0 where the oracle's is"
        assert np.all(gpu64 >= 0.0), f"{name} v: negative"
        if pos.any():
            rel = err[pos] / ref[pos]
            assert rel.max() <= RTOL, f"{name} v: relative error {rel.max():.3e}"
            stats["max_rel"] = float(rel.max())
    elif kind == "m":
        rms = float(np.sqrt(np.mean(ref ** 2))) if ref.size else 0.0
        if rms > 0:
            ratio = err / (RTOL * np.maximum(np.abs(ref), rms))
            assert ratio.max() <= 1.0, f"{name} m: err/(1e-5*max(|ref|, rms)) = {ratio.max():.3f} (rms {rms:.3e})"
            stats["max_over_scale"] = float(ratio.max() * RTOL)
    elif kind == "theta" and prev_gpu is not None:
        d_gpu = gpu64 - prev_gpu.astype(np.float64)
        d_ref = ref - prev_ref
        rms = float(np.sqrt(np.mean(d_ref ** 2))) if d_ref.size else 0.0
        if rms > 0:
            # fp32 storage of theta cannot hold the new value closer than half an ulp: 2^-24 |theta|
            ratio = np.abs(d_gpu - d_ref) / (RTOL * np.maximum(np.abs(d_ref), rms) + 2.0 ** -24 * np.abs(ref))
            assert ratio.max() <= 1.0, f"{name} dtheta: err/(1e-5*max(|ref|, rms)+ulp/2) = {ratio.max():.3f} (rms {rms:.3e})"
            stats["dtheta_over_scale"] = float(ratio.max() * RTOL)
    return stats


def slices_of(n: int, rng: np.random.Generator, full_below: int = FULL_BELOW, blocks: int = BLOCKS) -> list:
    """Element ranges compared for a tensor of n elements: everything if it has at most `full_below`
    elements (or if the sample would cover most of it anyway), else the first and last SLICE elements
    plus `blocks` random SLICE-element blocks (starts deliberately not aligned; blocks may overlap)."""
    if n <= full_below or n <= 2 * (blocks + 2) * SLICE:
        return [(0, n)]
    out = [(0, SLICE), (n - SLICE, n)]
    for _ in range(blocks):
        s = int(rng.integers(SLICE, n - 2 * SLICE))
        out.append((s, s + SLICE))
    return sorted(out)


class WorkloadRun:
    """One workload on the GPU (harness) and in the oracle (on all elements or on sampled slices)."""

    def __init__(self, w: configs.Workload, pack: str = "aligned", sampled: bool = False, device: str = "cuda:0",
                 fused: bool = False, optimizer: str = "adam", momentum: float = 0.9, weight_decay: float = 0.0,
                 grad_scale: float = 1.0, shadow: bool = False, fold_streams: int = 1):
        from paper_2305_19982_amd.harness import SimulatedBackward

        self.w = w
        self.sampled = sampled
        self.fused = fused      # decay inside micro-batch 0's folds, update inside micro-batch N-1's
        # variants: "sgdm" keeps its momentum buffer where Adam keeps m (no v); weight decay and the
        # gradient scale go through the *_opt entry points and the oracle's variant functions
        self.optimizer, self.momentum, self.weight_decay, self.grad_scale = optimizer, momentum, weight_decay, grad_scale
        self.hb = SimulatedBackward([t.n for t in w.tensors], w.layers, w.gdtype, device=device, pack=pack,
                                    optimizer=optimizer, momentum=momentum, weight_decay=weight_decay,
                                    grad_scale=grad_scale, fold_streams=fold_streams)
        rng = np.random.default_rng(1234)
        self.slices = [slices_of(t.n, rng) if sampled else [(0, t.n)] for t in w.tensors]
        # The oracle is called as it stands; a sampled full-size run merely calls it from several host
        # threads at once, each on its own compared range (ranges are independent: the method is elementwise).
        self.pool = ThreadPoolExecutor(max_workers=host_threads()) if sampled else None
        # theta0: the device writes it, the host regenerates the same bits for the oracle
        for t in w.tensors:
            synth.fill_device(self.hb.theta_ptr(t.index), w.theta_spec(t.index), "f32", t.n, self.hb.stream_handle)
        self.key = [(t.index, a, b) for t in w.tensors for (a, b) in self.slices[t.index]]
        theta0 = self._map(lambda k: synth.fill_host(w.theta_spec(k[0]), "f32", k[2] - k[1], first=k[1]), self.key)
        self.ref = oracle.OracleState(theta0)
        # Shadow state: a second set of theta, m, v arenas driven through a different launch geometry
        # (every fold as a single-tensor launch, decay and update as ONE flat launch over the whole
        # arena, padding included).  The two must end bit-identical over every element of the arenas,
        # which proves on the full-size workload that no chunk of any list launch was skipped,
        # repeated or misplaced.  (Adam, separate calls only.)
        self.shadow = None
        if shadow:
            assert optimizer == "adam" and not fused and weight_decay == 0.0 and grad_scale == 1.0 and fold_streams == 1
            import torch

            with torch.cuda.stream(self.hb.stream):
                self.shadow = {"theta": self.hb.theta.clone(), "m": torch.zeros_like(self.hb.m),
                               "v": torch.zeros_like(self.hb.v)}
        self.rows = {}
        for r, (ti, a, b) in enumerate(self.key):
            self.rows.setdefault(ti, []).append((r, a, b))
        self.prev_gpu_theta = [self.download("theta", r) for r in range(len(self.key))]
        for r in range(len(self.key)):
            assert np.array_equal(self.prev_gpu_theta[r].astype(np.float64), self.ref.theta[r]), \
                "device and host generators disagree on theta0"

    def close(self) -> None:
        if self.pool is not None:
            self.pool.shutdown()
            self.pool = None

    def _map(self, fn, items) -> list:
        if self.pool is None:
            return [fn(x) for x in items]
        return list(self.pool.map(fn, items))

    def download(self, which: str, r: int) -> np.ndarray:
        ti, a, b = self.key[r]
        self.hb.synchronize()
        return self.hb.tensor_view(which, ti)[a:b].cpu().numpy()

    def produce(self, step: int, micro: int, li: int) -> None:
        w = self.w
        for ti in w.layers[li]:
            synth.fill_device(self.hb.grad_ptr(ti), w.grad_spec(step, micro, ti), w.gdtype, w.tensors[ti].n,
                              self.hb.layer_stream_handle(li))

    def oracle_fold_layer(self, step: int, micro: int, li: int) -> None:
        w = self.w
        gd = None if w.gdtype == "f32" else w.gdtype

        def one(job) -> None:
            ti, r, a, b = job
            g = synth.fill_host(w.grad_spec(step, micro, ti), w.gdtype, b - a, first=a)
            if self.optimizer == "sgdm":
                oracle.sgdm_fold(self.ref.m[r], g, w.N, self.grad_scale, gdtype=gd)
            elif self.grad_scale != 1.0:
                oracle.fold_scaled(self.ref.m[r], self.ref.v[r], g, w.N, w.beta1, w.beta2, self.grad_scale, gdtype=gd)
            else:
                self.ref.fold(r, g, w.N, w.beta1, w.beta2, gdtype=gd)

        self._map(one, [(ti, r, a, b) for ti in w.layers[li] for (r, a, b) in self.rows[ti]])

    # ---- the shadow geometry (see __init__) ----
    def shadow_fold_layer(self, li: int) -> None:
        from paper_2305_19982_amd import binding

        w, hb, sh = self.w, self.hb, self.shadow
        for ti in w.layers[li]:
            o, n = 4 * hb.offset[ti], w.tensors[ti].n
            binding.adama_fold(sh["m"].data_ptr() + o, sh["v"].data_ptr() + o, hb.grad_ptr(ti), w.gdtype, n, w.N,
                               w.beta1, w.beta2, hb.stream_handle)

    def assert_shadow_identical(self) -> int:
        """Bitwise equality of the whole arenas (padding included); returns the number of elements compared."""
        import torch

        self.hb.synchronize()
        for which in ("theta", "m", "v"):
            a, b = getattr(self.hb, which), self.shadow[which]
            assert torch.equal(a.view(torch.int32), b.view(torch.int32)), \
                f"{self.w.name}: {which} differs between the list launches and the flat / single-tensor launches"
        return 3 * self.hb.arena_elems

    def run_step(self, step: int, check_grad_bits: bool = False) -> dict:
        w = self.w
        fused = self.fused and w.N > 1
        if fused:
            self.hb.begin_step_fused()
        else:
            self.hb.begin_step(w.beta1, w.beta2)
        if self.shadow is not None:
            from paper_2305_19982_amd import binding

            binding.adama_begin_step(self.shadow["m"], self.shadow["v"], self.hb.arena_elems, w.beta1, w.beta2,
                                     self.hb.stream_handle)
        self.oracle_begin_step()
        for i in range(w.N):
            for li in w.backward_layers():
                self.produce(step, i, li)
                if check_grad_bits:
                    self.assert_grad_bits(step, i, li)
                if self.fused and i == w.N - 1:
                    self.hb.fold_layer_last_apply(li, w.N, w.lr, w.eps, w.beta1, w.beta2)
                elif fused and i == 0:
                    self.hb.fold_layer_first(li, w.N, w.beta1, w.beta2)
                else:
                    self.hb.fold_layer(li, w.N, w.beta1, w.beta2)
                if self.shadow is not None:
                    self.shadow_fold_layer(li)
                self.oracle_fold_layer(step, i, li)
        if not self.fused:
            self.hb.apply(w.lr, w.eps, w.beta1, w.beta2)
        if self.shadow is not None:
            binding.adama_apply(self.shadow["theta"], self.shadow["m"], self.shadow["v"], self.hb.arena_elems, w.lr,
                                w.eps, w.beta1, w.beta2, self.hb.t, self.hb.stream_handle)
        self.oracle_apply()
        assert self.hb.t == self.ref.t == step
        return self.compare()

    def oracle_begin_step(self) -> None:
        w = self.w
        self.ref.t += 1
        if self.optimizer == "sgdm":
            self._map(lambda b: oracle.sgdm_begin_step(b, self.momentum), self.ref.m)
        else:
            self._map(lambda mv: oracle.begin_step(mv[0], mv[1], w.beta1, w.beta2), list(zip(self.ref.m, self.ref.v)))

    def oracle_apply(self) -> None:
        w = self.w

        def one(tmv) -> None:
            th, m, v = tmv
            if self.optimizer == "sgdm":
                oracle.sgdm_apply(th, m, w.lr, self.weight_decay)
            elif self.weight_decay != 0.0:
                oracle.apply_adamw(th, m, v, w.lr, w.eps, w.beta1, w.beta2, self.ref.t, self.weight_decay)
            else:
                oracle.apply(th, m, v, w.lr, w.eps, w.beta1, w.beta2, self.ref.t)

        self._map(one, list(zip(self.ref.theta, self.ref.m, self.ref.v)))

    def assert_grad_bits(self, step: int, micro: int, li: int) -> None:
        """What the device wrote into the gradient buffer is what the host regenerates for the oracle."""
        import torch

        w = self.w
        self.hb.synchronize()
        for ti in w.layers[li]:
            n = w.tensors[ti].n
            off = self.hb.grad_offset[ti] * self.hb.gbytes
            raw = self.hb.grad_buffer[off: off + n * self.hb.gbytes].cpu().numpy()
            dev = raw.view(np.float32 if w.gdtype == "f32" else np.uint16)
            host = synth.fill_host(w.grad_spec(step, micro, ti), w.gdtype, n)
            assert np.array_equal(dev, host), f"gradient bits differ for tensor {ti}"
        del torch

    def compare(self) -> dict:
        worst = {}
        for r, (ti, a, b) in enumerate(self.key):
            name = f"{self.w.name}:{self.w.tensors[ti].name}[{a}:{b}]"
            th = self.download("theta", r)
            moments = [("m", self.download("m", r), self.ref.m[r])]
            if self.optimizer != "sgdm":
                moments.append(("v", self.download("v", r), self.ref.v[r]))
            for kind, gpu, ref in moments:
                for k, val in check_close(name, kind, gpu, ref).items():
                    worst[f"{kind}.{k}"] = max(worst.get(f"{kind}.{k}", 0.0), val)
            prev_ref = getattr(self, "_prev_ref_theta", None)
            st = check_close(name, "theta", th, self.ref.theta[r], self.prev_gpu_theta[r],
                             prev_ref[r] if prev_ref is not None else self.prev_gpu_theta[r].astype(np.float64))
            for k, val in st.items():
                worst[f"theta.{k}"] = max(worst.get(f"theta.{k}", 0.0), val)
            self.prev_gpu_theta[r] = th
        self._prev_ref_theta = [x.copy() for x in self.ref.theta]
        return worst
