"""AdamA on a real PyTorch backward pass (paper Sec. 3.3, single-device scenario).

The paper inserts the optimizer-state accumulation and the gradient release into the backward pass
with hooks.  This module does the same on PyTorch-ROCm, with libadama doing all of the optimizer
arithmetic: a post-accumulate-grad hook on every parameter counts down its layer; when the last
gradient of a layer has been produced, ONE adama_fold_multi launch folds the whole layer's gradients
into m and v on the stream autograd is running on, and the gradients are released at once
(`p.grad = None` hands the memory back to the caching allocator, which reuses it for the next layer).
Peak gradient memory is therefore about one layer instead of the whole model.

PyTorch is the producer of gradients and the owner of memory here.  For float32 parameters theta is
the parameters' own storage.  For bfloat16 / float16 parameters (whose gradients autograd produces in
the same 16-bit format) this class keeps float32 master weights as theta, libadama updates those, and
the 16-bit parameters are refreshed from them with a plain cast right after the update (that cast is
the framework's weight refresh, not optimizer arithmetic).  m and v are always float32, allocated here.
"""
from __future__ import annotations

from typing import Iterable, Sequence

import torch

from . import binding

_GDT = {torch.float32: "f32", torch.bfloat16: "bf16", torch.float16: "f16"}


def leaf_layers(module: torch.nn.Module) -> list:
    """Default layer grouping: every module that directly owns parameters is one layer."""
    layers = []
    for sub in module.modules():
        ps = [p for p in sub.parameters(recurse=False) if p.requires_grad]
        if ps:
            layers.append(ps)
    return layers


class _HookedAccumulation:
    """Layer bookkeeping shared by the hooked optimizers: count down each layer's gradients inside the
    backward pass, fold the layer with one launch when the last one has arrived, release the gradients.

    Subclasses provide the state (`_alloc_state`) and the three kinds of launches (`_decay_all`,
    `_fold`, `_apply_all`).

    overlap=True queues every optimizer launch on a side stream (default priority) instead of the
    stream autograd runs on: a layer's fold waits for an event recorded when its gradients are complete
    and then runs next to the backward kernels of the following layers, so the memory-bound fold hides
    behind compute-bound work.  The gradients are handed to the side stream with record_stream(), which
    keeps the allocator from reusing their memory before the fold has read them; step() makes the
    autograd stream wait for the side stream, so the next forward pass sees the updated parameters."""

    def __init__(self, layers: Sequence[Iterable[torch.nn.Parameter]], N: int, fused_edges: bool,
                 weight_decay: float, grad_scale: float, overlap: bool = False):
        binding.load()
        self.overlap = bool(overlap)
        self._side = None
        self.N = int(N)
        self.fused_edges = bool(fused_edges) and self.N > 1
        self._opt = None if (weight_decay == 0.0 and grad_scale == 1.0) else binding.options(weight_decay, grad_scale)
        self.t = 0
        self.micro = 0
        self.layers = [list(ps) for ps in layers]
        self.master = {}            # float32 master weights of 16-bit parameters
        self._layer_of = {}
        self._pending = []
        self._handles = []
        self.peak_live_grad_bytes = 0
        self._live_grad_bytes = 0
        seen = set()
        for li, ps in enumerate(self.layers):
            for p in ps:
                if id(p) in seen:
                    raise ValueError("a parameter appears in two layers")
                seen.add(id(p))
                if p.dtype not in _GDT or not p.is_cuda or not p.is_contiguous():
                    raise ValueError("parameters must be contiguous float32, bfloat16 or float16 CUDA tensors")
                if p.dtype != torch.float32:
                    self.master[p] = p.detach().float()
                self._alloc_state(p)
                self._layer_of[p] = li
                self._handles.append(p.register_post_accumulate_grad_hook(self._on_grad))
            self._pending.append(len(ps))

    def _theta(self, p) -> torch.Tensor:
        """The float32 array the update writes: the parameter itself, or its master copy."""
        return self.master.get(p, p)

    def _refresh(self, ps, stream: int) -> None:
        """After an update: 16-bit parameters take the rounded value of their master weights."""
        low = [p for p in ps if p in self.master]
        if not low:
            return
        with torch.cuda.stream(torch.cuda.ExternalStream(stream) if self.overlap else torch.cuda.current_stream()):
            for p in low:
                p.data.copy_(self.master[p])

    # ---- streams ----
    def _launch_stream(self) -> int:
        """The stream optimizer launches go to, ordered after everything queued so far on the current one."""
        cur = torch.cuda.current_stream()
        if not self.overlap:
            return cur.cuda_stream
        if self._side is None:
            self._side = torch.cuda.Stream(device=cur.device)
        ev = torch.cuda.Event()
        ev.record(cur)
        self._side.wait_event(ev)
        return self._side.cuda_stream

    # ---- the mini-batch protocol ----
    def begin_mini_batch(self) -> None:
        """t <- t+1 and the moment decay (deferred into the first micro-batch's folds when fused)."""
        self.t += 1
        self.micro = 0
        if not self.fused_edges:
            self._decay_all(self._launch_stream())

    def _on_grad(self, p: torch.nn.Parameter) -> None:
        li = self._layer_of[p]
        self._live_grad_bytes += p.grad.numel() * p.grad.element_size()
        self.peak_live_grad_bytes = max(self.peak_live_grad_bytes, self._live_grad_bytes)
        self._pending[li] -= 1
        if self._pending[li] == 0:
            self._fold_layer(li)

    def _fold_layer(self, li: int) -> None:
        ps = self.layers[li]
        grads = [p.grad if p.grad.is_contiguous() else p.grad.contiguous() for p in ps]
        gdt = _GDT[grads[0].dtype]
        if any(g.dtype != grads[0].dtype for g in grads):
            raise ValueError("gradients of one layer must share a dtype")
        first = self.fused_edges and self.micro == 0
        last = self.fused_edges and self.micro == self.N - 1
        stream = self._launch_stream()
        self._fold(ps, grads, gdt, first, last, stream)
        if last:
            self._refresh(ps, stream)
        if self.overlap:
            for g in grads:                            # the side stream still reads them
                g.record_stream(self._side)
        for p in ps:                                   # release: the fold is queued, stream order does the rest
            self._live_grad_bytes -= p.grad.numel() * p.grad.element_size()
            p.grad = None
        self._pending[li] = len(ps)

    def micro_batch_done(self) -> None:
        """Call after each loss.backward()."""
        if any(k != len(ps) for k, ps in zip(self._pending, self.layers)):
            raise RuntimeError("a layer received only part of its gradients in this backward pass")
        self.micro += 1

    def step(self) -> None:
        """The parameter update (already done by the last micro-batch's folds when fused)."""
        if self.micro != self.N:
            raise RuntimeError(f"step() after {self.micro} of {self.N} micro-batches")
        if not self.fused_edges:
            stream = self._launch_stream()
            self._apply_all(stream)
            self._refresh([p for ps in self.layers for p in ps], stream)
        if self.overlap and self._side is not None:
            torch.cuda.current_stream().wait_stream(self._side)

    def remove_hooks(self) -> None:
        for h in self._handles:
            h.remove()
        self._handles = []


class AdamAccumulation(_HookedAccumulation):
    """Adam Accumulation driven by backward hooks.

    layers : groups of parameters folded by one launch each (e.g. leaf_layers(model), or one group per
             transformer block); every trainable parameter must appear in exactly one group
    N      : micro-batches per mini-batch; the loss of each micro-batch is NOT divided by N by the caller
             (the fold applies 1/N, as in Alg. 2)
    weight_decay : decoupled (AdamW); grad_scale : factor on every gradient read, 1/loss_scale when the
             caller scaled the loss up.  The defaults are the paper's plain AdamA.

    Per mini-batch:  begin_mini_batch();  N x (forward; loss.backward(); micro_batch_done());  step()
    """

    def __init__(self, layers: Sequence[Iterable[torch.nn.Parameter]], lr: float = 1e-3,
                 betas: tuple = (0.9, 0.999), eps: float = 1e-8, N: int = 1, fused_edges: bool = True,
                 weight_decay: float = 0.0, grad_scale: float = 1.0, overlap: bool = False):
        self.lr, self.beta1, self.beta2, self.eps = float(lr), float(betas[0]), float(betas[1]), float(eps)
        self.m, self.v = {}, {}
        super().__init__(layers, N, fused_edges, weight_decay, grad_scale, overlap)
        self._state_list = binding.state_list(
            [(self._theta(p).data_ptr(), self.m[p].data_ptr(), self.v[p].data_ptr(), p.numel())
             for ps in self.layers for p in ps])

    def _alloc_state(self, p) -> None:
        self.m[p] = torch.zeros_like(p, dtype=torch.float32)
        self.v[p] = torch.zeros_like(p, dtype=torch.float32)

    def _decay_all(self, stream: int) -> None:
        binding.adama_begin_step_multi(self._state_list, None, self.beta1, self.beta2, stream)

    def _fold(self, ps, grads, gdt, first: bool, last: bool, stream: int) -> None:
        if last:
            binding.adama_fold_last_apply_opt_multi(
                [(self._theta(p).data_ptr(), self.m[p].data_ptr(), self.v[p].data_ptr(), g.data_ptr(), p.numel())
                 for p, g in zip(ps, grads)], None, gdt, self.N, self.lr, self.eps, self.beta1, self.beta2, self.t,
                self._opt, stream)
            return
        entries = [(self.m[p].data_ptr(), self.v[p].data_ptr(), g.data_ptr(), p.numel()) for p, g in zip(ps, grads)]
        fn = binding.adama_fold_first_opt_multi if first else binding.adama_fold_opt_multi
        fn(entries, None, gdt, self.N, self.beta1, self.beta2, self._opt, stream)

    def _apply_all(self, stream: int) -> None:
        binding.adama_apply_opt_multi(self._state_list, None, self.lr, self.eps, self.beta1, self.beta2, self.t,
                                      self._opt, stream)


class MomentumAccumulation(_HookedAccumulation):
    """SGD with momentum accumulated the AdamA way (the paper's Discussion, Sec. 5): the momentum buffer takes
    each layer's gradient of each micro-batch as it is produced, and the gradient is released.  The
    result is the textbook step b <- mu b + mean gradient, theta <- theta - lr b (plus decoupled weight
    decay, if any) up to rounding.  Protocol and arguments as AdamAccumulation."""

    def __init__(self, layers: Sequence[Iterable[torch.nn.Parameter]], lr: float = 1e-2, momentum: float = 0.9,
                 N: int = 1, fused_edges: bool = True, weight_decay: float = 0.0, grad_scale: float = 1.0,
                 overlap: bool = False):
        self.lr, self.momentum = float(lr), float(momentum)
        self.b = {}
        super().__init__(layers, N, fused_edges, weight_decay, grad_scale, overlap)
        self._state_list = binding.sgdm_list(
            [(self._theta(p).data_ptr(), self.b[p].data_ptr(), None, p.numel()) for ps in self.layers for p in ps])

    def _alloc_state(self, p) -> None:
        self.b[p] = torch.zeros_like(p, dtype=torch.float32)

    def _decay_all(self, stream: int) -> None:
        binding.adama_sgdm_begin_step_multi(self._state_list, None, self.momentum, stream)

    def _fold(self, ps, grads, gdt, first: bool, last: bool, stream: int) -> None:
        entries = [(self._theta(p).data_ptr(), self.b[p].data_ptr(), g.data_ptr(), p.numel()) for p, g in zip(ps, grads)]
        if last:
            binding.adama_sgdm_fold_last_apply_multi(entries, None, gdt, self.N, self.lr, self._opt, stream)
        elif first:
            binding.adama_sgdm_fold_first_multi(entries, None, gdt, self.N, self.momentum, self._opt, stream)
        else:
            binding.adama_sgdm_fold_multi(entries, None, gdt, self.N, self._opt, stream)

    def _apply_all(self, stream: int) -> None:
        binding.adama_sgdm_apply_multi(self._state_list, None, self.lr, self._opt, stream)
