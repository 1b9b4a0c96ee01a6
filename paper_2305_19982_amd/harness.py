"""Simulated backward pass driving libadama the way Alg. 2 of the paper prescribes.

The harness owns theta, m, v for a list of parameter tensors grouped in layers,
and ONE gradient buffer sized for the largest layer.  For each micro-batch it
walks the layers in backward order; a caller-supplied producer writes that
layer's raw gradients into the buffer ("assign memory for g"), one
adama_fold_multi launch folds the whole layer into m and v, and the buffer is
free for the next layer as soon as the launch is queued ("release memory for
g"): stream order is the only synchronisation.  Peak gradient memory is
therefore the largest layer, not the whole model (Sec. 3.1, last paragraph).

PyTorch is used for device allocations and stream handles only.  All optimizer
arithmetic happens inside libadama's kernels.
"""
from __future__ import annotations

from typing import Callable, Sequence

import torch

from . import binding

_GRAD_BYTES = {"f32": 4, "bf16": 2, "f16": 2}


def _round_up(x: int, a: int) -> int:
    return (x + a - 1) // a * a


class SimulatedBackward:
    """theta/m/v state plus a single reusable per-layer gradient buffer.

    tensor_sizes : number of elements of every parameter tensor
    layers       : lists of tensor indices, forward order (backward visits them reversed)
    gdtype       : "f32" | "bf16" | "f16" gradient storage
    pack         : "aligned"  -> every tensor starts on a 256-byte boundary (separate-allocation like)
                   "tight"    -> tensors back to back, so starts are generally not 16-byte aligned
    grad_buffer  : "layer"    -> the AdamA layout: one buffer of the largest layer's size, reused
                   "model"    -> every layer has its own region (what gradient accumulation must keep);
                                 only for measurements that want all gradient inputs resident and
                                 distinct in HBM before the clock starts
    optimizer    : "adam"     -> AdamA as in the paper (moments m, v)
                   "sgdm"     -> SGD with momentum accumulated the same way (one moment, kept in the m
                                 arena; no v arena is allocated).  The beta1/beta2/eps arguments of the
                                 step methods are then ignored and `momentum` is used for the decay.
    weight_decay, grad_scale : decoupled weight decay of the update and the factor applied to every
                   gradient read (1/loss_scale); the defaults select the plain calls.
    arena_layout : "slab" (default): theta, m, v in one allocation, arena k starting k * pitch bytes after the
                   first, the pitch a multiple of 2 MiB; "separate": one allocation per arena, wherever the
                   allocator puts them.
    Placement.     What the memory system delivers for arrays that are streamed in lock step depends on which
                   channels and banks their addresses hash to, i.e. on the distance between the arenas and on
                   the physical pages the driver handed out: on MI355X the same mini-batch runs 2..6 % faster
                   or slower from one placement to the next (the fold of GPT-2-XL blocks: 6.37..6.61 TB/s over
                   pitches of one slab that differ by 2 MiB) and stays so for as long as the placement lives.
                   No rule for the distance held up across allocations, so the harness measures:
    pitch_tries  : how many pitches to try inside a slab (default 1: the smallest that fits; then 2 MiB more, then
                   pairs of consecutive distances next to the following multiples of 256 MiB, where the effect
                   of the distance is largest), or the list of extras to try, in 2 MiB units (e.g. [0, 1, 64,
                   65]).  Costs no extra memory beyond the largest extra (under 1 GB for 8 tries), so it works
                   for a state that fills the device.
    placement_tries : how many allocations to try (default 1).  All of them stay allocated until the search ends
                   (a freed one would be handed out again), so k tries need room for k copies of the state;
                   the search stops early when the next copy does not fit.  Every candidate (allocation x pitch)
                   is timed on decay + N fold sweeps + update with scratch contents like a workload's; the
                   fastest is kept and handed over zeroed.
                   `placement` records every candidate's estimated step time and which one was chosen.
    placement_micro_batches : the N the candidates are scored for (weight of the fold sweep in the score).
    arena_pitch_extra, arena_stagger_bytes : measurement knobs for a slab: 2 MiB units added to the first
                   pitch tried, and extra bytes (a multiple of 256) between consecutive arenas.
    fold_streams : number of HIP streams (default priority) the folds are spread over: layer l is produced
                   and folded on stream l mod fold_streams, so that the end of one layer's fold overlaps the
                   start of the next one's.  Folds of one layer stay on one stream, hence in order across
                   micro-batches; the decay precedes and the update follows all of them through events.  Each
                   stream owns a gradient buffer of the largest layer's size (stream order is then still the
                   only synchronisation a buffer needs), so peak gradient memory is fold_streams layers
                   instead of one.  Measured: no robust gain (BERT-Large-shaped +0.2..0.8 %, 2000 small tensors
                   -5 %, GPT-2-shaped -2 %: concurrent kernels interleave their address streams); off by default.
    """

    def __init__(self, tensor_sizes: Sequence[int], layers: Sequence[Sequence[int]], gdtype: str,
                 device: str = "cuda:0", stream: torch.cuda.Stream | None = None, pack: str = "aligned",
                 grad_buffer: str = "layer", optimizer: str = "adam", momentum: float = 0.9,
                 weight_decay: float = 0.0, grad_scale: float = 1.0, arena_layout: str = "slab",
                 arena_stagger_bytes: int = 0, arena_pitch_extra: int = 0, fold_streams: int = 1,
                 placement_tries: int = 1, pitch_tries: int = 1, placement_micro_batches: int = 8):
        if gdtype not in _GRAD_BYTES:
            raise ValueError(gdtype)
        if optimizer not in ("adam", "sgdm"):
            raise ValueError(optimizer)
        binding.load()
        self.optimizer = optimizer
        self.momentum = float(momentum)
        self._opt = None if (weight_decay == 0.0 and grad_scale == 1.0) else binding.options(weight_decay, grad_scale)
        self.device = torch.device(device)
        self.stream = stream if stream is not None else torch.cuda.Stream(device=self.device)
        if fold_streams < 1:
            raise ValueError("fold_streams must be >= 1")
        self.fold_streams = [self.stream] + [torch.cuda.Stream(device=self.device) for _ in range(fold_streams - 1)]
        self._grad_buffer_mode = grad_buffer
        self.gdtype = gdtype
        self.gbytes = _GRAD_BYTES[gdtype]
        self.sizes = [int(n) for n in tensor_sizes]
        self.layers = [list(l) for l in layers]
        self.t = 0
        align_elems = 64 if pack == "aligned" else 1          # 64 fp32 = 256 B
        # ---- persistent state: three flat fp32 arenas with identical tensor offsets ----
        self.offset = []
        off = 0
        for n in self.sizes:
            self.offset.append(off)
            off = _round_up(off + n, align_elems)
        self.arena_elems = max(off, 1)
        # ---- the one gradient buffer: layer-local offsets, reused by every layer ----
        self.grad_offset = [0] * len(self.sizes)             # element offset inside the buffer
        galign = align_elems * 4 // self.gbytes if pack == "aligned" else 1
        largest = 0
        if grad_buffer == "layer":
            for idx in self.layers:
                o = 0
                for ti in idx:
                    o = _round_up(o + self.sizes[ti], galign)
                largest = max(largest, o)
            largest = _round_up(largest, 64)                 # one such region per fold stream
        o = 0
        for li, idx in enumerate(self.layers):
            if grad_buffer == "layer":
                o = (li % fold_streams) * largest
            for ti in idx:
                self.grad_offset[ti] = o
                o = _round_up(o + self.sizes[ti], galign)
            if grad_buffer != "layer":
                largest = max(largest, o)
        if grad_buffer == "layer":
            largest *= fold_streams
        self.grad_buffer_elems = max(largest, 1)
        if arena_layout not in ("slab", "separate"):
            raise ValueError(arena_layout)
        if arena_stagger_bytes % 256 or arena_stagger_bytes < 0 or arena_pitch_extra < 0:
            raise ValueError("arena_stagger_bytes must be a non-negative multiple of 256, arena_pitch_extra >= 0")
        if arena_layout == "separate" and (arena_stagger_bytes or arena_pitch_extra or pitch_tries not in (1, [0], (0,))):
            raise ValueError('arena_stagger_bytes, arena_pitch_extra and pitch_tries apply to arena_layout="slab" only')
        self._arena_layout = arena_layout
        self._arena_stagger_bytes = arena_stagger_bytes
        self._arena_pitch_extra = arena_pitch_extra
        pitch_extras = self._pitch_candidates(pitch_tries) if isinstance(pitch_tries, int) else [int(x) for x in pitch_tries]
        if placement_tries < 1 or not pitch_extras or min(pitch_extras) < 0 or placement_micro_batches < 1:
            raise ValueError("placement_tries, pitch_tries and placement_micro_batches must be >= 1 (extras >= 0)")
        self._adopt(self._place(placement_tries, pitch_extras, placement_micro_batches))

    # ---- where the state lives ----
    _TWO_MIB = 1 << 21

    def _pitch_candidates(self, k: int) -> list:
        """The first k pitch extras (2 MiB units) worth trying.  Measured on MI355X (fold of GPT-2-XL blocks against the
        distance d between m and v in 2 MiB units, 1024 consecutive distances in one slab): the rate is a mean plus
        (-1)^d times a cosine of period 256 in d, so consecutive distances alternate between fast and slow, the
        difference is largest where d is near a multiple of 128 and vanishes half-way between, and which parity is the
        fast one flips from one half-period to the next (and was found flipped for a 150 GB state).  Hence pairs of
        consecutive distances: at the smallest pitch that fits, then next to the following multiples of 128."""
        if k < 1:
            return []
        dmin = _round_up(self.arena_elems * 4 + 2 * self._arena_stagger_bytes, self._TWO_MIB) // self._TWO_MIB \
            + self._arena_pitch_extra
        phases, e = [0], (-dmin) % 128
        while len(phases) * 2 < k:
            if e not in phases and e - 1 not in phases:
                phases.append(e)
            e += 128
        return [ph + parity for ph in phases for parity in (0, 1)][:k]

    def _pitch(self, j: int) -> int:
        """Bytes between consecutive arenas of a slab for candidate j: the smallest multiple of 2 MiB that holds an
        arena (and the stagger), plus arena_pitch_extra + j times 2 MiB."""
        return (_round_up(self.arena_elems * 4 + 2 * self._arena_stagger_bytes, self._TWO_MIB)
                + (self._arena_pitch_extra + j) * self._TWO_MIB)

    def _allocate(self, max_extra: int) -> dict:
        """Device memory for one allocation of the state: the slab (or the separate arenas) and the gradient buffer."""
        narena = 3 if self.optimizer == "adam" else 2
        with torch.cuda.stream(self.stream):
            if self._arena_layout == "separate":
                mem = {"arenas": [torch.zeros(self.arena_elems, dtype=torch.float32, device=self.device)
                                  for _ in range(narena)], "slab": None}
            else:       # room for the largest pitch that may be tried, and for starting on a 2 MiB boundary
                mem = {"slab": torch.zeros(narena * self._pitch(max_extra) + self._TWO_MIB, dtype=torch.uint8,
                                           device=self.device)}
            mem["grad_buffer"] = torch.empty(self.grad_buffer_elems * self.gbytes, dtype=torch.uint8, device=self.device)
        return mem

    def _bind(self, mem: dict, j: int) -> dict:
        """One placement inside an allocation: the arenas (for a slab: at pitch candidate j) and the launch lists that
        point into them."""
        optimizer = self.optimizer
        p = {"_slab": mem["slab"], "_pitch_bytes": None}
        if mem["slab"] is None:
            views = mem["arenas"]
        else:
            arena_bytes, pitch = self.arena_elems * 4, self._pitch(j)
            base = (-mem["slab"].data_ptr()) % self._TWO_MIB
            starts = [base + k * (pitch + self._arena_stagger_bytes) for k in range(3 if optimizer == "adam" else 2)]
            if starts[-1] + arena_bytes > mem["slab"].numel():
                raise RuntimeError("arena slab too small for its layout")
            views = [mem["slab"][o: o + arena_bytes].view(torch.float32) for o in starts]
            p["_pitch_bytes"] = pitch
        p["m"], p["v"], p["theta"] = (views[0], views[1], views[2]) if optimizer == "adam" else (views[0], None, views[1])
        p["grad_buffer"] = mem["grad_buffer"]
        # ---- descriptor lists, built once ----
        gb = p["grad_buffer"].data_ptr()
        if optimizer == "sgdm":
            base_t, base_b = p["theta"].data_ptr(), p["m"].data_ptr()
            p["_sgdm_lists"] = [binding.sgdm_list(
                [(base_t + 4 * self.offset[ti], base_b + 4 * self.offset[ti],
                  gb + self.gbytes * self.grad_offset[ti], self.sizes[ti]) for ti in idx]) for idx in self.layers]
            p["_sgdm_state"] = binding.sgdm_list(
                [(base_t + 4 * o, base_b + 4 * o, None, n) for o, n in zip(self.offset, self.sizes)])
            return p
        base_t, base_m, base_v = p["theta"].data_ptr(), p["m"].data_ptr(), p["v"].data_ptr()
        p["_fold_lists"] = []
        for idx in self.layers:
            p["_fold_lists"].append(binding.tensor_list(
                [(base_m + 4 * self.offset[ti], base_v + 4 * self.offset[ti],
                  gb + self.gbytes * self.grad_offset[ti], self.sizes[ti]) for ti in idx]))
        p["_update_lists"] = []
        for idx in self.layers:
            p["_update_lists"].append(binding.update_list(
                [(base_t + 4 * self.offset[ti], base_m + 4 * self.offset[ti], base_v + 4 * self.offset[ti],
                  gb + self.gbytes * self.grad_offset[ti], self.sizes[ti]) for ti in idx]))
        p["_state_list"] = binding.state_list(
            [(base_t + 4 * o, base_m + 4 * o, base_v + 4 * o, n) for o, n in zip(self.offset, self.sizes)])
        return p

    def _adopt(self, p: dict) -> None:
        for k, x in p.items():
            setattr(self, k, x)

    def _placement_bytes(self) -> int:
        return self.arena_elems * 4 * (3 if self.optimizer == "adam" else 2) + self.grad_buffer_elems * self.gbytes

    def _allocation_bytes(self, max_extra: int) -> int:
        """What _allocate(max_extra) asks the device for."""
        narena = 3 if self.optimizer == "adam" else 2
        state = narena * self.arena_elems * 4 if self._arena_layout == "separate" \
            else narena * self._pitch(max_extra) + self._TWO_MIB
        return state + self.grad_buffer_elems * self.gbytes

    def _placement_ms(self, p: dict, micro_batches: int) -> float:
        """Milliseconds of decay + micro_batches sweeps of folds + update over placement p, its arenas holding values
        like a workload's (what the memory system delivers depends on the contents too); leaves the state zeroed."""
        gt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[self.gdtype]
        sh = self.stream.cuda_stream
        with torch.cuda.stream(self.stream):
            p["theta"].normal_(0.0, 0.02)
            p["m"].normal_(0.0, 1e-4)
            if p["v"] is not None:
                p["v"].uniform_(1e-9, 1e-7)
            p["grad_buffer"].view(gt).normal_(0.0, 1e-3)

        def decay() -> None:
            if self.optimizer == "sgdm":
                binding.adama_sgdm_begin_step_multi(p["_sgdm_state"], None, 0.9, sh)
            else:
                binding.adama_begin_step_multi(p["_state_list"], None, 0.9, 0.999, sh)

        def folds() -> None:
            for li in range(len(self.layers) - 1, -1, -1):
                if self.optimizer == "sgdm":
                    binding.adama_sgdm_fold_multi(p["_sgdm_lists"][li], None, self.gdtype, 16, None, sh)
                else:
                    binding.adama_fold_multi(p["_fold_lists"][li], None, self.gdtype, 16, 0.9, 0.999, sh)

        def update() -> None:
            if self.optimizer == "sgdm":
                binding.adama_sgdm_apply_multi(p["_sgdm_state"], None, 1e-3, None, sh)
            else:
                binding.adama_apply_multi(p["_state_list"], None, 1e-3, 1e-8, 0.9, 0.999, 1, sh)

        total = 0.0
        for fn, weight in ((decay, 1), (folds, micro_batches), (update, 1)):
            fn()                                             # untimed first pass
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(self.stream)
            fn()
            fn()
            e1.record(self.stream)
            e1.synchronize()
            total += weight * e0.elapsed_time(e1) / 2
        with torch.cuda.stream(self.stream):
            for k in ("theta", "m", "v"):
                if p[k] is not None:
                    p[k].zero_()
        self.stream.synchronize()
        return total

    def _place(self, tries: int, pitch_extras: list, micro_batches: int) -> dict:
        self.placement = {"layout": self._arena_layout, "tries": 0, "pitch_tries": len(pitch_extras), "step_ms": [],
                          "chosen": [0, 0]}
        self.placement["pitch_extras_2mib"] = pitch_extras
        search = tries > 1 or len(pitch_extras) > 1
        best, best_ms = None, float("inf")
        held = []           # every allocation tried stays allocated until the search ends: a freed one would be
        for i in range(tries):                                # handed out again, and the search would go in circles
            if i > 0:
                free, _ = torch.cuda.mem_get_info(self.device)
                if free < self._allocation_bytes(max(pitch_extras)) + (1 << 30):
                    self.placement["note"] = "no room for another copy of the state: stopped"
                    break
            try:
                mem = self._allocate(max(pitch_extras))
            except torch.cuda.OutOfMemoryError:
                if i == 0:
                    raise
                self.placement["note"] = "no room for another copy of the state: stopped"
                break
            held.append(mem)
            self.placement["tries"] = i + 1
            row = []
            for j, extra in enumerate(pitch_extras):
                cand = self._bind(mem, extra)
                if not search:
                    if cand["_pitch_bytes"] is not None:
                        self.placement["pitch_2mib"] = cand["_pitch_bytes"] // self._TWO_MIB
                    return cand
                ms = self._placement_ms(cand, micro_batches)
                row.append(round(ms, 3))
                if ms < best_ms:
                    best, best_ms, self.placement["chosen"] = cand, ms, [i, j]
            self.placement["step_ms"].append(row)
            del mem, cand
        del held
        torch.cuda.empty_cache()                             # hand the losers' memory back to the driver
        if best["_pitch_bytes"] is not None:
            self.placement["pitch_2mib"] = best["_pitch_bytes"] // self._TWO_MIB
        with torch.cuda.stream(self.stream):                 # candidates of one slab overlap: zero the winner last
            for k in ("theta", "m", "v"):
                if best[k] is not None:
                    best[k].zero_()
        self.stream.synchronize()
        return best

    # ---- memory accounting (a4) ----
    @property
    def peak_grad_bytes(self) -> int:
        """Bytes of gradient storage that ever exist at once: the single buffer."""
        return self.grad_buffer_elems * self.gbytes

    @property
    def whole_model_grad_bytes(self) -> int:
        """What plain gradient accumulation would have to keep for the whole mini-batch."""
        return sum(self.sizes) * self.gbytes

    # ---- addresses for producers and checks ----
    @property
    def stream_handle(self) -> int:
        return self.stream.cuda_stream

    def use_fold_streams(self, k: int) -> None:
        """Change the number of fold streams between mini-batches.  Only with grad_buffer="model" (every layer has
        its own gradient region): the single-buffer layout fixes one region per stream at construction."""
        if self._grad_buffer_mode == "layer" and k != len(self.fold_streams):
            raise RuntimeError('the number of fold streams of a grad_buffer="layer" harness is fixed at construction')
        if k < 1:
            raise ValueError("fold_streams must be >= 1")
        self.synchronize()
        self.fold_streams = (self.fold_streams + [torch.cuda.Stream(device=self.device)
                                                  for _ in range(k - len(self.fold_streams))])[:k]

    def layer_stream(self, li: int) -> torch.cuda.Stream:
        """The stream layer li's gradients are produced and folded on."""
        return self.fold_streams[li % len(self.fold_streams)]

    def layer_stream_handle(self, li: int) -> int:
        return self.layer_stream(li).cuda_stream

    def _fan_out(self) -> None:
        """The other fold streams wait for what the main stream has queued so far."""
        if len(self.fold_streams) > 1:
            ev = torch.cuda.Event()
            ev.record(self.stream)
            for s in self.fold_streams[1:]:
                s.wait_event(ev)

    def _fan_in(self) -> None:
        """The main stream waits for what the other fold streams have queued so far."""
        for s in self.fold_streams[1:]:
            ev = torch.cuda.Event()
            ev.record(s)
            self.stream.wait_event(ev)

    def grad_ptr(self, ti: int) -> int:
        return self.grad_buffer.data_ptr() + self.gbytes * self.grad_offset[ti]

    def theta_ptr(self, ti: int) -> int:
        return self.theta.data_ptr() + 4 * self.offset[ti]

    def tensor_view(self, which: str, ti: int) -> torch.Tensor:
        arena = {"theta": self.theta, "m": self.m, "b": self.m, "v": self.v}[which]
        return arena[self.offset[ti]: self.offset[ti] + self.sizes[ti]]

    # ---- Alg. 2 ----
    def begin_step(self, beta1: float, beta2: float) -> None:
        """t <- t+1, m <- beta1 m, v <- beta2 v."""
        self.t += 1
        if self.optimizer == "sgdm":
            binding.adama_sgdm_begin_step_multi(self._sgdm_state, None, self.momentum, self.stream_handle)
        else:
            binding.adama_begin_step_multi(self._state_list, None, beta1, beta2, self.stream_handle)
        self._fan_out()

    def fold_layer(self, li: int, N: int, beta1: float, beta2: float) -> None:
        sh = self.layer_stream_handle(li)
        if self.optimizer == "sgdm":
            binding.adama_sgdm_fold_multi(self._sgdm_lists[li], None, self.gdtype, N, self._opt, sh)
        elif self._opt is None:
            binding.adama_fold_multi(self._fold_lists[li], None, self.gdtype, N, beta1, beta2, sh)
        else:
            binding.adama_fold_opt_multi(self._fold_lists[li], None, self.gdtype, N, beta1, beta2, self._opt, sh)

    # ---- the same mini-batch with the decay and the update riding along with the edge folds ----
    def begin_step_fused(self) -> None:
        """t <- t+1 only: the decay is performed by fold_layer_first in micro-batch 0."""
        self.t += 1
        self._fan_out()

    def fold_layer_first(self, li: int, N: int, beta1: float, beta2: float) -> None:
        """Micro-batch 0: decay + fold of layer li in one pass (Alg. 1's one-statement form)."""
        sh = self.layer_stream_handle(li)
        if self.optimizer == "sgdm":
            binding.adama_sgdm_fold_first_multi(self._sgdm_lists[li], None, self.gdtype, N, self.momentum, self._opt, sh)
        elif self._opt is None:
            binding.adama_fold_first_multi(self._fold_lists[li], None, self.gdtype, N, beta1, beta2, sh)
        else:
            binding.adama_fold_first_opt_multi(self._fold_lists[li], None, self.gdtype, N, beta1, beta2, self._opt, sh)

    def fold_layer_last_apply(self, li: int, N: int, lr: float, eps: float, beta1: float, beta2: float) -> None:
        """Micro-batch N-1: fold + parameter update of layer li in one pass."""
        sh = self.layer_stream_handle(li)
        if self.optimizer == "sgdm":
            binding.adama_sgdm_fold_last_apply_multi(self._sgdm_lists[li], None, self.gdtype, N, lr, self._opt, sh)
        elif self._opt is None:
            binding.adama_fold_last_apply_multi(self._update_lists[li], None, self.gdtype, N, lr, eps, beta1, beta2,
                                                self.t, sh)
        else:
            binding.adama_fold_last_apply_opt_multi(self._update_lists[li], None, self.gdtype, N, lr, eps, beta1,
                                                    beta2, self.t, self._opt, sh)

    def mini_batch_fused(self, produce: Callable[[int, int], None], N: int, lr: float, eps: float, beta1: float,
                         beta2: float) -> None:
        """One full pass of the hot path with fused edges; bit-identical to mini_batch()."""
        if N == 1:                       # a single micro-batch is both first and last: keep the decay separate
            self.begin_step(beta1, beta2)
        else:
            self.begin_step_fused()
        for i in range(N):
            for li in range(len(self.layers) - 1, -1, -1):
                produce(i, li)
                if i == N - 1:
                    self.fold_layer_last_apply(li, N, lr, eps, beta1, beta2)
                elif i == 0:
                    self.fold_layer_first(li, N, beta1, beta2)
                else:
                    self.fold_layer(li, N, beta1, beta2)

    def micro_batch(self, produce: Callable[[int], None], N: int, beta1: float, beta2: float) -> None:
        """One backward pass: for each layer, last to first, produce(li) must enqueue on
        self.layer_stream(li) (self.stream unless fold_streams > 1) the writes of that layer's gradients
        into the buffer; the layer is then folded."""
        for li in range(len(self.layers) - 1, -1, -1):
            produce(li)
            self.fold_layer(li, N, beta1, beta2)

    def apply(self, lr: float, eps: float, beta1: float, beta2: float) -> None:
        self._fan_in()
        if self.optimizer == "sgdm":
            binding.adama_sgdm_apply_multi(self._sgdm_state, None, lr, self._opt, self.stream_handle)
        elif self._opt is None:
            binding.adama_apply_multi(self._state_list, None, lr, eps, beta1, beta2, self.t, self.stream_handle)
        else:
            binding.adama_apply_opt_multi(self._state_list, None, lr, eps, beta1, beta2, self.t, self._opt,
                                          self.stream_handle)

    def mini_batch(self, produce: Callable[[int, int], None], N: int, lr: float, eps: float, beta1: float,
                   beta2: float) -> None:
        """One full pass of the hot path; produce(micro, li) fills the buffer with layer li's gradients."""
        self.begin_step(beta1, beta2)
        for i in range(N):
            self.micro_batch(lambda li, i=i: produce(i, li), N, beta1, beta2)
        self.apply(lr, eps, beta1, beta2)

    # ---- HIP graph of a launch-bound sequence ----
    def capture(self, enqueue: Callable[[], None]) -> "torch.cuda.CUDAGraph":
        """Record everything `enqueue` launches on self.stream into a HIP graph and return it; replay with
        graph.replay().  libadama's entry points neither allocate nor synchronise and carry their tensor
        tables inside the kernel arguments, so they can be captured as they are.  The step counter is host
        state: capture sequences whose scalars do not depend on t (decay and folds), or re-capture per step."""
        if len(self.fold_streams) > 1:
            raise RuntimeError("capture() records one stream: use fold_streams=1")
        graph = torch.cuda.CUDAGraph()
        self.stream.synchronize()
        with torch.cuda.graph(graph, stream=self.stream):
            enqueue()
        return graph

    def synchronize(self) -> None:
        for s in self.fold_streams:
            s.synchronize()
