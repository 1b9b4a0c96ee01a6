#!/usr/bin/env python3
"""Benchmark of the AdamA hot path (decay + N x per-layer fold + update) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3|c2|c5|c4|c1] [--optimizer adama|adamw|sgdm]

A "step" is one whole mini-batch of the workload through libadama: adama_begin_step over all state,
then for each of the N micro-batches one adama_fold_multi launch per layer in backward order, then
adama_apply.  All inputs (theta, m, v and one micro-batch's worth of per-layer gradients, each layer
at its own address) are resident in HBM before the clock starts; the timed region contains only
libadama launches.  Prints ONE JSON line.

--optimizer selects the same pass for a variant: "adamw" (decoupled weight decay 0.01 in the update,
same kernels and bytes) or "sgdm" (SGD with momentum 0.9 accumulated the same way: one moment, so
8 B decay + N x (8 + gradient) B folds + 12 B update per parameter).  The default is the paper's AdamA.

Before the warm-up the harness places the state: what HBM delivers depends on where the arrays lie (the
distance between the arenas, the physical pages behind them: 2..6 % of the step), so it times
--placement-tries allocations x --pitch-tries distances and keeps the fastest; every candidate's
estimated step time is reported as arena_placement (1 and 1 = take the first).

Other modes: --graph (a micro-batch's sweep eager and as a HIP graph), --fold-streams K (folds spread
over K streams, reported beside the one-stream figure), --library FILE (a variant build, for A/B),
--calibration-copy (a known-size copy kernel for scaling hardware counters), --stream-probe (instead of
the benchmark: what the memory system delivers for the path's read : write mixes, cache policies,
residency bounds, a persistent grid and a sweep of launch sizes, with no optimizer arithmetic).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published


WEIGHT_DECAY = {"adama": 0.0, "adamw": 0.01, "sgdm": 0.0}
MOMENTUM = 0.9


def state_bytes(optimizer: str) -> int:
    """Bytes per parameter a pass over the moments reads and writes: m, v (Adam) or b (SGD)."""
    return 8 if optimizer == "sgdm" else 16


def per_param_bytes(w, optimizer: str, fused: bool = False) -> int:
    """Separate calls: decay (moments r+w) + N folds (moments r+w + gradient) + update (theta r+w + moments r).
    Fused edges: no decay pass, and the update adds only theta r+w to the last fold."""
    s = state_bytes(optimizer)
    if fused:
        return w.N * (s + w.grad_bytes) + 8
    return s + w.N * (s + w.grad_bytes) + (8 + s // 2)


def algorithmic_bytes_per_step(w, optimizer: str = "adama") -> int:
    return per_param_bytes(w, optimizer) * w.P


def cpu_baseline(w, budget_s: float = 15.0, optimizer: str = "adama") -> dict:
    """The fp64 oracle, as it stands, timed on this host over the tensors of whole layers of the same
    workload (one full mini-batch each: decay, N folds, update) until about `budget_s` seconds are
    used.  Tensors longer than 16 M elements contribute their first 16 M (the method is elementwise, so
    a prefix is a fair sample)."""
    import numpy as np

    import oracle
    import synth

    cap = 16_000_000
    gd = None if w.gdtype == "f32" else w.gdtype
    spent, params, layers_done, capped = 0.0, 0, 0, False
    for li in sorted(range(len(w.layers)), key=lambda li: -w.layer_elems(li)):
        if spent >= budget_s:
            break
        for ti in w.layers[li]:
            if spent >= budget_s:
                break
            n = min(w.tensors[ti].n, cap)
            capped = capped or n < w.tensors[ti].n
            theta = synth.fill_host(w.theta_spec(ti), "f32", n).astype(np.float64)
            m = np.zeros(n)
            v = np.zeros(n)
            grads = [synth.fill_host(w.grad_spec(1, i, ti), w.gdtype, n) for i in range(min(w.N, 2))]
            t0 = time.perf_counter()
            if optimizer == "sgdm":
                oracle.sgdm_begin_step(m, MOMENTUM)
                for i in range(w.N):
                    oracle.sgdm_fold(m, grads[i % len(grads)], w.N, 1.0, gdtype=gd)
                oracle.sgdm_apply(theta, m, w.lr, WEIGHT_DECAY[optimizer])
            else:
                oracle.begin_step(m, v, w.beta1, w.beta2)
                for i in range(w.N):
                    oracle.fold(m, v, grads[i % len(grads)], w.N, w.beta1, w.beta2, gdtype=gd)
                if optimizer == "adamw":
                    oracle.apply_adamw(theta, m, v, w.lr, w.eps, w.beta1, w.beta2, 1, WEIGHT_DECAY[optimizer])
                else:
                    oracle.apply(theta, m, v, w.lr, w.eps, w.beta1, w.beta2, 1)
            spent += time.perf_counter() - t0
            params += n
        layers_done += 1
    per_param = per_param_bytes(w, optimizer)
    return {"value": round(params * per_param / spent / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "extrapolated": True,       # a rate per parameter from a bounded sample of the workload, not a run of all of it
            "params_per_s": round(params / spent, 1),
            "sample": f"extrapolated from a prefix sample: tensors of the {layers_done} largest layer(s) of {w.name} ({params} params"
                      f"{', at most the first 16 M elements of each' if capped else ''}), one full mini-batch "
                      f"each (decay + {w.N} folds + update) in {spent:.1f} s, single thread, fp64"}


def cpu_baseline_all_cores(w, budget_s: float = 8.0, optimizer: str = "adama") -> dict:
    """The same oracle loops, unchanged, called from one thread per host core on disjoint contiguous
    slices of each tensor (the method is elementwise, so slices are independent units)."""
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    import oracle
    import synth

    cores = max(1, min(16, len(os.sched_getaffinity(0))))
    gd = None if w.gdtype == "f32" else w.gdtype
    wd = WEIGHT_DECAY[optimizer]

    def work(theta, m, v, grads):
        if optimizer == "sgdm":
            oracle.sgdm_begin_step(m, MOMENTUM)
            for i in range(w.N):
                oracle.sgdm_fold(m, grads[i % len(grads)], w.N, 1.0, gdtype=gd)
            oracle.sgdm_apply(theta, m, w.lr, wd)
        else:
            oracle.begin_step(m, v, w.beta1, w.beta2)
            for i in range(w.N):
                oracle.fold(m, v, grads[i % len(grads)], w.N, w.beta1, w.beta2, gdtype=gd)
            if optimizer == "adamw":
                oracle.apply_adamw(theta, m, v, w.lr, w.eps, w.beta1, w.beta2, 1, wd)
            else:
                oracle.apply(theta, m, v, w.lr, w.eps, w.beta1, w.beta2, 1)

    spent, params, tensors_done = 0.0, 0, 0
    big = sorted((t for t in w.tensors if t.n >= 1_000_000), key=lambda t: t.n) or list(w.tensors)
    with ThreadPoolExecutor(max_workers=cores) as pool:
        for t in big:
            if spent >= budget_s:
                break
            n = min(t.n, 32_000_000)
            theta = synth.fill_host(w.theta_spec(t.index), "f32", n).astype(np.float64)
            m, v = np.zeros(n), np.zeros(n)
            grads = [synth.fill_host(w.grad_spec(1, i, t.index), w.gdtype, n) for i in range(min(w.N, 2))]
            cuts = [n * k // cores for k in range(cores + 1)]
            t0 = time.perf_counter()
            jobs = [pool.submit(work, theta[a:b], m[a:b], v[a:b], [g[a:b] for g in grads])
                    for a, b in zip(cuts[:-1], cuts[1:]) if b > a]
            for j in jobs:
                j.result()
            spent += time.perf_counter() - t0
            params += n
            tensors_done += 1
    per_param = per_param_bytes(w, optimizer)
    return {"value": round(params * per_param / spent / 1e9, 3), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "extrapolated": True,
            "params_per_s": round(params / spent, 1),
            "sample": f"{tensors_done} large tensor(s) of {w.name} ({params} params), one full mini-batch each, every "
                      f"tensor cut into {cores} contiguous slices run by {cores} threads calling the unchanged "
                      f"oracle, {spent:.1f} s, fp64"}


def stream_probe(block_sizes=(128, 256), launch_elems: int = 30_740_800, arena_elems: int = 1_557_611_200) -> dict:
    """What the memory system delivers for the access mixes of the path's kernels, without their arithmetic
    (synth_stream_probe_kernel): pure read, pure write, and the read : write mixes of fold, decay, update and
    rescale, as sustained launches of one transformer block's size marching through arrays as large as the
    GPT-2-1.5B-shaped state and filled with values like the workload's; then the fold mix on all-zero
    arrays (the delivered bandwidth depends on the contents), at bounded residency, and over a sweep of
    launch sizes."""
    import numpy as np
    import torch

    import synth
    from synth import gen

    dev = "cuda:0"
    stream = torch.cuda.Stream(device=dev)
    # one slab: three float32 arrays a pitch apart (a multiple of 2 MiB; the distance decides which memory channels
    # arrays streamed in lock step meet on, so two pitches that differ by 2 MiB are measured), then the gradients
    two_mib = 1 << 21
    pitch0 = (arena_elems * 4 + two_mib - 1) // two_mib * two_mib
    with torch.cuda.stream(stream):
        slab = torch.empty(3 * (pitch0 + two_mib) + arena_elems * 4 + 2 * two_mib, dtype=torch.uint8, device=dev)
        sink = torch.zeros(4, dtype=torch.float32, device=dev)
    stream.synchronize()
    sh = stream.cuda_stream
    slab_base = (-slab.data_ptr()) % two_mib
    g = slab[slab_base + 3 * (pitch0 + two_mib):][: arena_elems * 4].view(torch.float32)   # read as 16-bit or as float32 elements
    assert g.numel() == arena_elems
    arrays = []

    def place(extra: int) -> None:
        """The three float32 arrays at pitch0 + extra * 2 MiB from one another."""
        arrays[:] = [slab[slab_base + k * (pitch0 + extra * two_mib):][: arena_elems * 4].view(torch.float32) for k in range(3)]
        assert all(a.numel() == arena_elems for a in arrays)

    place(0)

    def fill(zero: bool) -> None:
        """Values like the workload's (weights N(0, 0.02), moments at their usual magnitudes, gradients N(0, 1e-3)
        in both 16-bit halves), or zeros."""
        with torch.cuda.stream(stream):
            if zero:
                for a in arrays + [g]:
                    a.zero_()
            else:
                arrays[0].normal_(0.0, 1e-4)
                arrays[1].uniform_(1e-9, 1e-7)
                arrays[2].normal_(0.0, 0.02)
                g.view(torch.bfloat16).normal_(0.0, 1e-3)
        stream.synchronize()

    def sustained(mode: str, block: int, n: int, passes: int = 2, lds: int = 0, groups: int = 1) -> tuple:
        n -= n % (block * 4 * groups)
        slots = max(1, arena_elems // n)

        def launch(r: int) -> None:
            off = (r % slots) * n
            gen.stream_probe(mode, block, g.data_ptr() + 4 * off, arrays[0].data_ptr() + 4 * off,
                             arrays[1].data_ptr() + 4 * off, arrays[2].data_ptr() + 4 * off, sink.data_ptr(), n, sh,
                             lds_bytes=lds, groups=groups)

        reps = max(passes * slots, 20)
        for r in range(min(slots, reps)):
            launch(r)
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for r in range(reps):
            launch(r)
        e1.record(stream)
        e1.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        return n, us, gen.stream_probe_bytes(mode) * n / (us * 1e-6) / 1e9

    out = {"launch_elems": launch_elems, "array_elems": arena_elems, "modes": {}, "note":
           "one workgroup per block*4 elements, 16-byte accesses, all non-temporal, no optimizer arithmetic; arrays hold "
           "values like the workload's; GB/s = bytes the mode moves / HIP-event time over back-to-back launches"}
    by_pitch = []
    for extra in (0, 1):
        place(extra)
        fill(zero=False)
        table = {}
        for rnd in range(2):                       # two rounds, the better one is kept (first-touch effects)
            for mode in gen.PROBE_MODES:
                for block in block_sizes:
                    n, us, gbs = sustained(mode, block, launch_elems)
                    key = f"{mode}/{block}"
                    if key not in table or gbs > table[key]["GB/s"]:
                        table[key] = {"bytes_per_element": gen.stream_probe_bytes(mode), "us_per_launch": round(us, 2),
                                      "GB/s": round(gbs, 1)}
                if mode == "write_m_v":
                    fill(zero=False)               # the pure-write mode overwrites the arrays: restore the contents
        by_pitch.append(table)
    # the pitch under which the fold's mix streams faster is used from here on; the other one is reported beside it
    keep = 0 if by_pitch[0]["fold_mix_g16/128"]["GB/s"] >= by_pitch[1]["fold_mix_g16/128"]["GB/s"] else 1
    out["modes"] = by_pitch[keep]
    out["pitch_2mib"] = pitch0 // two_mib + keep
    out["modes_at_the_other_pitch"] = {k: v["GB/s"] for k, v in by_pitch[1 - keep].items()}
    place(keep)
    fill(zero=False)
    best = {m: max(out["modes"][f"{m}/{b}"]["GB/s"] for b in block_sizes) for m in gen.PROBE_MODES}
    rd, wr = best["read_g16_m_v"], best["write_m_v"]
    out["best"] = best
    # time on the memory bus adds up: a mix of r read bytes and w written bytes cannot beat (r + w) / (r / R + w / W)
    out["harmonic_ceiling"] = {name: round((r + w) / (r / rd + w / wr), 1)
                               for name, (r, w) in {"fold_mix_g16": (10, 8), "fold_mix_g32": (12, 8), "decay_mix": (8, 8),
                                                    "update_mix": (12, 4), "rescale_mix": (12, 12)}.items()}
    # residency: the fold mix with the number of workgroups per compute unit bounded through unused LDS
    out["residency_fold_mix_g16"] = {}
    for block, groups, wgs in ((128, 1, 0), (128, 1, 12), (128, 1, 8), (128, 1, 6), (256, 1, 4), (128, 2, 4)):
        lds = 0 if wgs == 0 else (160 * 1024 // wgs) & ~1023
        fill(zero=False)
        _, _, gbs = sustained("fold_mix_g16", block, launch_elems, lds=lds, groups=groups)
        out["residency_fold_mix_g16"][f"{block}x{groups}@{wgs or 'all'}"] = round(gbs, 1)
    # persistent grid: k workgroups of 128 threads per compute unit walk the chunks with a fixed stride
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    n_per = launch_elems - launch_elems % 512
    slots_per = max(1, arena_elems // n_per)
    out["persistent_grid_fold_mix_g16"] = {}
    for k in (2, 3, 4, 6, 8, 16):
        fill(zero=False)

        def launch(r: int, k: int = k) -> None:
            off = (r % slots_per) * n_per
            gen.stream_probe_persistent("fold_mix_g16", 128, cus * k, g.data_ptr() + 4 * off, arrays[0].data_ptr() + 4 * off,
                                        arrays[1].data_ptr() + 4 * off, arrays[2].data_ptr() + 4 * off, sink.data_ptr(), n_per, sh)
        for r in range(slots_per):
            launch(r)
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for r in range(2 * slots_per):
            launch(r)
        e1.record(stream)
        e1.synchronize()
        out["persistent_grid_fold_mix_g16"][f"{k} workgroups per compute unit"] = round(
            18 * n_per * 2 * slots_per / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    sweep = []
    for n in (1 << 20, 1 << 22, 1 << 23, 1 << 24, launch_elems, 1 << 26, 1 << 27, 1 << 28):
        n_, us, gbs = sustained("fold_mix_g16", 128, n)
        sweep.append({"elems": n_, "us_per_launch": round(us, 2), "GB/s": round(gbs, 1)})
    xs = np.array([p["elems"] * 18.0 for p in sweep[:5]])      # up to one transformer block: beyond, long launches slow down
    ts = np.array([p["us_per_launch"] for p in sweep[:5]])
    slope, icpt = np.polyfit(xs, ts, 1)
    out["launch_size_sweep"] = {"mode": "fold_mix_g16/128", "points": sweep,
                                "fit_up_to_one_block": {"fixed_us_per_launch": round(float(icpt), 2),
                                                        "asymptotic_GB/s": round(1.0 / slope / 1e3, 1)}}
    # cache policy: the fold mix (16-bit gradient, 128 x 1) with each combination of the sc0 / sc1 / nt modifiers
    fill(zero=False)
    n_pol = launch_elems - launch_elems % 512
    slots = max(1, arena_elems // n_pol)

    def policy_rate(lp: str, sp: str, what: str) -> float:
        def launch(r: int) -> None:
            off = (r % slots) * n_pol
            gen.cache_policy_probe(lp, sp, what, g.data_ptr() + 4 * off, arrays[0].data_ptr() + 4 * off,
                                   arrays[1].data_ptr() + 4 * off, sink.data_ptr(), n_pol, sh)
        for r in range(slots):
            launch(r)
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for r in range(2 * slots):
            launch(r)
        e1.record(stream)
        e1.synchronize()
        bytes_per = {"mix": 18, "read": 10, "write": 8}[what]
        return round(bytes_per * n_pol * 2 * slots / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)

    pol = list(gen.CACHE_POLICIES)
    out["cache_policy"] = {
        "note": "fold mix with written-out global loads / stores; '' = no modifier; GB/s",
        "mix_loads_nt_stores": {sp: policy_rate("nt", sp, "mix") for sp in pol},
        "mix_stores_sc1_nt_loads": {lp: policy_rate(lp, "sc1 nt", "mix") for lp in pol},
        "mix_no_modifiers": policy_rate("", "", "mix"),
        "reads_alone": {lp: policy_rate(lp, "", "read") for lp in pol},
    }
    out["cache_policy"]["writes_alone"] = {sp: policy_rate("", sp, "write") for sp in pol}
    # the same fold mix on all-zero arrays: the contents matter
    fill(zero=True)
    out["all_zero_arrays"] = {f"fold_mix_g16/{b}": round(sustained("fold_mix_g16", b, launch_elems)[2], 1) for b in block_sizes}
    lds = (160 * 1024 // 4) & ~1023
    out["all_zero_arrays"]["fold_mix_g16/256x1@4"] = round(sustained("fold_mix_g16", 256, launch_elems, lds=lds)[2], 1)
    del synth
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--optimizer", default="adama", choices=["adama", "adamw", "sgdm"],
                    help="adama: the paper's method (default); adamw / sgdm: the same pass for the variants")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB copy kernel (the known-size reference for hardware traffic counters)")
    ap.add_argument("--graph", action="store_true",
                    help="also time one micro-batch's fold sweep as eager launches and as a HIP graph replay")
    ap.add_argument("--cpu-budget", type=float, default=15.0, help="seconds of oracle time for cpu_baseline (0 = skip)")
    ap.add_argument("--stream-probe", action="store_true",
                    help="instead of the benchmark: measure what the memory system delivers for the read : write mixes "
                         "of the path's kernels (no optimizer arithmetic) and print that as one JSON line")
    ap.add_argument("--fold-streams", type=int, default=1,
                    help="also time the same mini-batch with the folds of different layers spread over this many streams "
                         "(layer l on stream l mod K; measured: no robust gain); reported as overlapped_folds")
    ap.add_argument("--placement-tries", type=int, default=8,
                    help="allocations of the state the harness may try before the run (untimed set-up; needs room for a "
                         "second copy): the same step runs 2..6 %% faster or slower depending on where the arrays lie; "
                         "every candidate's estimated step time is reported as arena_placement")
    ap.add_argument("--arena-layout", default="slab", choices=["slab", "separate"],
                    help="how the harness lays out theta, m, v: one allocation with the arenas a multiple of 2 MiB apart "
                         "(default), or one allocation per arena")
    ap.add_argument("--pitch-tries", type=int, default=8,
                    help="distances between the arenas of a slab the harness may try: pairs 2 MiB apart, at the smallest "
                         "distance that fits and next to the following multiples of 256 MiB (under 1 GB of extra memory)")
    ap.add_argument("--library", default=None,
                    help="run a variant build of the library (python -m paper_2305_19982_amd.build --out ...) instead "
                         "of the package's own, for A/B measurements; the line's library_build then reads \"variant\"")
    ap.add_argument("--no-torch-ops", action="store_true",
                    help="skip the context figure for the same fold written as stock PyTorch tensor ops")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (no sharding, no collectives); run with --gpus 1",
              file=sys.stderr)
        return 2

    import torch

    import synth
    from paper_2305_19982_amd import binding
    from paper_2305_19982_amd.harness import SimulatedBackward
    from synth import configs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    if args.library:
        binding.use_library(args.library)
    if args.stream_probe:
        print(json.dumps({"stream_probe": stream_probe(), "peak_GB/s": HBM_PEAK_GBS}), flush=True)
        return 0
    binding.load()                      # raises if libadama.so is missing or older than its sources
    w = configs.FULL[args.workload]()
    opt = args.optimizer
    hb = SimulatedBackward([t.n for t in w.tensors], w.layers, w.gdtype, grad_buffer="model",
                           optimizer="sgdm" if opt == "sgdm" else "adam", momentum=MOMENTUM,
                           weight_decay=WEIGHT_DECAY[opt], arena_layout=args.arena_layout,
                           placement_tries=args.placement_tries,
                           pitch_tries=args.pitch_tries if args.arena_layout == "slab" else 1,
                           placement_micro_batches=w.N)
    sh = hb.stream_handle
    # ---- resident inputs: theta0 and one micro-batch of gradients, every layer at its own address ----
    for t in w.tensors:
        synth.fill_device(hb.theta_ptr(t.index), w.theta_spec(t.index), "f32", t.n, sh)
        synth.fill_device(hb.grad_ptr(t.index), w.grad_spec(1, 0, t.index), w.gdtype, t.n, sh)
    hb.synchronize()

    # the dominant kernel: the multi-tensor, big-chunk fold instantiation (whole transformer blocks)
    tune = binding.adama_tuning()
    big_layers = {li for li in range(len(w.layers))
                  if w.layer_elems(li) >= tune["big_launch_elems"] and len(w.layers[li]) > 1}
    if not big_layers:        # workloads without such layers: time every big-chunk launch
        big_layers = {li for li in range(len(w.layers)) if w.layer_elems(li) >= tune["big_launch_elems"]}
    fold_events = []
    class_events = {"decay": [], "fold": [], "update": []}     # (start, end) pairs per kernel class

    def mark():
        e = torch.cuda.Event(enable_timing=True)
        e.record(hb.stream)
        return e

    def one_step(timed: bool) -> None:
        """timed: bracket every run of consecutive dominant-kernel launches with one HIP event pair
        recorded on the launch stream (a pair per launch would add its own overhead to each), and the
        decay, each micro-batch's sweep of folds, and the update with one pair each."""
        t_a = mark() if timed else None
        hb.begin_step(w.beta1, w.beta2)
        t_b = mark() if timed else None
        if timed:
            class_events["decay"].append((t_a, t_b))
        for _ in range(w.N):
            t_s = mark() if timed else None
            run_start, run_elems, run_launches = None, 0, 0
            for li in w.backward_layers():
                big = li in big_layers
                if timed and big and run_start is None:
                    run_start = torch.cuda.Event(enable_timing=True)
                    run_start.record(hb.stream)
                if timed and not big and run_start is not None:
                    end = torch.cuda.Event(enable_timing=True)
                    end.record(hb.stream)
                    fold_events.append((run_start, end, run_elems, run_launches))
                    run_start, run_elems, run_launches = None, 0, 0
                hb.fold_layer(li, w.N, w.beta1, w.beta2)
                if big:
                    run_elems += w.layer_elems(li)
                    run_launches += 1
            if timed and run_start is not None:
                end = torch.cuda.Event(enable_timing=True)
                end.record(hb.stream)
                fold_events.append((run_start, end, run_elems, run_launches))
            if timed:
                class_events["fold"].append((t_s, mark()))
        t_c = mark() if timed else None
        hb.apply(w.lr, w.eps, w.beta1, w.beta2)
        if timed:
            class_events["update"].append((t_c, mark()))

    if args.calibration_copy:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0")
        torch.cuda.synchronize()
        synth.gen.copy_device(dst.data_ptr(), src.data_ptr(), 1 << 30, sh)
        hb.synchronize()
        del src, dst

    for _ in range(args.warmup):
        one_step(False)
    hb.synchronize()
    torch.cuda.synchronize()
    step_marks = [mark()]
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step(False)
        step_marks.append(mark())          # recorded on the stream, not waited for
    hb.synchronize()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    in_order = [a.elapsed_time(b) for a, b in zip(step_marks[:-1], step_marks[1:])]
    per_step = sorted(in_order)
    # up to 16 evenly spaced steps in the order they ran: shows a drift over the timed region, if any
    trace_ms = [round(in_order[(i * (len(in_order) - 1)) // 15 if len(in_order) > 16 else i], 3) for i in range(min(16, len(in_order)))]
    median_ms = per_step[len(per_step) // 2] if len(per_step) % 2 else 0.5 * (per_step[len(per_step) // 2 - 1] + per_step[len(per_step) // 2])

    # ---- the same mini-batch with fused edges (decay inside micro-batch 0's folds, update inside the last) ----
    def one_step_fused() -> None:
        hb.begin_step_fused()
        for i in range(w.N):
            for li in w.backward_layers():
                if i == w.N - 1:
                    hb.fold_layer_last_apply(li, w.N, w.lr, w.eps, w.beta1, w.beta2)
                elif i == 0:
                    hb.fold_layer_first(li, w.N, w.beta1, w.beta2)
                else:
                    hb.fold_layer(li, w.N, w.beta1, w.beta2)

    # ---- launch-bound workloads: one micro-batch's fold sweep as a HIP graph ----
    graph_sweep = None
    if args.graph:
        def sweep() -> None:
            for li in w.backward_layers():
                hb.fold_layer(li, w.N, w.beta1, w.beta2)

        g = hb.capture(sweep)
        reps = 20
        for fn, label in ((lambda: sweep(), "eager"), (lambda: g.replay(), "graph")):
            with torch.cuda.stream(hb.stream):
                fn()
                hb.synchronize()
                t2 = time.perf_counter()
                for _ in range(reps):
                    fn()
                hb.synchronize()
            us = (time.perf_counter() - t2) / reps / len(w.layers) * 1e6
            graph_sweep = dict(graph_sweep or {}, **{f"{label}_us_per_launch": round(us, 2)})
        graph_sweep["launches_per_sweep"] = len(w.layers)

    # ---- context: the fold of one micro-batch written as stock PyTorch tensor ops (the style of the
    # paper's own hook implementation), on the same tensors, same GPU.  Not the product path.
    torch_ops = None
    if not args.no_torch_ops and opt != "sgdm" and w.P <= 4_000_000_000:
        tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[w.gdtype]
        c1, c2 = (1.0 - w.beta1) / w.N, (1.0 - w.beta2) / (w.N * w.N)
        views = []
        for li in w.backward_layers():
            ms_, vs_, gs_ = [], [], []
            for ti in w.layers[li]:
                n, go = w.tensors[ti].n, hb.grad_offset[ti] * hb.gbytes
                ms_.append(hb.tensor_view("m", ti))
                vs_.append(hb.tensor_view("v", ti))
                gs_.append(hb.grad_buffer[go: go + n * hb.gbytes].view(tdt))
            views.append((ms_, vs_, gs_))

        def torch_sweep() -> None:
            for ms_, vs_, gs_ in views:
                g32 = [g.float() for g in gs_] if tdt != torch.float32 else gs_
                torch._foreach_add_(ms_, g32, alpha=c1)
                torch._foreach_addcmul_(vs_, g32, g32, value=c2)

        with torch.cuda.stream(hb.stream):
            torch_sweep()
            hb.synchronize()
            t3 = time.perf_counter()
            for _ in range(3):
                torch_sweep()
            hb.synchronize()
            tms = (time.perf_counter() - t3) / 3 * 1e3
        torch_ops = {"fold_sweep_ms": round(tms, 3),
                     "GB/s": round((state_bytes(opt) + w.grad_bytes) * w.P / (tms * 1e-3) / 1e9, 1),
                     "note": "one micro-batch's folds as torch._foreach_add_ / _foreach_addcmul_ on the same tensors "
                             "(float32 copy of 16-bit gradients first); algorithmic bytes / time; context only"}
        del views

    fused = None
    if w.N > 1:
        one_step_fused()
        hb.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            one_step_fused()
        hb.synchronize()
        fused_ms = (time.perf_counter() - t1) / args.steps * 1e3
        fused_bytes = per_param_bytes(w, opt, fused=True) * w.P
        fused = {"ms_per_step": round(fused_ms, 3), "bytes_per_step": fused_bytes,
                 "value": round(fused_bytes / (fused_ms * 1e-3) / 1e9, 1), "unit": "GB/s",
                 "params_per_s": round(w.P / (fused_ms * 1e-3), 1),
                 "note": "same results bit for bit; the fold_first / fold_last_apply entry points at the edges"}

    # ---- the same mini-batch with the folds of different layers on K streams (ends and starts of launches overlap) ----
    overlapped = None
    if args.fold_streams > 1:
        hb.use_fold_streams(args.fold_streams)
        one_step(False)
        hb.synchronize()
        t4 = time.perf_counter()
        for _ in range(args.steps):
            one_step(False)
        hb.synchronize()
        ov_ms = (time.perf_counter() - t4) / args.steps * 1e3
        hb.use_fold_streams(1)
        overlapped = {"streams": args.fold_streams, "ms_per_step": round(ov_ms, 3),
                      "value": round(algorithmic_bytes_per_step(w, opt) / (ov_ms * 1e-3) / 1e9, 1), "unit": "GB/s",
                      "note": "layer l folded on stream l mod K; same results bit for bit; each stream would own a gradient "
                              "buffer in the single-buffer layout"}

    # ---- live per-launch timing of the dominant kernel, HIP events on the launch stream ----
    for _ in range(min(2, args.steps)):
        one_step(True)
    hb.synchronize()
    fold_ms = sum(e0.elapsed_time(e1) for e0, e1, _, _ in fold_events)
    fold_bytes = sum(n for _, _, n, _ in fold_events) * (state_bytes(opt) + w.grad_bytes)
    launches = sum(k for _, _, _, k in fold_events)
    achieved = fold_bytes / (fold_ms * 1e-3) / 1e9 if fold_ms > 0 else 0.0

    sb = state_bytes(opt)
    class_bytes = {"decay": sb * w.P, "fold": (sb + w.grad_bytes) * w.P, "update": (8 + sb // 2) * w.P}
    kernel_classes = {}
    for name, pairs in class_events.items():
        ms = sum(a.elapsed_time(b) for a, b in pairs) / max(len(pairs), 1)
        if ms > 0:
            kernel_classes[name] = {"ms": round(ms, 4), "GB/s": round(class_bytes[name] / (ms * 1e-3) / 1e9, 1),
                                    "params_per_s": round(w.P / (ms * 1e-3), 1)}
    if "fold" in kernel_classes:
        kernel_classes["fold"]["us_per_launch"] = round(kernel_classes["fold"]["ms"] * 1e3 / len(w.layers), 2)
        kernel_classes["fold"]["note"] = "one micro-batch's sweep: one launch per layer"
    step_bytes = algorithmic_bytes_per_step(w, opt)
    placement = dict(hb.placement)
    if placement["step_ms"]:        # what the candidates' estimated step times mean in the metric's unit
        est = lambda ms: round(step_bytes / (ms * 1e-3) / 1e9, 1)                                          # noqa: E731
        flat = [ms for row in placement["step_ms"] for ms in row]
        placement["estimated_GB/s"] = {"first_candidate": est(placement["step_ms"][0][0]), "kept": est(min(flat)),
                                       "slowest_candidate": est(max(flat)),
                                       "note": "from the search's own timing (decay + N fold sweeps + update on scratch "
                                               "contents); first_candidate is what a program that does not search gets"}
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    metric = "AdamA fold+apply effective HBM GB/s (algorithmic bytes of decay + N folds + update per second)"
    if opt != "adama":
        metric = f"{opt} variant: " + metric
    op_label = "sgd_fold" if opt == "sgdm" else "fold"
    dom = binding.adama_tuning(op_label, max((w.layer_elems(li) for li in big_layers), default=0))
    out = {
        "metric": metric,
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3),
        "ms_per_step_median": round(median_ms, 3),
        "ms_per_step_trace": trace_ms,
        "arena_placement": placement,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "library_build": binding.adama_build_id(),
        "dtype": "f32",                     # the arithmetic type; gradient storage is config.grad_dtype
        "data": "synthetic",
        "config": {"workload": w.name, "params": w.P, "tensors": len(w.tensors), "layers": len(w.layers),
                   "optimizer": opt, "micro_batches": w.N, "grad_dtype": w.gdtype, "bytes_per_step": step_bytes,
                   "fold_launches_per_step": w.N * len(w.layers)},
        "params_per_s": round(w.P / (ms_per_step * 1e-3), 1),
        "param_folds_per_s": round(w.P * w.N / (ms_per_step * 1e-3), 1),
        "frac_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                     "kernel": f"multi_tensor_kernel<{op_label},{w.gdtype},block={dom['block']},U={dom['groups_per_thread']},policy={dom['policy_bits']},multi-tensor>",
                     "launches_timed": launches,
                     "avg_launch_ms": round(fold_ms / launches, 4) if launches else None,
                     "bytes_per_launch": round(fold_bytes / launches) if launches else None},
        "kernel_classes": kernel_classes,
        "fused_edges": fused,
        "fold_sweep": graph_sweep,
        "overlapped_folds": overlapped,
        "torch_ops_baseline": torch_ops,
        "grad_memory": {"resident_for_timing_bytes": hb.peak_grad_bytes,
                        "adama_peak_bytes_largest_layer": w.largest_layer_elems * w.grad_bytes,
                        "whole_model_bytes": w.P * w.grad_bytes},
    }
    # hardware-counter traffic of the dominant kernel: taken by two rocprofv3 --pmc runs of this command and
    # reduced by bench_traffic.py; quoted only while the library that was profiled is the one loaded now
    traffic_file = os.path.join(ROOT, "profiles", f"traffic_{w.name}.json" if opt != "sgdm" else f"traffic_{w.name}_sgdm.json")
    if os.path.exists(traffic_file):
        with open(traffic_file) as fh:
            tr = json.load(fh)
        if tr.get("build_id") == binding.adama_build_id():
            out["roofline"]["traffic"] = tr.get("bytes_per_launch")
        else:
            out["roofline"]["traffic_note"] = (f"{os.path.basename(traffic_file)} was measured on library build "
                                               f"{tr.get('build_id')}, the loaded one is {binding.adama_build_id()}: not quoted")
    if args.cpu_budget > 0:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_budget, opt)
        out["cpu_baseline_all_cores"] = cpu_baseline_all_cores(w, args.cpu_budget / 2, opt)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
