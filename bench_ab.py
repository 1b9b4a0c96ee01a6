#!/usr/bin/env python3
"""In-process A/B of libadama builds and launch policies on GPT-2-XL-shaped state (one MI355X).

    python -m paper_2305_19982_amd.build --out /tmp/v128x2.so --shape 128x2      # a variant build (any number of them)
    python bench_ab.py --libraries paper_2305_19982_amd/libadama.so,/tmp/v128x2.so \\
                       --ops fold,decay,apply,fold32,fold_last_apply,rescale --residency 0,12,8,4 [--rounds 2] [--zero]

State: 48 transformer blocks of 12 tensors (30,740,800 elements each; theta, m, v float32, gradients bf16) with
realistic contents (--zero: all-zero arrays, to show how much the contents matter).  Every (library, op, residency
bound) combination is timed with HIP events over three back-to-back passes, all in this one process and interleaved,
so that the figures are comparable (processes and boxes differ from each other by 1..3 %).  The residency bound is
set through adama_debug_set_residency (0 = unbounded, -1 = the library's own policy).  Prints one line per (op, library)
and, last, one JSON line with all figures (GB/s of algorithmic bytes).

Ops: fold (12-tensor launches, bf16), single (one 30.7 M-element tensor per launch), fold32 (fp32 gradients, 16-tensor
BERT-Large-shaped launches of 12.6 M elements), fold_first, fold_last_apply, decay, apply, rescale (whole-state lists),
sgd_fold, sgd_fold_first, sgd_fold_last_apply, sgd_decay, sgd_apply, and fold@<elements>, fold_first@<elements>,
sgd_fold@<elements>, sgd_fold_first@<elements> (one-tensor bf16 launches of that many elements marching through the arena: the launch-length dependence).  A library built from an older revision of the sources
(without adama_debug_set_residency) can be timed with --residency -1.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

BLOCK12 = [1600, 1600, 7680000, 4800, 2560000, 1600, 1600, 1600, 10240000, 6400, 10240000, 1600]      # a GPT-2-XL block
BLOCK16 = [1024 * 1024, 1024] * 4 + [1024, 1024, 1024 * 4096, 4096, 4096 * 1024, 1024, 1024, 1024]    # a BERT-Large layer
LAYERS = 48
BYTES = {"fold": 18, "single": 18, "fold32": 20, "fold_first": 18, "fold_last_apply": 26, "decay": 16, "apply": 16,
         "rescale": 24, "sgd_fold": 10, "sgd_fold_first": 10, "sgd_fold_last_apply": 18, "sgd_decay": 8, "sgd_apply": 12}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--libraries", default=None, help="comma-separated library files (default: the package's own build)")
    ap.add_argument("--ops", default="fold,decay,apply")
    ap.add_argument("--residency", default="-1", help="comma-separated workgroups per compute unit; 0 unbounded, -1 library policy")
    ap.add_argument("--rounds", type=int, default=2)
    ap.add_argument("--zero", action="store_true", help="all-zero arrays instead of realistic contents")
    args = ap.parse_args()

    import torch

    from paper_2305_19982_amd import binding as B

    libs = args.libraries.split(",") if args.libraries else [B.library_path()]
    ops = args.ops.split(",")
    bounds = [int(x) for x in args.residency.split(",")]
    per_layer = sum(BLOCK12)
    P = per_layer * LAYERS
    dev = "cuda:0"
    stream = torch.cuda.Stream(device=dev)
    with torch.cuda.stream(stream):
        theta = torch.zeros(P, dtype=torch.float32, device=dev)
        m = torch.zeros(P, dtype=torch.float32, device=dev)
        v = torch.zeros(P, dtype=torch.float32, device=dev)
        g = torch.zeros(P, dtype=torch.float32, device=dev)        # read as bf16 (first half) or as fp32 gradients
        if not args.zero:
            theta.normal_(0, 0.02)
            g.view(torch.bfloat16).normal_(0, 1e-3)
            m.normal_(0, 1e-4)
            v.uniform_(1e-9, 1e-7)
    stream.synchronize()
    sh = stream.cuda_stream
    tp, mp, vp, gp = theta.data_ptr(), m.data_ptr(), v.data_ptr(), g.data_ptr()
    fold_l, upd_l, sgd_l, state, sgd_state, off = [], [], [], [], [], 0
    for _ in range(LAYERS):
        ef, eu, es = [], [], []
        for n in BLOCK12:
            ef.append((mp + 4 * off, vp + 4 * off, gp + 2 * off, n))
            eu.append((tp + 4 * off, mp + 4 * off, vp + 4 * off, gp + 2 * off, n))
            es.append((tp + 4 * off, mp + 4 * off, gp + 2 * off, n))
            state.append((tp + 4 * off, mp + 4 * off, vp + 4 * off, n))
            sgd_state.append((tp + 4 * off, mp + 4 * off, None, n))
            off += n
        fold_l.append(B.tensor_list(ef))
        upd_l.append(B.update_list(eu))
        sgd_l.append(B.sgdm_list(es))
    single_l = [B.tensor_list([(mp + 4 * li * per_layer, vp + 4 * li * per_layer, gp + 2 * li * per_layer, per_layer)])
                for li in range(LAYERS)]
    state_l, sgd_state_l = B.state_list(state), B.sgdm_list(sgd_state)
    per16 = sum(BLOCK16)
    layers16 = P // per16
    fold32_l, off = [], 0
    for _ in range(layers16):
        e = []
        for n in BLOCK16:
            e.append((mp + 4 * off, vp + 4 * off, gp + 4 * off, n))
            off += n
        fold32_l.append(B.tensor_list(e))

    def load(path: str) -> ctypes.CDLL:
        lib = ctypes.CDLL(path)
        vpt, dbl, i32, i64 = ctypes.c_void_p, ctypes.c_double, ctypes.c_int, ctypes.c_longlong
        tl, ul, sl, gl = (ctypes.POINTER(t) for t in (B.adama_tensor, B.adama_update_tensor, B.adama_state, B.adama_sgdm_tensor))
        lib.adama_fold_multi.argtypes = [tl, i32, i32, i32, dbl, dbl, vpt]
        lib.adama_fold_first_multi.argtypes = [tl, i32, i32, i32, dbl, dbl, vpt]
        lib.adama_fold_last_apply_multi.argtypes = [ul, i32, i32, i32, dbl, dbl, dbl, dbl, i64, vpt]
        lib.adama_begin_step_multi.argtypes = [sl, i32, dbl, dbl, vpt]
        lib.adama_apply_multi.argtypes = [sl, i32, dbl, dbl, dbl, dbl, i64, vpt]
        lib.adama_rescale_apply_multi.argtypes = [sl, i32, dbl, dbl, dbl, dbl, dbl, dbl, i64, vpt]
        lib.adama_sgdm_begin_step_multi.argtypes = [gl, i32, dbl, vpt]
        lib.adama_sgdm_fold_multi.argtypes = [gl, i32, i32, i32, vpt, vpt]
        lib.adama_sgdm_fold_first_multi.argtypes = [gl, i32, i32, i32, dbl, vpt, vpt]
        lib.adama_sgdm_apply_multi.argtypes = [gl, i32, dbl, vpt, vpt]
        lib.adama_sgdm_fold_last_apply_multi.argtypes = [gl, i32, i32, i32, dbl, vpt, vpt]
        if hasattr(lib, "adama_debug_set_residency"):
            lib.adama_debug_set_residency.argtypes = [i32, i32, i32]
            lib.adama_debug_set_residency.restype = None
        elif bounds != [-1]:
            raise SystemExit(f"{path} has no adama_debug_set_residency: time it with --residency -1")
        return lib

    def timed(fn, reps: int = 3) -> float:
        fn()
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) / reps

    back = range(LAYERS - 1, -1, -1)
    sized = {}

    def run(lib, op: str) -> float:
        """GB/s of one pass of `op` over the whole state."""
        if op == "fold":
            fn, elems = (lambda: [lib.adama_fold_multi(fold_l[li], 12, B.BF16, 16, 0.9, 0.999, sh) for li in back]), P
        elif op == "single":
            fn, elems = (lambda: [lib.adama_fold_multi(single_l[li], 1, B.BF16, 16, 0.9, 0.999, sh) for li in back]), P
        elif op == "fold32":
            fn = lambda: [lib.adama_fold_multi(fold32_l[li], 16, B.F32, 8, 0.9, 0.999, sh) for li in range(layers16 - 1, -1, -1)]  # noqa: E731
            elems = per16 * layers16
        elif op == "fold_first":
            fn, elems = (lambda: [lib.adama_fold_first_multi(fold_l[li], 12, B.BF16, 16, 0.9, 0.999, sh) for li in back]), P
        elif op == "fold_last_apply":
            fn = lambda: [lib.adama_fold_last_apply_multi(upd_l[li], 12, B.BF16, 16, 1e-3, 1e-8, 0.9, 0.999, 3, sh) for li in back]  # noqa: E731
            elems = P
        elif op == "decay":
            fn, elems = (lambda: lib.adama_begin_step_multi(state_l, len(state_l), 0.9, 0.999, sh)), P
        elif op == "apply":
            fn, elems = (lambda: lib.adama_apply_multi(state_l, len(state_l), 1e-3, 1e-8, 0.9, 0.999, 3, sh)), P
        elif op == "rescale":
            fn, elems = (lambda: lib.adama_rescale_apply_multi(state_l, len(state_l), 1.0, 1.0, 1e-3, 1e-8, 0.9, 0.999, 3, sh)), P
        elif op == "sgd_fold":
            fn, elems = (lambda: [lib.adama_sgdm_fold_multi(sgd_l[li], 12, B.BF16, 16, None, sh) for li in back]), P
        elif op == "sgd_fold_first":
            fn, elems = (lambda: [lib.adama_sgdm_fold_first_multi(sgd_l[li], 12, B.BF16, 16, 0.9, None, sh) for li in back]), P
        elif op == "sgd_fold_last_apply":
            fn, elems = (lambda: [lib.adama_sgdm_fold_last_apply_multi(sgd_l[li], 12, B.BF16, 16, 0.05, None, sh) for li in back]), P
        elif op == "sgd_decay":
            fn, elems = (lambda: lib.adama_sgdm_begin_step_multi(sgd_state_l, len(sgd_state_l), 0.9, sh)), P
        elif op == "sgd_apply":
            fn, elems = (lambda: lib.adama_sgdm_apply_multi(sgd_state_l, len(sgd_state_l), 0.05, None, sh)), P
        elif "@" in op and op.split("@")[0] in ("fold", "fold_first", "sgd_fold", "sgd_fold_first"):
            kind, n = op.split("@")[0], int(op.split("@")[1]) // 4 * 4
            cnt = min(P // n, 400)
            if op not in sized:
                if kind.startswith("sgd_"):
                    sized[op] = [B.sgdm_list([(tp + 4 * i * n, mp + 4 * i * n, gp + 2 * i * n, n)]) for i in range(cnt)]
                else:
                    sized[op] = [B.tensor_list([(mp + 4 * i * n, vp + 4 * i * n, gp + 2 * i * n, n)]) for i in range(cnt)]
            if kind == "fold":
                fn = lambda: [lib.adama_fold_multi(l, 1, B.BF16, 16, 0.9, 0.999, sh) for l in sized[op]]  # noqa: E731
            elif kind == "fold_first":
                fn = lambda: [lib.adama_fold_first_multi(l, 1, B.BF16, 16, 0.9, 0.999, sh) for l in sized[op]]  # noqa: E731
            elif kind == "sgd_fold":
                fn = lambda: [lib.adama_sgdm_fold_multi(l, 1, B.BF16, 16, None, sh) for l in sized[op]]  # noqa: E731
            else:
                fn = lambda: [lib.adama_sgdm_fold_first_multi(l, 1, B.BF16, 16, 0.9, None, sh) for l in sized[op]]  # noqa: E731
            return (10 if kind.startswith("sgd_") else 18) * n * cnt / timed(fn) / 1e6
        else:
            raise SystemExit(f"unknown op {op!r}")
        return BYTES[op] * elems / timed(fn) / 1e6

    handles = {os.path.basename(p): load(p) for p in libs}
    results = {}
    for rnd in range(args.rounds):
        for op in ops:
            for name, lib in handles.items():
                row = []
                for r in bounds:
                    if hasattr(lib, "adama_debug_set_residency"):
                        for o in range(11):
                            for cls in (1, 2):
                                lib.adama_debug_set_residency(o, cls, r)
                    gbs = run(lib, op)
                    key = f"{op}|{name}|r{r}"
                    results[key] = max(results.get(key, 0.0), round(gbs, 1))
                    row.append(f"r{r}:{gbs:6.0f}")
                print(f"{op:20s} {name:24s} " + "  ".join(row), flush=True)
    print(json.dumps({"bench_ab": results, "contents": "zero" if args.zero else "realistic", "unit": "GB/s"}), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
