"""Builds libadama.so for gfx950 with hipcc, in-tree (next to this file)."""
from __future__ import annotations

import hashlib
import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libadama.so")
SOURCES = [os.path.join(PKG, "csrc", "adama.hip")]
HEADERS = [os.path.join(PKG, "csrc", "adama_kernels.hpp"), os.path.join(PKG, "csrc", "adama_index.hpp"),
           os.path.join(ROOT, "include", "adama.h")]
# -ffp-contract=off: the kernels spell out every fused multiply-add they want.
# -fno-slp-vectorize: every wide access is written as a vector type already; the SLP pass only turns
# the scalar table search into a long vector-ALU bit-twiddling sequence.
# Packed-fp32 instructions are disabled on purpose (target feature below).
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off", "-fno-slp-vectorize",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-command-line-argument", "-fPIC", "-shared"]


_ID_MARKER = b"ADAMA_BUILD_ID="


def source_id() -> str:
    """Identifies what a library is built from: the compiler flags and the bytes of every source and header."""
    h = hashlib.sha256(" ".join(HIPCC_FLAGS).encode())
    for p in SOURCES + HEADERS:
        with open(p, "rb") as fh:
            h.update(b"\0" + os.path.basename(p).encode() + b"\0" + fh.read())
    return h.hexdigest()[:16]


def library_id(path: str = LIB) -> str | None:
    """The source_id() a built library carries (the string adama_build_id() returns), read from the file
    without loading it; None if the file is missing or carries none."""
    if not os.path.exists(path):
        return None
    with open(path, "rb") as fh:
        blob = fh.read()
    at = blob.find(_ID_MARKER)
    if at < 0:
        return None
    return blob[at + len(_ID_MARKER): at + len(_ID_MARKER) + 16].decode("ascii", "replace")


def stale() -> bool:
    """True when libadama.so is missing or was built from sources (or flags) other than the present ones.
    Compares contents, not file times, so a copied or checked-out tree is judged correctly."""
    return library_id() != source_id()


OPS = ["decay", "fold", "apply", "fold_first", "fold_last_apply", "rescale_apply", "sgd_decay", "sgd_fold", "sgd_apply",
       "sgd_fold_first", "sgd_fold_last_apply"]


def policy_define(shape: str) -> str:
    """-D option that gives every op's big and huge launches the workgroup shape "BLOCKxGROUPS" (e.g. "128x2"),
    unbounded residency, the decay's launch-length limit kept: for A/B builds of the launch policy."""
    block, groups = (int(x) for x in shape.lower().split("x"))
    rows = ", ".join("{{256, 1, 0}, {%d, %d, 0}, {%d, %d, 0}, %s}" % (block, groups, block, groups,
                                                                    "ADAMA_DECAY_LAUNCH_CAP" if op == "decay" else "0")
                     for op in OPS)
    return "-DADAMA_POLICY_TABLE={" + rows + "}"


def build_libadama(verbose: bool = False, out: str | None = None, extra_flags: list | None = None) -> str:
    """Builds the library next to this file, or a variant (other -D options) at `out`; a variant carries the
    build id "variant" so that it is never mistaken for the library of the sources as they stand."""
    target = out or LIB
    tmp = target + f".tmp{os.getpid()}"
    build_id = source_id() if not extra_flags and out is None else "variant"
    cmd = ["hipcc", *HIPCC_FLAGS, *(extra_flags or []), f'-DADAMA_BUILD_ID="{build_id}"', "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(PKG, "csrc"), "-o", tmp, *SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "packed-fp32-ops"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    os.replace(tmp, target)
    return target


if __name__ == "__main__":
    import argparse

    ap = argparse.ArgumentParser(description="Build libadama.so, or a variant for A/B measurements (bench_ab.py).")
    ap.add_argument("--out", default=None, help="write the library here instead of next to the package")
    ap.add_argument("--shape", default=None, help='give every op\'s big and huge launches this workgroup shape, e.g. "128x2"')
    ap.add_argument("--define", action="append", default=[], help="extra NAME=VALUE preprocessor definition (repeatable)")
    a = ap.parse_args()
    flags = [f"-D{d}" for d in a.define] + ([policy_define(a.shape)] if a.shape else [])
    print(build_libadama(verbose=True, out=a.out, extra_flags=flags))
