"""Python front end of the seeded synthetic-input generator (synth_gen.h).

Inputs only: gradient-like and weight-like values.  None of the optimizer's
arithmetic lives here, and neither the oracle nor the HIP library imports it;
tests, the harness and the benchmark feed both sides from it.

Host and device builds of the generator produce identical bits for the same
(spec, element index), so a slice of what the device wrote into a gradient
buffer can be regenerated on the host for the oracle without reading it back.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
HOST_LIB = os.path.join(_HERE, "libsynth_host.so")
DEVICE_LIB = os.path.join(_HERE, "libsynth_device.so")

F32, BF16, F16 = 0, 1, 2
DTYPE_ID = {"f32": F32, "bf16": BF16, "f16": F16}
DTYPE_BYTES = {"f32": 4, "bf16": 2, "f16": 2}
_MASK = (1 << 64) - 1


class _Spec(ctypes.Structure):
    _fields_ = [("key", ctypes.c_uint64), ("sigma", ctypes.c_float), ("outlier_scale", ctypes.c_float),
                ("t_zero", ctypes.c_uint32), ("t_outlier", ctypes.c_uint32), ("t_sub", ctypes.c_uint32),
                ("reserved", ctypes.c_uint32)]


@dataclass(frozen=True)
class Spec:
    """One stream of synthetic values (see synth_gen.h for the value classes)."""
    key: int
    sigma: float
    p_zero: float = 0.0
    p_outlier: float = 0.0
    outlier_scale: float = 10.0
    p_sub: float = 0.0

    def c_struct(self) -> _Spec:
        thr = lambda p: min(int(round(p * 2.0 ** 32)), 2 ** 32 - 1)   # noqa: E731
        return _Spec(self.key & _MASK, self.sigma, self.outlier_scale, thr(self.p_zero),
                     thr(self.p_outlier), thr(self.p_sub), 0)


def mix64(z: int) -> int:
    z &= _MASK
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK
    return z ^ (z >> 31)


def stream_key(seed: int, *ids: int) -> int:
    """Key of the stream named by (seed, ids...): a chain of 64-bit mixes."""
    k = mix64(seed + 0x632BE59BD9B4E019)
    for i in ids:
        k = mix64(k ^ mix64((int(i) + 0x9E3779B97F4A7C15) & _MASK))
    return k


def unit_uniform(key: int) -> float:
    """A uniform in [0,1) derived from a key (host side only, e.g. per-tensor sigma draws)."""
    return (mix64(key ^ 0xA0761D6478BD642F) >> 11) * 2.0 ** -53


def log_uniform(key: int, lo: float, hi: float) -> float:
    return math.exp(math.log(lo) + unit_uniform(key) * (math.log(hi) - math.log(lo)))


def build_host(force: bool = False) -> str:
    src = os.path.join(_HERE, "synth_host.c")
    hdr = os.path.join(_HERE, "synth_gen.h")
    if (not force and os.path.exists(HOST_LIB)
            and os.path.getmtime(HOST_LIB) >= max(os.path.getmtime(src), os.path.getmtime(hdr))):
        return HOST_LIB
    tmp = HOST_LIB + f".tmp{os.getpid()}"
    subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-std=c11", "-fPIC",
                    "-shared", "-o", tmp, src, "-lm"], check=True)
    os.replace(tmp, HOST_LIB)
    return HOST_LIB


def build_device() -> str:
    src = os.path.join(_HERE, "synth_device.hip")
    tmp = DEVICE_LIB + f".tmp{os.getpid()}"
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-O3", "-ffp-contract=off",
                    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                    "-fPIC", "-shared", "-o", tmp, src], check=True)
    os.replace(tmp, DEVICE_LIB)
    return DEVICE_LIB


_host = None
_device = None


def _host_lib():
    global _host
    if _host is None:
        _host = ctypes.CDLL(build_host())
        _host.synth_fill_host.restype = ctypes.c_int
        _host.synth_fill_host.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64,
                                          ctypes.POINTER(_Spec)]
        _host.synth_mix64_host.restype = ctypes.c_uint64
        _host.synth_mix64_host.argtypes = [ctypes.c_uint64]
    return _host


def _device_lib():
    global _device
    if _device is None:
        if not os.path.exists(DEVICE_LIB):
            build_device()
        _device = ctypes.CDLL(DEVICE_LIB)
        _device.synth_fill_device.restype = ctypes.c_int
        _device.synth_fill_device.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64,
                                              ctypes.POINTER(_Spec), ctypes.c_void_p]
        _device.synth_copy_device.restype = ctypes.c_int
        _device.synth_copy_device.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p]
        _device.synth_stream_probe.restype = ctypes.c_int
        _device.synth_stream_probe.argtypes = [ctypes.c_int, ctypes.c_int] + [ctypes.c_void_p] * 5 + [ctypes.c_uint64,
                                                                                                    ctypes.c_void_p]
        _device.synth_stream_probe_shape.restype = ctypes.c_int
        _device.synth_stream_probe_shape.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_uint] + [
            ctypes.c_void_p] * 5 + [ctypes.c_uint64, ctypes.c_void_p]
        _device.synth_stream_probe_persistent.restype = ctypes.c_int
        _device.synth_stream_probe_persistent.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_uint] + [
            ctypes.c_void_p] * 5 + [ctypes.c_uint64, ctypes.c_void_p]
        _device.synth_cache_policy_probe.restype = ctypes.c_int
        _device.synth_cache_policy_probe.argtypes = [ctypes.c_int] * 3 + [ctypes.c_void_p] * 4 + [ctypes.c_uint64, ctypes.c_void_p]
        _device.synth_stream_probe_bytes.restype = ctypes.c_int
        _device.synth_stream_probe_bytes.argtypes = [ctypes.c_int]
    return _device


# Traffic-mix probe (synth_device.hip): streams with the access mix of the optimizer's kernels, no arithmetic.
PROBE_MODES = {"read_g16_m_v": 0, "write_m_v": 1, "fold_mix_g16": 2, "fold_mix_g32": 3, "decay_mix": 4,
               "update_mix": 5, "rescale_mix": 6, "read_3xf32": 7}


CACHE_POLICIES = {"": 0, "nt": 1, "sc0": 2, "sc1": 3, "sc0 sc1": 4, "sc0 sc1 nt": 5, "sc0 nt": 6, "sc1 nt": 7}


def cache_policy_probe(load_policy: str, store_policy: str, what: str, g: int, a0: int, a1: int, sink: int, n: int,
                       stream: int) -> None:
    """Enqueue one launch of the fold's access mix ("mix", 18 B/element), its reads ("read", 10) or its writes
    ("write", 8) over n elements (a multiple of 512) with the given modifiers on the loads and on the stores."""
    rc = _device_lib().synth_cache_policy_probe(CACHE_POLICIES[load_policy], CACHE_POLICIES[store_policy],
                                                {"mix": 0, "read": 1, "write": 2}[what], ctypes.c_void_p(g),
                                                ctypes.c_void_p(a0), ctypes.c_void_p(a1), ctypes.c_void_p(sink), n,
                                                ctypes.c_void_p(stream))
    if rc:
        raise RuntimeError(f"synth_cache_policy_probe({load_policy!r}, {store_policy!r}, {what}, n={n}) failed ({rc})")


def stream_probe_bytes(mode: str) -> int:
    return int(_device_lib().synth_stream_probe_bytes(PROBE_MODES[mode]))


def stream_probe(mode: str, block: int, g: int, a0: int, a1: int, a2: int, sink: int, n: int, stream: int,
                 lds_bytes: int = 0, groups: int = 1) -> None:
    """Enqueue one probe launch over n elements (a multiple of block*4*groups) of device arrays at the given
    addresses; lds_bytes of unused LDS per workgroup cap the number of workgroups resident on a compute unit."""
    rc = _device_lib().synth_stream_probe_shape(PROBE_MODES[mode], block, groups, lds_bytes, ctypes.c_void_p(g),
                                                ctypes.c_void_p(a0), ctypes.c_void_p(a1), ctypes.c_void_p(a2),
                                                ctypes.c_void_p(sink), n, ctypes.c_void_p(stream))
    if rc:
        raise RuntimeError(f"synth_stream_probe({mode}, block={block}, groups={groups}, lds={lds_bytes}, n={n}) failed ({rc})")


def stream_probe_persistent(mode: str, block: int, grid: int, g: int, a0: int, a1: int, a2: int, sink: int, n: int,
                            stream: int) -> None:
    """The same streams from a persistent grid: workgroup w of `grid` takes chunks w, w + grid, ... of block*4 elements."""
    rc = _device_lib().synth_stream_probe_persistent(PROBE_MODES[mode], block, grid, ctypes.c_void_p(g),
                                                     ctypes.c_void_p(a0), ctypes.c_void_p(a1), ctypes.c_void_p(a2),
                                                     ctypes.c_void_p(sink), n, ctypes.c_void_p(stream))
    if rc:
        raise RuntimeError(f"synth_stream_probe_persistent({mode}, block={block}, grid={grid}, n={n}) failed ({rc})")


def copy_device(dst: int, src: int, nbytes: int, stream: int) -> None:
    """Enqueue a plain device-to-device copy kernel (reference traffic for counter calibration)."""
    rc = _device_lib().synth_copy_device(ctypes.c_void_p(dst), ctypes.c_void_p(src), nbytes, ctypes.c_void_p(stream))
    if rc:
        raise RuntimeError(f"synth_copy_device failed ({rc})")


def fill_host(spec: Spec, dtype: str, n: int, first: int = 0) -> np.ndarray:
    """Elements first .. first+n-1 of the stream: float32 array, or uint16 bit patterns for bf16/f16."""
    out = np.empty(n, dtype=np.float32 if dtype == "f32" else np.uint16)
    cs = spec.c_struct()
    rc = _host_lib().synth_fill_host(out.ctypes.data, DTYPE_ID[dtype], n, first, ctypes.byref(cs))
    if rc:
        raise RuntimeError(f"synth_fill_host failed ({rc})")
    return out


def fill_device(ptr: int, spec: Spec, dtype: str, n: int, stream: int, first: int = 0) -> None:
    """Enqueue a fill of device memory at `ptr` with elements first .. first+n-1 on HIP stream `stream`."""
    cs = spec.c_struct()
    rc = _device_lib().synth_fill_device(ctypes.c_void_p(ptr), DTYPE_ID[dtype], n, first, ctypes.byref(cs),
                                         ctypes.c_void_p(stream))
    if rc:
        raise RuntimeError(f"synth_fill_device failed ({rc})")


def widen(arr: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float64 value of stored gradients, by library conversions (for checks, not for the oracle)."""
    if dtype == "f32":
        return arr.astype(np.float64)
    if dtype == "f16":
        return arr.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (arr.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    raise ValueError(dtype)
