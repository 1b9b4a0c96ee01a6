"""ctypes front end of the fp64 AdamA oracle (oracle/adama_oracle.c).

TEST INFRASTRUCTURE, NOT THE PRODUCT.  Every function below only marshals numpy
arrays into the C loops, which follow Alg. 1, Alg. 2 and Sec. 3.3 of the paper
statement by statement.  Nothing here imports or is imported by the HIP
package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adama_oracle.c")
_LIB = os.path.join(_HERE, "libadama_oracle.so")
# -ffp-contract=off: gcc would otherwise fuse a*b+c into one rounding on
# targets with FMA, and the N=1 identity with textbook Adam is checked bit for bit.
_CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c11", "-fPIC", "-shared"]

_lock = threading.Lock()
_lib = None

_dp = ctypes.POINTER(ctypes.c_double)


def lib_path() -> str:
    return _LIB


def build(force: bool = False, src: str | None = None, out: str | None = None) -> str:
    """Compile the oracle with gcc.  `src`/`out` let tests compile altered copies."""
    src = src or _SRC
    out = out or _LIB
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(src):
        return out
    tmp = out + f".tmp{os.getpid()}"
    subprocess.run(["gcc", *_CFLAGS, "-o", tmp, src, "-lm"], check=True)
    os.replace(tmp, out)
    return out


def load(path: str | None = None) -> ctypes.CDLL:
    """Load a compiled oracle library and declare its prototypes."""
    lib = ctypes.CDLL(path or build())
    sz, dbl, i32, i64 = ctypes.c_size_t, ctypes.c_double, ctypes.c_int, ctypes.c_longlong
    vp = ctypes.c_void_p
    lib.adama_oracle_bf16_to_f64.restype = dbl
    lib.adama_oracle_bf16_to_f64.argtypes = [ctypes.c_uint16]
    lib.adama_oracle_f16_to_f64.restype = dbl
    lib.adama_oracle_f16_to_f64.argtypes = [ctypes.c_uint16]
    lib.adama_oracle_begin_step.restype = None
    lib.adama_oracle_begin_step.argtypes = [_dp, _dp, sz, dbl, dbl]
    for name in ("adama_oracle_fold", "adama_oracle_fold_f32", "adama_oracle_fold_bf16",
                 "adama_oracle_fold_f16"):
        fn = getattr(lib, name)
        fn.restype = None
        fn.argtypes = [_dp, _dp, vp, sz, i32, dbl, dbl]
    lib.adama_oracle_apply.restype = None
    lib.adama_oracle_apply.argtypes = [_dp, _dp, _dp, sz, dbl, dbl, dbl, dbl, i64]
    lib.adama_oracle_alg1_step.restype = None
    lib.adama_oracle_alg1_step.argtypes = [_dp, _dp, _dp, _dp, sz, i32, i32, dbl, dbl, dbl, dbl, i64]
    lib.adama_oracle_ddp_combine.restype = None
    lib.adama_oracle_ddp_combine.argtypes = [_dp, _dp, _dp, _dp, sz, i32]
    lib.adama_oracle_widen.restype = i32
    lib.adama_oracle_widen.argtypes = [_dp, vp, sz, i32]
    lib.adama_oracle_fold_scaled.restype = None
    lib.adama_oracle_fold_scaled.argtypes = [_dp, _dp, _dp, sz, i32, dbl, dbl, dbl]
    lib.adama_oracle_apply_adamw.restype = None
    lib.adama_oracle_apply_adamw.argtypes = [_dp, _dp, _dp, sz, dbl, dbl, dbl, dbl, i64, dbl]
    lib.adama_oracle_sgdm_begin_step.restype = None
    lib.adama_oracle_sgdm_begin_step.argtypes = [_dp, sz, dbl]
    lib.adama_oracle_sgdm_fold.restype = None
    lib.adama_oracle_sgdm_fold.argtypes = [_dp, _dp, sz, i32, dbl]
    lib.adama_oracle_sgdm_apply.restype = None
    lib.adama_oracle_sgdm_apply.argtypes = [_dp, _dp, sz, dbl, dbl]
    return lib


def _get() -> ctypes.CDLL:
    global _lib
    with _lock:
        if _lib is None:
            _lib = load()
        return _lib


def _f64(a: np.ndarray, name: str) -> ctypes.POINTER(ctypes.c_double):
    if not (isinstance(a, np.ndarray) and a.dtype == np.float64 and a.flags.c_contiguous
            and a.flags.writeable):
        raise TypeError(f"{name}: need a writable C-contiguous float64 ndarray")
    return a.ctypes.data_as(_dp)


def _f64_ro(a: np.ndarray, name: str) -> ctypes.POINTER(ctypes.c_double):
    if not (isinstance(a, np.ndarray) and a.dtype == np.float64 and a.flags.c_contiguous):
        raise TypeError(f"{name}: need a C-contiguous float64 ndarray")
    return a.ctypes.data_as(_dp)


def bf16_to_f64(bits: int, lib: ctypes.CDLL | None = None) -> float:
    return float((lib or _get()).adama_oracle_bf16_to_f64(int(bits)))


def f16_to_f64(bits: int, lib: ctypes.CDLL | None = None) -> float:
    return float((lib or _get()).adama_oracle_f16_to_f64(int(bits)))


def begin_step(m, v, beta1: float, beta2: float, lib=None) -> None:
    """Alg. 2: m <- beta1 m, v <- beta2 v (in place)."""
    assert m.size == v.size
    (lib or _get()).adama_oracle_begin_step(_f64(m, "m"), _f64(v, "v"), m.size, beta1, beta2)


def fold(m, v, grad, N: int, beta1: float, beta2: float, gdtype: str | None = None, lib=None) -> None:
    """Alg. 2 inner body for one gradient tensor (in place on m, v).

    grad: float64, or float32, or uint16 holding bf16 / fp16 bit patterns
    (then `gdtype` is "bf16" or "f16").
    """
    lib = lib or _get()
    assert m.size == v.size == grad.size
    if N < 1:
        raise ValueError("N must be >= 1")
    if not grad.flags.c_contiguous:
        raise TypeError("grad must be C-contiguous")
    gp = ctypes.c_void_p(grad.ctypes.data)
    if grad.dtype == np.float64 and gdtype in (None, "f64"):
        fn = lib.adama_oracle_fold
    elif grad.dtype == np.float32 and gdtype in (None, "f32"):
        fn = lib.adama_oracle_fold_f32
    elif grad.dtype == np.uint16 and gdtype == "bf16":
        fn = lib.adama_oracle_fold_bf16
    elif grad.dtype == np.uint16 and gdtype == "f16":
        fn = lib.adama_oracle_fold_f16
    elif grad.dtype == np.float16 and gdtype in (None, "f16"):
        fn = lib.adama_oracle_fold_f16
    else:
        raise TypeError(f"unsupported gradient dtype {grad.dtype} / {gdtype}")
    fn(_f64(m, "m"), _f64(v, "v"), gp, m.size, int(N), beta1, beta2)


def apply(theta, m, v, lr: float, eps: float, beta1: float, beta2: float, t: int, lib=None) -> None:
    """Alg. 2 Update: bias-corrected parameter step (in place on theta), t >= 1."""
    assert theta.size == m.size == v.size
    if t < 1:
        raise ValueError("t must be >= 1")
    (lib or _get()).adama_oracle_apply(_f64(theta, "theta"), _f64_ro(m, "m"), _f64_ro(v, "v"),
                                       theta.size, lr, eps, beta1, beta2, int(t))


def alg1_step(theta, m, v, grads, variant: str, lr, eps, beta1, beta2, t: int, lib=None) -> None:
    """Alg. 1 closed form over one mini-batch; grads is [N, n] raw micro-batch gradients.

    variant "adam": v uses (sum_i g_i)^2;  variant "adama": v uses sum_i g_i^2.
    """
    N, n = grads.shape
    assert theta.size == m.size == v.size == n
    (lib or _get()).adama_oracle_alg1_step(
        _f64(theta, "theta"), _f64(m, "m"), _f64(v, "v"), _f64_ro(grads, "grads"), n, N,
        {"adam": 0, "adama": 1}[variant], lr, eps, beta1, beta2, int(t))


def ddp_combine(m_ranks, v_ranks, lib=None):
    """Sec. 3.3: m = sum_r m_r / M, v = sum_r v_r / M^2 from [M, n] device-local states."""
    M, n = m_ranks.shape
    m_out = np.empty(n, dtype=np.float64)
    v_out = np.empty(n, dtype=np.float64)
    (lib or _get()).adama_oracle_ddp_combine(_f64(m_out, "m"), _f64(v_out, "v"),
                                             _f64_ro(m_ranks, "m_ranks"),
                                             _f64_ro(v_ranks, "v_ranks"), n, M)
    return m_out, v_out


def widen(grad: np.ndarray, gdtype: str | None = None, lib=None) -> np.ndarray:
    """Exact float64 copy of a stored gradient: float32, float16, or uint16 bits ("bf16"/"f16")."""
    grad = np.ascontiguousarray(grad).reshape(-1)
    if grad.dtype == np.float64 and gdtype in (None, "f64"):
        return grad.copy()
    if grad.dtype == np.float32 and gdtype in (None, "f32"):
        code = 0
    elif grad.dtype == np.uint16 and gdtype == "bf16":
        code = 1
    elif (grad.dtype == np.uint16 and gdtype == "f16") or (grad.dtype == np.float16 and gdtype in (None, "f16")):
        code = 2
    else:
        raise TypeError(f"unsupported gradient dtype {grad.dtype} / {gdtype}")
    out = np.empty(grad.size, dtype=np.float64)
    rc = (lib or _get()).adama_oracle_widen(_f64(out, "out"), ctypes.c_void_p(grad.ctypes.data), grad.size, code)
    assert rc == 0
    return out


def fold_scaled(m, v, grad, N: int, beta1: float, beta2: float, grad_scale: float, gdtype: str | None = None,
                lib=None) -> None:
    """Fold of a gradient taken on a scaled loss: the gradient is grad * grad_scale (in place on m, v)."""
    assert m.size == v.size == grad.size
    if N < 1:
        raise ValueError("N must be >= 1")
    g64 = widen(grad, gdtype, lib=lib)
    (lib or _get()).adama_oracle_fold_scaled(_f64(m, "m"), _f64(v, "v"), _f64_ro(g64, "grad"), m.size, int(N),
                                             beta1, beta2, grad_scale)


def apply_adamw(theta, m, v, lr, eps, beta1, beta2, t: int, weight_decay: float, lib=None) -> None:
    """Update with decoupled weight decay (in place on theta), t >= 1."""
    assert theta.size == m.size == v.size
    if t < 1:
        raise ValueError("t must be >= 1")
    (lib or _get()).adama_oracle_apply_adamw(_f64(theta, "theta"), _f64_ro(m, "m"), _f64_ro(v, "v"), theta.size,
                                             lr, eps, beta1, beta2, int(t), weight_decay)


def sgdm_begin_step(b, mu: float, lib=None) -> None:
    """Momentum SGD, once per mini-batch: b <- mu b (in place)."""
    (lib or _get()).adama_oracle_sgdm_begin_step(_f64(b, "b"), b.size, mu)


def sgdm_fold(b, grad, N: int, grad_scale: float = 1.0, gdtype: str | None = None, lib=None) -> None:
    """Momentum SGD, per layer per micro-batch: b <- b + grad_scale * grad / N (in place)."""
    assert b.size == grad.size
    if N < 1:
        raise ValueError("N must be >= 1")
    g64 = widen(grad, gdtype, lib=lib)
    (lib or _get()).adama_oracle_sgdm_fold(_f64(b, "b"), _f64_ro(g64, "grad"), b.size, int(N), grad_scale)


def sgdm_apply(theta, b, lr: float, weight_decay: float = 0.0, lib=None) -> None:
    """Momentum SGD, once per mini-batch: theta <- theta - lr*weight_decay*theta - lr*b (in place)."""
    assert theta.size == b.size
    (lib or _get()).adama_oracle_sgdm_apply(_f64(theta, "theta"), _f64_ro(b, "b"), theta.size, lr, weight_decay)


class OracleState:
    """theta, m, v in fp64 for a list of tensors plus the step counter t (Alg. 2 init)."""

    def __init__(self, theta0: list[np.ndarray], lib=None):
        self.lib = lib
        self.theta = [np.ascontiguousarray(x, dtype=np.float64).reshape(-1).copy() for x in theta0]
        self.m = [np.zeros_like(x) for x in self.theta]
        self.v = [np.zeros_like(x) for x in self.theta]
        self.t = 0

    def begin_step(self, beta1: float, beta2: float) -> None:
        self.t += 1
        for m, v in zip(self.m, self.v):
            begin_step(m, v, beta1, beta2, lib=self.lib)

    def fold(self, idx: int, grad: np.ndarray, N: int, beta1: float, beta2: float,
             gdtype: str | None = None) -> None:
        fold(self.m[idx], self.v[idx], np.ascontiguousarray(grad).reshape(-1), N, beta1, beta2,
             gdtype=gdtype, lib=self.lib)

    def apply(self, lr: float, eps: float, beta1: float, beta2: float) -> None:
        for th, m, v in zip(self.theta, self.m, self.v):
            apply(th, m, v, lr, eps, beta1, beta2, self.t, lib=self.lib)
