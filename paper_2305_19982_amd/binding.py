"""Thin ctypes binding of libadama's C ABI (include/adama.h): argument marshalling only.

Every function has the name and argument order of its C counterpart.  Device
arrays are passed as integer device addresses or as objects with `.data_ptr()`
(e.g. torch tensors, used here only as owners of device memory); `stream` is a
raw `hipStream_t` value such as `torch.cuda.Stream().cuda_stream` (0 = null
stream).  A non-zero status raises AdamaError carrying adama_last_error().

There is no CPU fallback: if the library has not been built, importing this
module's functions fails loudly.
"""
from __future__ import annotations

import ctypes
import os



class _Build:
    """The build module, imported at first use (so that `python -m paper_2305_19982_amd.build` finds it unloaded)."""

    def __getattr__(self, name):
        from . import build
        return getattr(build, name)


_build = _Build()

F32, BF16, F16 = 0, 1, 2
DTYPES = {"f32": F32, "bf16": BF16, "f16": F16, F32: F32, BF16: BF16, F16: F16}
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED_DTYPE, ERR_TOO_LARGE, ERR_HIP = range(5)
STATUS_NAMES = {OK: "ADAMA_OK", ERR_INVALID_ARG: "ADAMA_ERR_INVALID_ARG",
                ERR_UNSUPPORTED_DTYPE: "ADAMA_ERR_UNSUPPORTED_DTYPE", ERR_TOO_LARGE: "ADAMA_ERR_TOO_LARGE",
                ERR_HIP: "ADAMA_ERR_HIP"}


class AdamaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status
        self.message = message


class adama_tensor(ctypes.Structure):
    _fields_ = [("m", ctypes.c_void_p), ("v", ctypes.c_void_p), ("grad", ctypes.c_void_p), ("n", ctypes.c_size_t)]


class adama_update_tensor(ctypes.Structure):
    _fields_ = [("theta", ctypes.c_void_p), ("m", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("grad", ctypes.c_void_p), ("n", ctypes.c_size_t)]


class adama_state(ctypes.Structure):
    _fields_ = [("theta", ctypes.c_void_p), ("m", ctypes.c_void_p), ("v", ctypes.c_void_p), ("n", ctypes.c_size_t)]


class adama_options(ctypes.Structure):
    _fields_ = [("weight_decay", ctypes.c_double), ("grad_scale", ctypes.c_double)]


class adama_sgdm_tensor(ctypes.Structure):
    _fields_ = [("theta", ctypes.c_void_p), ("b", ctypes.c_void_p), ("grad", ctypes.c_void_p), ("n", ctypes.c_size_t)]


_lib = None
_path_override = None


def library_path() -> str:
    return _path_override or _build.LIB


def use_library(path: str) -> None:
    """Load this library file instead of the package's own build (a variant made by
    `python -m paper_2305_19982_amd.build --out ...` for an A/B measurement).  It is taken as it is: no check
    against the sources, no rebuild.  Must be called before the first call into the library."""
    global _path_override
    if _lib is not None:
        raise RuntimeError("a library is already loaded")
    if not os.path.exists(path):
        raise FileNotFoundError(path)
    _path_override = os.path.abspath(path)


def _may_build_here() -> bool:
    """A build spawns hipcc: not from a process that has already initialised the GPU, nor under a profiler
    (whose preloaded tool library the compiler processes would inherit)."""
    import sys

    torch = sys.modules.get("torch")
    if torch is not None and torch.cuda.is_initialized():
        return False
    return not any("rocprof" in os.environ.get(k, "").lower() for k in ("LD_PRELOAD", "ROCP_TOOL_LIBRARIES"))


def load() -> ctypes.CDLL:
    """Load libadama.so.  A library that is missing, or that was built from other sources than the present
    ones (build.stale()), is rebuilt first where that is safe and refused with an error otherwise: a
    stale binary is never used silently."""
    global _lib
    if _lib is not None:
        return _lib
    if _path_override is None and _build.stale():
        if not _may_build_here():
            raise RuntimeError(f"{_build.LIB} is missing or was built from other sources (library "
                               f"{_build.library_id()}, sources {_build.source_id()}); build it first: "
                               "python -c 'import __graft_entry__ as g; g.build()'")
        _build.build_libadama()
    lib = ctypes.CDLL(library_path())
    vp, sz, dbl, i32, i64 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_double, ctypes.c_int, ctypes.c_longlong
    lib.adama_begin_step.argtypes = [vp, vp, sz, dbl, dbl, vp]
    lib.adama_begin_step_multi.argtypes = [ctypes.POINTER(adama_state), i32, dbl, dbl, vp]
    lib.adama_fold.argtypes = [vp, vp, vp, i32, sz, i32, dbl, dbl, vp]
    lib.adama_fold_multi.argtypes = [ctypes.POINTER(adama_tensor), i32, i32, i32, dbl, dbl, vp]
    lib.adama_fold_first.argtypes = [vp, vp, vp, i32, sz, i32, dbl, dbl, vp]
    lib.adama_fold_first_multi.argtypes = [ctypes.POINTER(adama_tensor), i32, i32, i32, dbl, dbl, vp]
    lib.adama_fold_last_apply.argtypes = [vp, vp, vp, vp, i32, sz, i32, dbl, dbl, dbl, dbl, i64, vp]
    lib.adama_fold_last_apply_multi.argtypes = [ctypes.POINTER(adama_update_tensor), i32, i32, i32, dbl, dbl, dbl,
                                                dbl, i64, vp]
    lib.adama_apply.argtypes = [vp, vp, vp, sz, dbl, dbl, dbl, dbl, i64, vp]
    lib.adama_apply_multi.argtypes = [ctypes.POINTER(adama_state), i32, dbl, dbl, dbl, dbl, i64, vp]
    lib.adama_rescale_apply.argtypes = [vp, vp, vp, sz, dbl, dbl, dbl, dbl, dbl, dbl, i64, vp]
    lib.adama_rescale_apply_multi.argtypes = [ctypes.POINTER(adama_state), i32, dbl, dbl, dbl, dbl, dbl, dbl, i64, vp]
    lib.adama_debug_walk.argtypes = [ctypes.POINTER(adama_update_tensor), i32, i32, i32, ctypes.POINTER(vp),
                                     ctypes.POINTER(ctypes.c_ulonglong), ctypes.POINTER(ctypes.c_ulonglong),
                                     ctypes.POINTER(i32)]
    optp = ctypes.POINTER(adama_options)
    sgdp = ctypes.POINTER(adama_sgdm_tensor)
    lib.adama_fold_opt_multi.argtypes = [ctypes.POINTER(adama_tensor), i32, i32, i32, dbl, dbl, optp, vp]
    lib.adama_fold_first_opt_multi.argtypes = [ctypes.POINTER(adama_tensor), i32, i32, i32, dbl, dbl, optp, vp]
    lib.adama_fold_last_apply_opt_multi.argtypes = [ctypes.POINTER(adama_update_tensor), i32, i32, i32, dbl, dbl, dbl,
                                                    dbl, i64, optp, vp]
    lib.adama_apply_opt_multi.argtypes = [ctypes.POINTER(adama_state), i32, dbl, dbl, dbl, dbl, i64, optp, vp]
    lib.adama_rescale_apply_opt_multi.argtypes = [ctypes.POINTER(adama_state), i32, dbl, dbl, dbl, dbl, dbl, dbl, i64,
                                                  optp, vp]
    lib.adama_sgdm_begin_step_multi.argtypes = [sgdp, i32, dbl, vp]
    lib.adama_sgdm_fold_multi.argtypes = [sgdp, i32, i32, i32, optp, vp]
    lib.adama_sgdm_fold_first_multi.argtypes = [sgdp, i32, i32, i32, dbl, optp, vp]
    lib.adama_sgdm_apply_multi.argtypes = [sgdp, i32, dbl, optp, vp]
    lib.adama_sgdm_fold_last_apply_multi.argtypes = [sgdp, i32, i32, i32, dbl, optp, vp]
    for name in ("adama_fold_opt_multi", "adama_fold_first_opt_multi", "adama_fold_last_apply_opt_multi",
                 "adama_apply_opt_multi", "adama_rescale_apply_opt_multi", "adama_sgdm_begin_step_multi",
                 "adama_sgdm_fold_multi", "adama_sgdm_fold_first_multi", "adama_sgdm_apply_multi",
                 "adama_sgdm_fold_last_apply_multi"):
        getattr(lib, name).restype = i32
    for name in ("adama_begin_step", "adama_begin_step_multi", "adama_fold", "adama_fold_multi", "adama_apply",
                 "adama_apply_multi", "adama_fold_first", "adama_fold_first_multi", "adama_fold_last_apply",
                 "adama_fold_last_apply_multi", "adama_rescale_apply", "adama_rescale_apply_multi",
                 "adama_debug_walk"):
        getattr(lib, name).restype = i32
    lib.adama_last_error.restype = ctypes.c_char_p
    lib.adama_last_error.argtypes = []
    lib.adama_max_tensors_per_launch.restype = i32
    lib.adama_max_tensors_per_launch.argtypes = []
    lib.adama_residency.restype = i32
    lib.adama_residency.argtypes = [i32, ctypes.c_ulonglong]
    lib.adama_debug_set_residency.restype = None
    lib.adama_debug_set_residency.argtypes = [i32, i32, i32]
    lib.adama_build_id.restype = ctypes.c_char_p
    lib.adama_build_id.argtypes = []
    lib.adama_launch_chunk.restype = i32
    lib.adama_launch_chunk.argtypes = [i32, ctypes.c_ulonglong]
    lib.adama_tuning.restype = None
    lib.adama_tuning.argtypes = [i32, ctypes.c_ulonglong, ctypes.POINTER(i32), ctypes.POINTER(i32),
                                 ctypes.POINTER(ctypes.c_ulonglong), ctypes.POINTER(i32)]
    _lib = lib
    return lib


def _ptr(x) -> int | None:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _check(status: int) -> None:
    if status != OK:
        raise AdamaError(status, load().adama_last_error().decode("utf-8", "replace"))


def adama_last_error() -> str:
    return load().adama_last_error().decode("utf-8", "replace")


def adama_residency(op, launch_elems: int) -> int:
    return int(load().adama_residency(OPS.get(op, op), int(launch_elems)))


def adama_debug_set_residency(op, size_class: int, wgs_per_cu: int) -> None:
    load().adama_debug_set_residency(OPS.get(op, op), size_class, wgs_per_cu)


def adama_build_id() -> str:
    return load().adama_build_id().decode()


def adama_max_tensors_per_launch() -> int:
    return int(load().adama_max_tensors_per_launch())


OPS = {"decay": 0, "fold": 1, "apply": 2, "fold_first": 3, "fold_last_apply": 4, "rescale_apply": 5,
       "sgd_decay": 6, "sgd_fold": 7, "sgd_apply": 8, "sgd_fold_first": 9, "sgd_fold_last_apply": 10}


def adama_launch_chunk(op, launch_elems: int) -> int:
    return int(load().adama_launch_chunk(OPS.get(op, op), int(launch_elems)))


def adama_tuning(op="fold", launch_elems: int = 1 << 25) -> dict:
    """Workgroup shape, large-launch threshold and cache-policy bits for a launch of `op` over `launch_elems` elements."""
    blk, grp, pol, big = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0), ctypes.c_ulonglong(0)
    load().adama_tuning(OPS.get(op, op), int(launch_elems), ctypes.byref(blk), ctypes.byref(grp), ctypes.byref(big),
                        ctypes.byref(pol))
    return {"block": blk.value, "groups_per_thread": grp.value, "big_launch_elems": big.value,
            "policy_bits": pol.value}


def tensor_list(entries) -> ctypes.Array:
    """Host array of adama_tensor from (m, v, grad, n) tuples; reusable across calls."""
    arr = (adama_tensor * len(entries))()
    for i, (m, v, g, n) in enumerate(entries):
        arr[i] = adama_tensor(_ptr(m), _ptr(v), _ptr(g), int(n))
    return arr


def update_list(entries) -> ctypes.Array:
    """Host array of adama_update_tensor from (theta, m, v, grad, n) tuples; reusable across calls."""
    arr = (adama_update_tensor * len(entries))()
    for i, (th, m, v, g, n) in enumerate(entries):
        arr[i] = adama_update_tensor(_ptr(th), _ptr(m), _ptr(v), _ptr(g), int(n))
    return arr


def state_list(entries) -> ctypes.Array:
    """Host array of adama_state from (theta, m, v, n) tuples; reusable across calls."""
    arr = (adama_state * len(entries))()
    for i, (th, m, v, n) in enumerate(entries):
        arr[i] = adama_state(_ptr(th), _ptr(m), _ptr(v), int(n))
    return arr


def adama_begin_step(m, v, n: int, beta1: float, beta2: float, stream: int = 0) -> None:
    _check(load().adama_begin_step(_ptr(m), _ptr(v), n, beta1, beta2, stream))


def adama_begin_step_multi(lst, count: int | None, beta1: float, beta2: float, stream: int = 0) -> None:
    if not isinstance(lst, ctypes.Array):
        lst = state_list(lst)
    _check(load().adama_begin_step_multi(lst, len(lst) if count is None else count, beta1, beta2, stream))


def adama_fold(m, v, grad, gdt, n: int, N: int, beta1: float, beta2: float, stream: int = 0) -> None:
    _check(load().adama_fold(_ptr(m), _ptr(v), _ptr(grad), DTYPES.get(gdt, gdt), n, N, beta1, beta2, stream))


def adama_fold_multi(lst, count: int | None, gdt, N: int, beta1: float, beta2: float, stream: int = 0) -> None:
    if not isinstance(lst, ctypes.Array):
        lst = tensor_list(lst)
    _check(load().adama_fold_multi(lst, len(lst) if count is None else count, DTYPES.get(gdt, gdt), N, beta1,
                                   beta2, stream))


def adama_fold_first(m, v, grad, gdt, n: int, N: int, beta1: float, beta2: float, stream: int = 0) -> None:
    _check(load().adama_fold_first(_ptr(m), _ptr(v), _ptr(grad), DTYPES.get(gdt, gdt), n, N, beta1, beta2, stream))


def adama_fold_first_multi(lst, count: int | None, gdt, N: int, beta1: float, beta2: float, stream: int = 0) -> None:
    if not isinstance(lst, ctypes.Array):
        lst = tensor_list(lst)
    _check(load().adama_fold_first_multi(lst, len(lst) if count is None else count, DTYPES.get(gdt, gdt), N, beta1,
                                         beta2, stream))


def adama_fold_last_apply(theta, m, v, grad, gdt, n: int, N: int, lr: float, eps: float, beta1: float, beta2: float,
                          t: int, stream: int = 0) -> None:
    _check(load().adama_fold_last_apply(_ptr(theta), _ptr(m), _ptr(v), _ptr(grad), DTYPES.get(gdt, gdt), n, N, lr, eps,
                                        beta1, beta2, t, stream))


def adama_fold_last_apply_multi(lst, count: int | None, gdt, N: int, lr: float, eps: float, beta1: float,
                                beta2: float, t: int, stream: int = 0) -> None:
    if not isinstance(lst, ctypes.Array):
        lst = update_list(lst)
    _check(load().adama_fold_last_apply_multi(lst, len(lst) if count is None else count, DTYPES.get(gdt, gdt), N, lr,
                                              eps, beta1, beta2, t, stream))


def adama_apply(theta, m, v, n: int, lr: float, eps: float, beta1: float, beta2: float, t: int,
                stream: int = 0) -> None:
    _check(load().adama_apply(_ptr(theta), _ptr(m), _ptr(v), n, lr, eps, beta1, beta2, t, stream))


def adama_apply_multi(lst, count: int | None, lr: float, eps: float, beta1: float, beta2: float, t: int,
                      stream: int = 0) -> None:
    if not isinstance(lst, ctypes.Array):
        lst = state_list(lst)
    _check(load().adama_apply_multi(lst, len(lst) if count is None else count, lr, eps, beta1, beta2, t, stream))


def adama_rescale_apply(theta, m, v, n: int, m_scale: float, v_scale: float, lr: float, eps: float, beta1: float,
                        beta2: float, t: int, stream: int = 0) -> None:
    _check(load().adama_rescale_apply(_ptr(theta), _ptr(m), _ptr(v), n, m_scale, v_scale, lr, eps, beta1, beta2, t,
                                      stream))


def adama_rescale_apply_multi(lst, count: int | None, m_scale: float, v_scale: float, lr: float, eps: float,
                              beta1: float, beta2: float, t: int, stream: int = 0) -> None:
    if not isinstance(lst, ctypes.Array):
        lst = state_list(lst)
    _check(load().adama_rescale_apply_multi(lst, len(lst) if count is None else count, m_scale, v_scale, lr, eps,
                                            beta1, beta2, t, stream))


def options(weight_decay: float = 0.0, grad_scale: float = 1.0) -> adama_options:
    return adama_options(weight_decay, grad_scale)


def _opt(opt):
    """None (-> NULL), an adama_options, or a (weight_decay, grad_scale) pair."""
    if opt is None:
        return None
    if isinstance(opt, adama_options):
        return ctypes.byref(opt)
    return ctypes.byref(adama_options(float(opt[0]), float(opt[1])))


def sgdm_list(entries) -> ctypes.Array:
    """Host array of adama_sgdm_tensor from (theta, b, grad, n) tuples; reusable across calls."""
    arr = (adama_sgdm_tensor * len(entries))()
    for i, (th, b, g, n) in enumerate(entries):
        arr[i] = adama_sgdm_tensor(_ptr(th), _ptr(b), _ptr(g), int(n))
    return arr


def adama_fold_opt_multi(lst, count: int | None, gdt, N: int, beta1: float, beta2: float, opt=None,
                         stream: int = 0) -> None:
    if not isinstance(lst, ctypes.Array):
        lst = tensor_list(lst)
    _check(load().adama_fold_opt_multi(lst, len(lst) if count is None else count, DTYPES.get(gdt, gdt), N, beta1,
                                       beta2, _opt(opt), stream))


def adama_fold_first_opt_multi(lst, count: int | None, gdt, N: int, beta1: float, beta2: float, opt=None,
                               stream: int = 0) -> None:
    if not isinstance(lst, ctypes.Array):
        lst = tensor_list(lst)
    _check(load().adama_fold_first_opt_multi(lst, len(lst) if count is None else count, DTYPES.get(gdt, gdt), N,
                                             beta1, beta2, _opt(opt), stream))


def adama_fold_last_apply_opt_multi(lst, count: int | None, gdt, N: int, lr: float, eps: float, beta1: float,
                                    beta2: float, t: int, opt=None, stream: int = 0) -> None:
    if not isinstance(lst, ctypes.Array):
        lst = update_list(lst)
    _check(load().adama_fold_last_apply_opt_multi(lst, len(lst) if count is None else count, DTYPES.get(gdt, gdt), N,
                                                  lr, eps, beta1, beta2, t, _opt(opt), stream))


def adama_apply_opt_multi(lst, count: int | None, lr: float, eps: float, beta1: float, beta2: float, t: int,
                          opt=None, stream: int = 0) -> None:
    if not isinstance(lst, ctypes.Array):
        lst = state_list(lst)
    _check(load().adama_apply_opt_multi(lst, len(lst) if count is None else count, lr, eps, beta1, beta2, t,
                                        _opt(opt), stream))


def adama_rescale_apply_opt_multi(lst, count: int | None, m_scale: float, v_scale: float, lr: float, eps: float,
                                  beta1: float, beta2: float, t: int, opt=None, stream: int = 0) -> None:
    if not isinstance(lst, ctypes.Array):
        lst = state_list(lst)
    _check(load().adama_rescale_apply_opt_multi(lst, len(lst) if count is None else count, m_scale, v_scale, lr, eps,
                                                beta1, beta2, t, _opt(opt), stream))


def adama_sgdm_begin_step_multi(lst, count: int | None, momentum: float, stream: int = 0) -> None:
    if not isinstance(lst, ctypes.Array):
        lst = sgdm_list(lst)
    _check(load().adama_sgdm_begin_step_multi(lst, len(lst) if count is None else count, momentum, stream))


def adama_sgdm_fold_multi(lst, count: int | None, gdt, N: int, opt=None, stream: int = 0) -> None:
    if not isinstance(lst, ctypes.Array):
        lst = sgdm_list(lst)
    _check(load().adama_sgdm_fold_multi(lst, len(lst) if count is None else count, DTYPES.get(gdt, gdt), N, _opt(opt),
                                        stream))


def adama_sgdm_fold_first_multi(lst, count: int | None, gdt, N: int, momentum: float, opt=None,
                                stream: int = 0) -> None:
    if not isinstance(lst, ctypes.Array):
        lst = sgdm_list(lst)
    _check(load().adama_sgdm_fold_first_multi(lst, len(lst) if count is None else count, DTYPES.get(gdt, gdt), N,
                                              momentum, _opt(opt), stream))


def adama_sgdm_apply_multi(lst, count: int | None, lr: float, opt=None, stream: int = 0) -> None:
    if not isinstance(lst, ctypes.Array):
        lst = sgdm_list(lst)
    _check(load().adama_sgdm_apply_multi(lst, len(lst) if count is None else count, lr, _opt(opt), stream))


def adama_sgdm_fold_last_apply_multi(lst, count: int | None, gdt, N: int, lr: float, opt=None,
                                     stream: int = 0) -> None:
    if not isinstance(lst, ctypes.Array):
        lst = sgdm_list(lst)
    _check(load().adama_sgdm_fold_last_apply_multi(lst, len(lst) if count is None else count, DTYPES.get(gdt, gdt), N,
                                                   lr, _opt(opt), stream))


def adama_debug_walk(entries, op: int, gdt):
    """Host-only geometry walk.  entries: (theta, m, v, grad, n) integer addresses (never dereferenced;
    fields the op does not use may be None).  Returns (touch counts per tensor as bytes, vector accesses,
    scalar accesses, launches)."""
    lst = update_list(entries)
    bufs = [(ctypes.c_ubyte * max(1, int(e[4])))() for e in entries]
    ptrs = (ctypes.c_void_p * max(1, len(entries)))(*[ctypes.addressof(b) for b in bufs])
    nvec, nsc, nl = ctypes.c_ulonglong(0), ctypes.c_ulonglong(0), ctypes.c_int(0)
    _check(load().adama_debug_walk(lst, len(entries), op, DTYPES.get(gdt, gdt), ptrs, ctypes.byref(nvec),
                                   ctypes.byref(nsc), ctypes.byref(nl)))
    return [bytes(b)[:int(e[4])] for b, e in zip(bufs, entries)], nvec.value, nsc.value, nl.value
