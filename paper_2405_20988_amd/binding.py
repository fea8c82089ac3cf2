"""ctypes binding of include/fda.h: same names, argument marshalling only.

Device pointers are plain integers (for a torch tensor: ``t.data_ptr()``); streams are the
integer ``torch.cuda.current_stream().cuda_stream``.  Nothing here computes anything: if
the HIP library is missing the import of a symbol fails loudly (there is no fallback).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

FDA_OK, FDA_EINVAL, FDA_ERANGE, FDA_ENOMEM, FDA_EHIP = 0, -1, -2, -3, -4
FDA_F32, FDA_BF16 = 0, 1
FDA_VARIANT_LINEAR, FDA_VARIANT_SKETCH = 1, 2
FDA_DESC_PLAIN_TABLE = 1

_PKG = os.path.dirname(os.path.abspath(__file__))
# FDA_LIBRARY: load another build of the library instead of the in-tree one (experiments)
_LIB_PATH = os.environ.get("FDA_LIBRARY") or os.path.join(_PKG, "lib", "libfda.so")
_lib = None


class FdaError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {fda_strerror(code)} ({code}): {fda_last_error()}")
        self.code = code


class FdaDesc(C.Structure):
    _fields_ = [("K", C.c_int32), ("dtype", C.c_int32), ("d", C.c_int64),
                ("row_stride", C.c_int64), ("variants", C.c_int32), ("l", C.c_int32),
                ("m", C.c_int32), ("flags", C.c_int32), ("eps", C.c_double),
                ("hash_coef", C.POINTER(C.c_uint32))]


class FdaEstimate(C.Structure):
    _fields_ = [("mean_sqnorm", C.c_double), ("mean_proj", C.c_double), ("m2", C.c_double),
                ("h_linear", C.c_double), ("h_sketch", C.c_double),
                ("sync_linear", C.c_int32), ("sync_sketch", C.c_int32),
                ("near_tie_linear", C.c_int32), ("near_tie_sketch", C.c_int32),
                ("nonfinite", C.c_int32), ("state_path", C.c_int32)]

    def as_dict(self) -> dict:
        return {name: getattr(self, name) for name, _ in self._fields_}


class FdaPlanInfo(C.Structure):
    _fields_ = [("worker_groups", C.c_int32), ("workers_per_group", C.c_int32),
                ("row_groups", C.c_int32), ("rows_per_group", C.c_int32),
                ("partitions", C.c_int32), ("threads", C.c_int32), ("chunk", C.c_int64),
                ("lds_bytes", C.c_int64), ("workspace_bytes", C.c_int64),
                ("state_floats", C.c_int64),
                ("mean_row_groups", C.c_int32), ("mean_rows_per_group", C.c_int32),
                ("mean_partitions", C.c_int32), ("mean_workgroups_per_cu", C.c_int32),
                ("mean_chunk", C.c_int64), ("mean_lds_bytes", C.c_int64),
                ("sign_split_rows", C.c_int32), ("worker_slots", C.c_int32),
                ("placed_row_group", C.c_int32), ("reserved", C.c_int32)]

    def as_dict(self) -> dict:
        return {name: getattr(self, name) for name, _ in self._fields_}


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libfda.so (built in-tree by paper_2405_20988_amd.build; built here if it does not exist
    yet).  Raises if it is absent and cannot be built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        # nothing built yet: build once (a stale library is never rebuilt here; rebuild explicitly)
        try:
            from .build import build_library
            build_library()
        except Exception as exc:
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing and could not be built ({exc}): build it with "
                "`python -m paper_2405_20988_amd.build` (needs hipcc); there is no CPU fallback") from exc
    lib = C.CDLL(_LIB_PATH)
    vp, i32p = C.c_void_p, C.c_void_p
    lib.fda_strerror.restype = C.c_char_p
    lib.fda_strerror.argtypes = [C.c_int]
    lib.fda_last_error.restype = C.c_char_p
    lib.fda_last_error.argtypes = []
    lib.fda_plan.argtypes = [C.POINTER(FdaDesc), C.c_int32, C.c_int64, C.POINTER(FdaPlanInfo)]
    lib.fda_workspace_bytes.argtypes = [C.POINTER(FdaDesc), C.POINTER(C.c_size_t)]
    lib.fda_create.argtypes = [C.POINTER(vp), C.POINTER(FdaDesc), vp, C.c_size_t]
    lib.fda_destroy.argtypes = [vp]
    lib.fda_state_floats.argtypes = [vp, C.POINTER(C.c_int64)]
    lib.fda_get_plan.argtypes = [vp, C.POINTER(FdaPlanInfo)]
    lib.fda_local_state.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.fda_estimate_variance.argtypes = [vp, vp, C.c_double, C.c_double, vp,
                                          C.POINTER(FdaEstimate), vp]
    lib.fda_mean_state.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.fda_sync_from_mean.argtypes = [vp, vp, vp, vp, vp, vp, i32p, vp]
    lib.fda_estimate_variance_mean.argtypes = [vp, vp, C.c_double, C.c_double, vp,
                                               C.POINTER(FdaEstimate), vp]
    lib.fda_last_mean_state_path.argtypes = [vp, C.POINTER(C.c_int32), vp]
    lib.fda_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, C.c_double, C.c_double, C.c_int32, C.c_int32, vp,
                             C.POINTER(FdaEstimate), vp]
    lib.fda_sync.argtypes = [vp, vp, vp, vp, i32p, vp]
    lib.fda_update_xi.argtypes = [vp, vp, vp, vp, i32p, vp]
    lib.fda_sync_xi.argtypes = [vp, vp, vp, vp, vp, i32p, vp]
    lib.fda_last_state_path.argtypes = [vp, C.POINTER(C.c_int32), vp]
    lib.fda_profile_enable.argtypes = [vp, C.c_int]
    lib.fda_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.c_int]
    lib.fda_calib_stream.argtypes = [C.c_int, vp, vp, C.c_size_t, C.c_int, vp, C.POINTER(C.c_double)]
    lib.fda_calib_lds_atomics.argtypes = [C.c_int, C.c_int, C.c_int, vp, vp, C.POINTER(C.c_double),
                                          C.POINTER(C.c_double)]
    lib.fda_estimate_variance_static.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_double,
                                                 C.c_double, C.c_double, vp, vp]
    for name in ("fda_estimate_variance_static", "fda_calib_stream", "fda_calib_lds_atomics", "fda_step", "fda_sync_from_mean", "fda_mean_state", "fda_estimate_variance_mean", "fda_last_mean_state_path",
                 "fda_last_state_path", "fda_profile_enable", "fda_profile_read", "fda_plan", "fda_workspace_bytes", "fda_create", "fda_destroy",
                 "fda_state_floats", "fda_get_plan", "fda_local_state",
                 "fda_estimate_variance", "fda_sync", "fda_sync_xi", "fda_update_xi"):
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _check(rc: int, what: str) -> None:
    if rc != FDA_OK:
        raise FdaError(rc, what)


def make_desc(K, d, dtype, variants, l=0, m=0, eps=0.0, hash_coef=None, row_stride=None, flags=0):
    """Fill an FdaDesc; returns (desc, keepalive) -- keepalive owns the coefficient array."""
    desc = FdaDesc()
    desc.K, desc.d, desc.dtype, desc.variants = int(K), int(d), int(dtype), int(variants)
    desc.row_stride = int(d if row_stride is None else row_stride)
    desc.l, desc.m, desc.flags, desc.eps = int(l), int(m), int(flags), float(eps)
    keep = None
    if hash_coef is not None:
        keep = np.ascontiguousarray(hash_coef, dtype=np.uint32)
        desc.hash_coef = keep.ctypes.data_as(C.POINTER(C.c_uint32))
    return desc, keep


def fda_strerror(code: int) -> str:
    return load_library().fda_strerror(int(code)).decode()


def fda_last_error() -> str:
    return load_library().fda_last_error().decode()


def fda_plan(desc: FdaDesc, compute_units: int, lds_bytes_per_cu: int) -> FdaPlanInfo:
    out = FdaPlanInfo()
    _check(load_library().fda_plan(C.byref(desc), compute_units, lds_bytes_per_cu, C.byref(out)),
           "fda_plan")
    return out


def fda_workspace_bytes(desc: FdaDesc) -> int:
    n = C.c_size_t(0)
    _check(load_library().fda_workspace_bytes(C.byref(desc), C.byref(n)), "fda_workspace_bytes")
    return int(n.value)


def fda_create(desc: FdaDesc, workspace_ptr: int, workspace_bytes: int) -> int:
    ctx = C.c_void_p(None)
    _check(load_library().fda_create(C.byref(ctx), C.byref(desc), workspace_ptr, workspace_bytes),
           "fda_create")
    return ctx.value


def fda_destroy(ctx: int) -> None:
    _check(load_library().fda_destroy(ctx), "fda_destroy")


def fda_state_floats(ctx: int) -> int:
    s = C.c_int64(0)
    _check(load_library().fda_state_floats(ctx, C.byref(s)), "fda_state_floats")
    return int(s.value)


def fda_get_plan(ctx: int) -> FdaPlanInfo:
    out = FdaPlanInfo()
    _check(load_library().fda_get_plan(ctx, C.byref(out)), "fda_get_plan")
    return out


def fda_local_state(ctx: int, w: int, w_t0: int, xi: int | None, state: int, stream: int = 0) -> None:
    _check(load_library().fda_local_state(ctx, w, w_t0, xi, state, stream), "fda_local_state")


def fda_estimate_variance(ctx: int, state: int, theta: float, tie_tol: float, out_dev: int,
                          want_host: bool = True, stream: int = 0):
    """Returns the host copy of the result (an FdaEstimate) if want_host, else None."""
    host = FdaEstimate() if want_host else None
    _check(load_library().fda_estimate_variance(ctx, state, theta, tie_tol, out_dev,
                                                C.byref(host) if want_host else None, stream),
           "fda_estimate_variance")
    return host


def fda_estimate_variance_static(state: int, K: int, l: int, m: int, variants: int, eps: float, theta: float,
                                 tie_tol: float, out_dev: int, stream: int = 0) -> None:
    """fda_estimate_variance without a context: its scratch is a static device array of the library."""
    _check(load_library().fda_estimate_variance_static(state, K, l, m, variants, eps, theta, tie_tol, out_dev,
                                                       stream), "fda_estimate_variance_static")


def fda_mean_state(ctx: int, w: int, w_t0: int, xi: int | None, mean_state: int,
                   w_bar: int | None = None, stream: int = 0) -> None:
    _check(load_library().fda_mean_state(ctx, w, w_t0, xi, mean_state, w_bar, stream), "fda_mean_state")


def fda_sync_from_mean(ctx: int, w: int, w_t0: int, w_prev: int | None, xi: int | None, w_bar: int,
                       pred_dev: int | None = None, stream: int = 0) -> None:
    _check(load_library().fda_sync_from_mean(ctx, w, w_t0, w_prev, xi, w_bar, pred_dev, stream),
           "fda_sync_from_mean")


def fda_estimate_variance_mean(ctx: int, mean_state: int, theta: float, tie_tol: float, out_dev: int,
                               want_host: bool = True, stream: int = 0):
    """Returns the host copy of the result (an FdaEstimate) if want_host, else None."""
    host = FdaEstimate() if want_host else None
    _check(load_library().fda_estimate_variance_mean(ctx, mean_state, theta, tie_tol, out_dev,
                                                     C.byref(host) if want_host else None, stream),
           "fda_estimate_variance_mean")
    return host


def fda_sync(ctx: int, w: int, w_t0: int, w_prev: int | None, pred_dev: int | None = None,
             stream: int = 0) -> None:
    _check(load_library().fda_sync(ctx, w, w_t0, w_prev, pred_dev, stream), "fda_sync")


def fda_sync_xi(ctx: int, w: int, w_t0: int, w_prev: int, xi: int, pred_dev: int | None = None,
                stream: int = 0) -> None:
    _check(load_library().fda_sync_xi(ctx, w, w_t0, w_prev, xi, pred_dev, stream), "fda_sync_xi")


def fda_update_xi(ctx: int, w_t0: int, w_prev: int, xi: int, pred_dev: int | None = None,
                  stream: int = 0) -> None:
    _check(load_library().fda_update_xi(ctx, w_t0, w_prev, xi, pred_dev, stream), "fda_update_xi")


FDA_STEP_MEAN_STATE = 1


def fda_step(ctx: int, w: int, w_t0: int, w_prev: int | None, xi: int | None, state: int,
             w_bar: int | None, theta: float, tie_tol: float, decide_by: int, flags: int, out_dev: int,
             want_host: bool = False, stream: int = 0):
    """Algorithm 1 lines 6-9 as one enqueue; returns the host copy of the result if want_host."""
    host = FdaEstimate() if want_host else None
    _check(load_library().fda_step(ctx, w, w_t0, w_prev, xi, state, w_bar, theta, tie_tol, decide_by,
                                   flags, out_dev, C.byref(host) if want_host else None, stream),
           "fda_step")
    return host


def fda_profile_enable(ctx: int, on: bool) -> None:
    _check(load_library().fda_profile_enable(ctx, 1 if on else 0), "fda_profile_enable")


def fda_profile_read(ctx: int, reset: bool = True):
    """(total state-kernel milliseconds, launches) since the last reset."""
    ms, n = C.c_double(0.0), C.c_int64(0)
    _check(load_library().fda_profile_read(ctx, C.byref(ms), C.byref(n), 1 if reset else 0),
           "fda_profile_read")
    return float(ms.value), int(n.value)


def fda_last_state_path(ctx: int, stream: int = 0) -> int:
    """0 / 1 / 2: the last fda_local_state used 32-bit, 64-bit integer or fp64 sketch cells."""
    v = C.c_int32(0)
    _check(load_library().fda_last_state_path(ctx, C.byref(v), stream), "fda_last_state_path")
    return int(v.value)


def fda_last_mean_state_path(ctx: int, stream: int = 0) -> int:
    """0 / 1: the last fda_mean_state used integer sums in 64-bit cells, or fp64."""
    v = C.c_int32(0)
    _check(load_library().fda_last_mean_state_path(ctx, C.byref(v), stream), "fda_last_mean_state_path")
    return int(v.value)


CALIB_READ, CALIB_WRITE, CALIB_COPY, CALIB_NONTEMPORAL = 0, 1, 2, 4
LDS_OPS = {"u32_rtn": 0, "u32": 1, "u64": 2, "f64": 3, "f32": 4, "u64_rtn": 5, "read8": 6, "read16": 7}
LDS_PATTERNS = {"random": 0, "consecutive": 1, "groups4": 2, "groups8": 3, "groups16": 4, "groups32": 5}


def fda_calib_stream(mode: int, src: int | None, dst: int, nbytes: int, reps: int = 5, stream: int = 0) -> float:
    """Milliseconds per pass of a read (0), fill (1) or copy (2) kernel over nbytes; +4: with the
    nontemporal hint on loads and stores (measurement aid)."""
    ms = C.c_double(0.0)
    _check(load_library().fda_calib_stream(mode, src, dst, nbytes, reps, stream, C.byref(ms)), "fda_calib_stream")
    return float(ms.value)


def fda_calib_lds_atomics(op: int, pattern: int, iters: int, sink: int, stream: int = 0):
    """(LDS atomic additions per lane, clock and compute unit; clock in GHz) of the calibration kernel."""
    rate, ghz = C.c_double(0.0), C.c_double(0.0)
    _check(load_library().fda_calib_lds_atomics(op, pattern, iters, sink, stream, C.byref(rate), C.byref(ghz)),
           "fda_calib_lds_atomics")
    return float(rate.value), float(ghz.value)
