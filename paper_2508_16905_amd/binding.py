"""ctypes binding of the C ABI in ``include/triaccel.h`` -- argument marshalling only.

Every step of the optimizer path runs in the HIP library; nothing is computed here.  If the
library has not been built (``python -m paper_2508_16905_amd.build`` or ``__graft_entry__.build()``)
or cannot be loaded, every call raises: there is no CPU fallback.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
# TRIACCEL_LIBRARY overrides the in-tree build (e.g. to try a differently tuned build of the library)
LIB_PATH = os.environ.get("TRIACCEL_LIBRARY") or os.path.join(_HERE, "libtriaccel.so")

FP16, BF16, FP32 = 0, 1, 2
N_STAGES = 7
STAGE_NAMES = ("grad_stats", "curv_ema", "layer", "select_refine", "update", "update_resize", "select_finish")


class Config(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32),
        ("beta_var", C.c_float),
        ("beta_curv", C.c_float),
        ("tau_low", C.c_float),
        ("tau_high", C.c_float),
        ("tau_curv", C.c_float),
        ("alpha", C.c_float),
        ("sparsity_ppm", C.c_uint32),
        ("momentum", C.c_float),
        ("weight_decay", C.c_float),
        ("ctrl_interval", C.c_int32),
        ("scale_backoff", C.c_float),
        ("scale_growth", C.c_float),
        ("growth_interval", C.c_int32),
        ("rho_low", C.c_double),
        ("rho_high", C.c_double),
        ("delta_up", C.c_int32),
        ("delta_down", C.c_int32),
        ("b_min", C.c_int32),
        ("b_max", C.c_int32),
        ("power_k", C.c_int32),
        ("lambda_source", C.c_int32),
        ("curvature_source", C.c_int32),
        ("elementwise_scale", C.c_int32),
        ("topk_abs", C.c_uint32),
    ]
    # fields a hyper-parameter dict may leave out
    _OPTIONAL = {"power_k": 0, "lambda_source": 0, "curvature_source": 0, "elementwise_scale": 0, "topk_abs": 0}

    @classmethod
    def from_hyper(cls, hyper: dict) -> "Config":
        cfg = cls()
        cfg.struct_size = C.sizeof(cls)
        for name, _ in cls._fields_[1:]:
            setattr(cfg, name, hyper[name] if name in hyper else cls._OPTIONAL[name])
        return cfg


class Tensor(C.Structure):
    _fields_ = [
        ("param", C.c_void_p),
        ("grad", C.c_void_p),
        ("z", C.c_void_p),
        ("hz", C.c_void_p),
        ("curv", C.c_void_p),
        ("mom", C.c_void_p),
        ("mask", C.c_void_p),
        ("numel", C.c_int64),
        ("grad_dtype", C.c_int32),
        ("param_dtype", C.c_int32),
    ]


class StepArgs(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32),
        ("lr", C.c_float),
        ("loss_scale", C.c_float),
        ("batch_size", C.c_int32),
        ("mem_used_bytes", C.c_uint64),
        ("mem_total_bytes", C.c_uint64),
        ("update_curvature", C.c_int32),
        ("reserved_", C.c_int32),
    ]


class StepResult(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32),
        ("skipped", C.c_int32),
        ("step_index", C.c_uint64),
        ("next_loss_scale", C.c_float),
        ("next_batch_size", C.c_int32),
    ]


class LayerInfo(C.Structure):
    _fields_ = [
        ("numel", C.c_int64),
        ("mean", C.c_float),
        ("var", C.c_float),
        ("v", C.c_float),
        ("theta", C.c_float),
        ("nnz", C.c_uint32),
        ("lambda_", C.c_float),
        ("lambda_ctrl", C.c_float),
        ("eta", C.c_float),
        ("code", C.c_int32),
        ("prev_code", C.c_int32),
        ("found_inf", C.c_uint32),
        ("curv_nonfinite", C.c_uint32),
        ("sel_passes", C.c_uint32),
        ("sel_listed", C.c_uint32),
        ("sel_outcome", C.c_uint32),
    ]


class PowerTensor(C.Structure):
    _fields_ = [("u", C.c_void_p), ("hu", C.c_void_p), ("stride", C.c_int64)]


class PowerInfo(C.Structure):
    _fields_ = [
        ("rayleigh", C.c_float * 8),
        ("resid", C.c_float * 8),
        ("hnorm", C.c_float * 8),
        ("deficient", C.c_uint32),
        ("lambda_max", C.c_float),
        ("lambda_latched", C.c_float),
    ]


class StageTimes(C.Structure):
    _fields_ = [("ms", C.c_float * N_STAGES)]


EXPORTS = {
    "triaccel_init": (C.c_int, [C.POINTER(C.c_void_p), C.POINTER(Config), C.POINTER(Tensor), C.c_int32, C.c_void_p]),
    "triaccel_step": (C.c_int, [C.c_void_p, C.POINTER(Tensor), C.c_int32, C.POINTER(StepArgs)]),
    "triaccel_result": (C.c_int, [C.c_void_p, C.POINTER(StepResult)]),
    "triaccel_layer_state": (C.c_int, [C.c_void_p, C.POINTER(LayerInfo), C.c_int32]),
    "triaccel_batch_next": (C.c_int32, [C.POINTER(Config), C.c_int32, C.c_uint64, C.c_uint64]),
    "triaccel_destroy": (None, [C.c_void_p]),
    "triaccel_strerror": (C.c_char_p, [C.c_int]),
    "triaccel_last_error": (C.c_char_p, []),
    "triaccel_set_profiling": (C.c_int, [C.c_void_p, C.c_int32]),
    "triaccel_set_graph": (C.c_int, [C.c_void_p, C.c_int32]),
    "triaccel_stage_times_get": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(StageTimes)]),
    "triaccel_cast_f32": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p]),
    "triaccel_state_size": (C.c_int64, [C.c_void_p]),
    "triaccel_get_state": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64]),
    "triaccel_set_state": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64]),
    "triaccel_power_iter": (C.c_int, [C.c_void_p, C.POINTER(PowerTensor), C.c_int32, C.c_int32, C.c_int32]),
    "triaccel_power_state": (C.c_int, [C.c_void_p, C.POINTER(PowerInfo), C.c_int32]),
    "triaccel_power_times_get": (C.c_int, [C.c_void_p, C.POINTER(C.c_float)]),
    "triaccel_power_iter_static": (C.c_int, [C.POINTER(PowerTensor), C.POINTER(C.c_int64), C.c_int32, C.c_int32,
                                             C.c_void_p, C.c_void_p]),
}

_lib: Optional[C.CDLL] = None


class TriAccelError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        detail = ""
        if _lib is not None:
            detail = _lib.triaccel_strerror(code).decode()
            if code == -6 or (code == -1 and where == "triaccel_power_iter_static"):
                detail += " -- " + _lib.triaccel_last_error().decode()
        super().__init__(f"{where} failed with code {code}: {detail}")


def load_library() -> C.CDLL:
    """Load ``libtriaccel.so`` (built in-tree).  Raises if it is missing: no fallback exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} not found: build the HIP library first "
            "(python -m paper_2508_16905_amd.build, or __graft_entry__.build())"
        )
    lib = C.CDLL(LIB_PATH)
    for name, (res, args) in EXPORTS.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _check(code: int, where: str) -> None:
    if code != 0:
        raise TriAccelError(code, where)


# ---- thin wrappers with the C names ------------------------------------------------------------

def triaccel_init(config: Config, tensors: Sequence[Tensor], stream: int = 0) -> C.c_void_p:
    lib = load_library()
    arr = (Tensor * len(tensors))(*tensors)
    handle = C.c_void_p()
    _check(lib.triaccel_init(C.byref(handle), C.byref(config), arr, len(tensors), C.c_void_p(stream)), "triaccel_init")
    return handle


def triaccel_step(handle, tensors, lr: float, loss_scale: float, batch_size: int = 0, mem_used_bytes: int = 0,
                  mem_total_bytes: int = 0, update_curvature: bool = True) -> None:
    """``tensors`` is a ctypes array ``(Tensor * n)`` or a sequence of ``Tensor``."""
    lib = load_library()
    arr = tensors if isinstance(tensors, C.Array) else (Tensor * len(tensors))(*tensors)
    args = StepArgs(C.sizeof(StepArgs), lr, loss_scale, batch_size, mem_used_bytes, mem_total_bytes,
                    int(update_curvature), 0)
    _check(lib.triaccel_step(handle, arr, len(arr), C.byref(args)), "triaccel_step")


def triaccel_result(handle) -> StepResult:
    lib = load_library()
    res = StepResult()
    res.struct_size = C.sizeof(StepResult)
    _check(lib.triaccel_result(handle, C.byref(res)), "triaccel_result")
    return res


def triaccel_layer_state(handle, n: int):
    lib = load_library()
    arr = (LayerInfo * n)()
    _check(lib.triaccel_layer_state(handle, arr, n), "triaccel_layer_state")
    return arr


def triaccel_batch_next(config: Config, batch_size: int, mem_used_bytes: int, mem_total_bytes: int) -> int:
    return load_library().triaccel_batch_next(C.byref(config), batch_size, mem_used_bytes, mem_total_bytes)


def triaccel_destroy(handle) -> None:
    load_library().triaccel_destroy(handle)


def triaccel_strerror(code: int) -> str:
    return load_library().triaccel_strerror(code).decode()


def triaccel_set_profiling(handle, on) -> None:
    _check(load_library().triaccel_set_profiling(handle, int(on)), "triaccel_set_profiling")


def triaccel_set_graph(handle, on: bool) -> None:
    _check(load_library().triaccel_set_graph(handle, int(on)), "triaccel_set_graph")


def triaccel_stage_times_get(handle, steps_back: int = 0):
    st = StageTimes()
    _check(load_library().triaccel_stage_times_get(handle, steps_back, C.byref(st)), "triaccel_stage_times_get")
    return list(st.ms)


def triaccel_cast_f32(src_ptr: int, dst_ptr: int, n: int, dtype: int, stream: int = 0) -> None:
    _check(load_library().triaccel_cast_f32(C.c_void_p(src_ptr), C.c_void_p(dst_ptr), n, dtype, C.c_void_p(stream)),
           "triaccel_cast_f32")


def triaccel_power_iter(handle, vectors, k: int, latch: bool) -> None:
    """``vectors`` is a ctypes array ``(PowerTensor * n)`` or a sequence of ``PowerTensor``."""
    arr = vectors if isinstance(vectors, C.Array) else (PowerTensor * len(vectors))(*vectors)
    _check(load_library().triaccel_power_iter(handle, arr, len(arr), k, int(latch)), "triaccel_power_iter")


def triaccel_power_iter_static(vectors, numel: Sequence[int], k: int, info_ptr: int, stream: int = 0) -> None:
    """The power iteration without a handle and without allocations.  ``vectors`` as for
    ``triaccel_power_iter``; ``info_ptr`` is the device address of ``len(vectors)`` PowerInfo records."""
    arr = vectors if isinstance(vectors, C.Array) else (PowerTensor * len(vectors))(*vectors)
    ns = (C.c_int64 * len(arr))(*numel)
    _check(load_library().triaccel_power_iter_static(arr, ns, len(arr), k, C.c_void_p(info_ptr), C.c_void_p(stream)),
           "triaccel_power_iter_static")


def triaccel_power_state(handle, n: int):
    arr = (PowerInfo * n)()
    _check(load_library().triaccel_power_state(handle, arr, n), "triaccel_power_state")
    return arr


def triaccel_power_times_get(handle):
    ms = (C.c_float * 3)()
    _check(load_library().triaccel_power_times_get(handle, ms), "triaccel_power_times_get")
    return list(ms)


def triaccel_get_state(handle) -> bytes:
    lib = load_library()
    size = lib.triaccel_state_size(handle)
    if size < 0:
        raise TriAccelError(int(size), "triaccel_state_size")
    buf = C.create_string_buffer(size)
    _check(lib.triaccel_get_state(handle, buf, size), "triaccel_get_state")
    return buf.raw


def triaccel_set_state(handle, blob: bytes) -> None:
    _check(load_library().triaccel_set_state(handle, blob, len(blob)), "triaccel_set_state")
