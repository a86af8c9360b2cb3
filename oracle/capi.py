"""Build and load the C oracle (test infrastructure only)."""

from __future__ import annotations

import ctypes as C
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "triaccel_oracle.c")
_SO = os.path.join(_HERE, "liboracle.so")
_SAN_SO = os.path.join(_HERE, "liboracle_san.so")
_lib = None


def build(force: bool = True, sanitize: bool = False) -> str:
    """Compile the oracle with gcc.  No contraction, no fast-math; fmaf() maps to the
    hardware fused multiply-add when the host has one (same result as libm's).
    ``sanitize``: a second library, ``liboracle_san.so``, instrumented with AddressSanitizer and
    UndefinedBehaviorSanitizer (every report is fatal); a process loads it instead of the plain one
    when TRIACCEL_ORACLE_SO names it, and must then have the ASan runtime preloaded."""
    so = _SAN_SO if sanitize else _SO
    if not force and os.path.exists(so) and os.path.getmtime(so) >= os.path.getmtime(_SRC):
        return so
    cmd = ["gcc", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math"]
    cmd += ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"] \
        if sanitize else ["-O2"]
    try:
        with open("/proc/cpuinfo") as f:
            if " fma " in f.read():
                cmd.append("-mfma")
    except OSError:
        pass
    cmd += ["-o", so, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return so


def lib() -> C.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    override = os.environ.get("TRIACCEL_ORACLE_SO")
    if override:
        L = C.CDLL(override)  # an instrumented build of the same source (sanitizer run of the pins)
    else:
        build(force=False)
        L = C.CDLL(_SO)
    vp, i64, i32, u32, f32, f64 = C.c_void_p, C.c_int64, C.c_int32, C.c_uint32, C.c_float, C.c_double
    u64 = C.c_uint64
    P = C.POINTER
    sig = {
        "oracle_f16_to_f32": (f32, [C.c_uint16]),
        "oracle_bf16_to_f32": (f32, [C.c_uint16]),
        "oracle_f32_to_f16": (C.c_uint16, [f32]),
        "oracle_f32_to_bf16": (C.c_uint16, [f32]),
        "oracle_f32_to_f16_array": (None, [vp, vp, i64]),
        "oracle_f32_to_bf16_array": (None, [vp, vp, i64]),
        "oracle_f16_to_f32_array": (None, [vp, vp, i64]),
        "oracle_found_nonfinite": (C.c_int, [vp, C.c_int, i64]),
        "oracle_grad_stats": (None, [vp, C.c_int, i64, f32, P(f64), P(f64)]),
        "oracle_var_ema": (f32, [f32, f64, f32, C.c_int]),
        "oracle_curv_ema": (None, [vp, vp, vp, i64, f32, f32, C.c_int, P(u32)]),
        "oracle_fisher_ema": (None, [vp, C.c_int, vp, i64, f32, f32, C.c_int, P(u32)]),
        "oracle_topk_count": (i64, [i64, u32]),
        "oracle_threshold_mask": (None, [vp, i64, u32, vp, P(f32), P(u32), P(f32)]),
        "oracle_threshold_mask_k": (None, [vp, i64, i64, vp, P(f32), P(u32), P(f32)]),
        "oracle_precision_code": (C.c_int, [f32, f32, f32, f32, f32]),
        "oracle_eta": (f32, [f32, f32, f32]),
        "oracle_update": (None, [vp, C.c_int, C.c_int, vp, C.c_int, vp, i64, f32, f32, f32, f32]),
        "oracle_update_elementwise": (None, [vp, C.c_int, C.c_int, vp, C.c_int, vp, vp, vp, i64, f32, f32, f32, f32, f32]),
        "oracle_loss_scale_next": (f32, [f32, C.c_int, P(i32), f32, f32, i32]),
        "oracle_batch_next": (i32, [i32, u64, u64, f64, f64, i32, i32, i32, i32]),
        "oracle_power_step": (None, [vp, vp, vp, i64, i32, P(f64), P(f64), P(f64), P(u32)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L
