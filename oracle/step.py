"""One Tri-Accel optimizer step on the CPU, in the order the control loop of the paper's
Sec. 3.4 lists its stages -- TEST INFRASTRUCTURE ONLY.

The arithmetic of every stage is in ``triaccel_oracle.c``; this module only holds
the state (numpy arrays) and calls the stages one after another, tensor by tensor.
"""

from __future__ import annotations

import ctypes as C
from dataclasses import dataclass, fields
from typing import List, Optional, Sequence

import numpy as np

from .capi import lib

FP16, BF16, FP32 = 0, 1, 2
_NP = {FP16: np.uint16, BF16: np.uint16, FP32: np.float32}


@dataclass
class OracleConfig:
    beta_var: float = 0.9        # beta of the variance EMA, Sec. 3.1
    beta_curv: float = 0.9       # smoothing of the curvature EMA
    tau_low: float = 1e-5        # Sec. 3.1 thresholds
    tau_high: float = 3e-5
    tau_curv: float = 1.0        # Sec. 3.2 promotion threshold
    alpha: float = 0.1           # Sec. 3.2 step-size coefficient
    sparsity_ppm: int = 900000
    topk_abs: int = 0            # > 0: keep this many entries per layer instead of a fraction (Sec. 4.1: k = 5)
    momentum: float = 0.9        # Sec. 4.1 baseline optimizer
    weight_decay: float = 5e-4
    ctrl_interval: int = 1       # T_ctrl, Sec. 3.4
    scale_backoff: float = 0.5
    scale_growth: float = 2.0
    growth_interval: int = 2000
    rho_low: float = 0.70        # Sec. 3.3
    rho_high: float = 0.90
    delta_up: int = 16
    delta_down: int = 16
    b_min: int = 16
    b_max: int = 4096
    curvature_source: int = 0    # sample behind the diagonal EMA: 0 = Hutchinson pair z * Hz, 1 = squared gradient
    elementwise_scale: int = 0   # 1: the step size is scaled per element by the masked |h_i| instead of per layer
    lambda_source: int = 0       # lambda_l of Sec. 3.2: 0 = largest kept |h_i| of the diagonal EMA,
                                 # 1 = largest |Rayleigh quotient| of the latched power iteration

    @classmethod
    def from_hyper(cls, hyper: dict) -> "OracleConfig":
        names = {f.name for f in fields(cls)}
        return cls(**{k: v for k, v in hyper.items() if k in names})


class OracleTensor:
    """State of one parameter tensor ("layer")."""

    def __init__(self, param: np.ndarray, param_dtype: int, grad_dtype: int, momentum: bool):
        n = int(param.size)
        self.numel = n
        self.grad_dtype = int(grad_dtype)
        self.code = int(param_dtype)
        self.prev_code = int(param_dtype)
        self.buf = np.zeros(4 * n, dtype=np.uint8)  # capacity 4n bytes, like the device buffer
        self.param_view()[:] = np.ascontiguousarray(param).view(_NP[self.code]).reshape(-1)
        self.curv = np.zeros(n, dtype=np.float32)
        self.mom = np.zeros(n, dtype=np.float32) if momentum else None
        self.mask = np.zeros((n + 31) // 32, dtype=np.uint32)
        self.mean = np.float32(0)
        self.var = np.float32(0)
        self.v = np.float32(0)
        self.theta = np.float32(0)
        self.nnz = 0
        self.lam = np.float32(0)
        self.lam_ctrl = np.float32(0)
        self.eta = np.float32(0)
        self.found_inf = 0
        self.curv_nonfinite = 0
        self.probes_seen = 0
        # power iteration (Sec. 3.2, third equation)
        self.rayleigh = np.zeros(0, dtype=np.float32)
        self.resid = np.zeros(0, dtype=np.float32)
        self.hnorm = np.zeros(0, dtype=np.float32)
        self.deficient = 0
        self.lam_power = np.float32(0)

    def param_view(self) -> np.ndarray:
        """The stored parameters in their current dtype (uint16 bit patterns for 2-byte codes)."""
        return self.buf.view(_NP[self.code])[: self.numel]

    def param_f32(self) -> np.ndarray:
        """Stored parameters widened to fp32 (exact)."""
        v = self.param_view()
        if self.code == FP32:
            return v.copy()
        if self.code == BF16:
            return (v.astype(np.uint32) << 16).view(np.float32)
        out = np.empty(self.numel, dtype=np.float32)
        lib().oracle_f16_to_f32_array(v.ctypes.data, out.ctypes.data, self.numel)
        return out

    def mask_bits(self) -> np.ndarray:
        return np.unpackbits(self.mask.view(np.uint8), bitorder="little")[: self.numel].astype(bool)


class OracleTriAccel:
    def __init__(self, config: OracleConfig, params: Sequence[np.ndarray], param_dtypes: Sequence[int],
                 grad_dtypes: Sequence[int], workers: int = 1):
        self.cfg = config
        self.workers = int(workers)
        self._executor = None
        self.tensors: List[OracleTensor] = [
            OracleTensor(p, d, gd, config.momentum != 0.0) for p, d, gd in zip(params, param_dtypes, grad_dtypes)
        ]
        self.applied_steps = 0   # steps that were not skipped
        self.step_index = 0      # all calls
        self.good_steps = C.c_int32(0)

    def _pool(self):
        if self._executor is None:
            from concurrent.futures import ThreadPoolExecutor

            self._executor = ThreadPoolExecutor(self.workers)
        return self._executor

    def _tensor_step(self, t, g, z, hz, lr, inv_scale, control_step, first, update_curvature):
        L, cfg, f32 = lib(), self.cfg, np.float32
        # (1) collect per-layer gradient variance ...
        mean, var = C.c_double(), C.c_double()
        L.oracle_grad_stats(g.ctypes.data, t.grad_dtype, t.numel, inv_scale, C.byref(mean), C.byref(var))
        t.mean, t.var = f32(mean.value), f32(var.value)
        t.v = f32(L.oracle_var_ema(t.v, var.value, f32(cfg.beta_var), int(first)))
        # ... and curvature statistics
        t.curv_nonfinite = 0
        fisher = cfg.curvature_source == 1
        if (update_curvature if fisher else z is not None):
            flag = C.c_uint32(0)
            if fisher:
                L.oracle_fisher_ema(g.ctypes.data, t.grad_dtype, t.curv.ctypes.data, t.numel, inv_scale,
                                    f32(cfg.beta_curv), int(t.probes_seen == 0), C.byref(flag))
            else:
                L.oracle_curv_ema(z.ctypes.data, hz.ctypes.data, t.curv.ctypes.data, t.numel, inv_scale,
                                  f32(cfg.beta_curv), int(t.probes_seen == 0), C.byref(flag))
            t.curv_nonfinite = int(flag.value)
            t.probes_seen += 1
            theta, nnz, lam = C.c_float(), C.c_uint32(), C.c_float()
            if cfg.topk_abs > 0:
                L.oracle_threshold_mask_k(t.curv.ctypes.data, t.numel, int(cfg.topk_abs), t.mask.ctypes.data,
                                          C.byref(theta), C.byref(nnz), C.byref(lam))
            else:
                L.oracle_threshold_mask(t.curv.ctypes.data, t.numel, cfg.sparsity_ppm, t.mask.ctypes.data,
                                        C.byref(theta), C.byref(nnz), C.byref(lam))
            t.theta, t.nnz, t.lam = f32(theta.value), int(nnz.value), f32(lam.value)
        if cfg.lambda_source == 1:
            t.lam = t.lam_power
        # (2) precision allocation, (3) per-layer learning rate
        t.prev_code = t.code
        if control_step:
            t.lam_ctrl = t.lam
            t.code = int(L.oracle_precision_code(t.v, t.lam_ctrl, f32(cfg.tau_low), f32(cfg.tau_high),
                                                 f32(cfg.tau_curv)))
        t.eta = f32(L.oracle_eta(f32(lr), f32(cfg.alpha), t.lam_ctrl))
        # update and store in the chosen precision
        if cfg.elementwise_scale == 1:
            L.oracle_update_elementwise(t.buf.ctypes.data, t.prev_code, t.code, g.ctypes.data, t.grad_dtype,
                                        None if t.mom is None else t.mom.ctypes.data, t.curv.ctypes.data,
                                        t.mask.ctypes.data, t.numel, inv_scale, f32(cfg.weight_decay),
                                        f32(cfg.momentum), f32(lr), f32(cfg.alpha))
        else:
            L.oracle_update(t.buf.ctypes.data, t.prev_code, t.code, g.ctypes.data, t.grad_dtype,
                            None if t.mom is None else t.mom.ctypes.data, t.numel, inv_scale,
                            f32(cfg.weight_decay), f32(cfg.momentum), t.eta)

    def power_step(self, us: Sequence[np.ndarray], hus: Sequence[np.ndarray], k: int, latch: bool) -> None:
        """One power iteration (Sec. 3.2) per tensor on k supplied pairs (u_j, H u_j); ``us[l]`` and
        ``hus[l]`` are fp32 arrays of shape (k, numel).  The new vectors overwrite ``us[l]``.  With
        ``latch`` the layer's lambda for the following steps becomes max_j |rayleigh_j|."""
        L = lib()
        for t, u, hu in zip(self.tensors, us, hus):
            assert u.dtype == np.float32 and hu.dtype == np.float32 and u.size == k * t.numel == hu.size
            ray, res, hn = (np.zeros(k, dtype=np.float64) for _ in range(3))
            deficient = C.c_uint32(0)
            out = np.empty(k * t.numel, dtype=np.float32)
            L.oracle_power_step(u.ctypes.data, hu.ctypes.data, out.ctypes.data, t.numel, int(k),
                                ray.ctypes.data_as(C.POINTER(C.c_double)), res.ctypes.data_as(C.POINTER(C.c_double)),
                                hn.ctypes.data_as(C.POINTER(C.c_double)), C.byref(deficient))
            u.reshape(-1)[:] = out
            t.rayleigh, t.resid, t.hnorm = ray.astype(np.float32), res.astype(np.float32), hn.astype(np.float32)
            t.deficient = int(deficient.value)
            if latch:
                t.lam_power = np.float32(np.max(np.abs(ray)))

    def step(self, grads: Sequence[np.ndarray], zs: Sequence[Optional[np.ndarray]],
             hzs: Sequence[Optional[np.ndarray]], lr: float, loss_scale: float, batch_size: int,
             mem_used: int, mem_total: int, overflow_elsewhere: bool = False, update_curvature: bool = True) -> dict:
        """``overflow_elsewhere``: a tensor that this oracle does not hold (when it tracks a subset
        of a larger parameter set) had a non-finite gradient, so the step is skipped for all.
        ``update_curvature``: with ``curvature_source == 1``, whether this step updates the EMA."""
        L, cfg = lib(), self.cfg
        f32 = np.float32
        inv_scale = f32(1.0) / f32(loss_scale)
        self.step_index += 1

        # overflow detection on the stored gradients; all-or-nothing skip
        for t, g in zip(self.tensors, grads):
            t.found_inf = int(L.oracle_found_nonfinite(g.ctypes.data, t.grad_dtype, t.numel))
        skipped = int(any(t.found_inf for t in self.tensors) or overflow_elsewhere)

        if not skipped:
            self.applied_steps += 1
            control_step = self.applied_steps % cfg.ctrl_interval == 0
            first = self.applied_steps == 1

            def one(args):
                self._tensor_step(*args, lr=lr, inv_scale=inv_scale, control_step=control_step, first=first,
                                  update_curvature=update_curvature)

            work = list(zip(self.tensors, grads, zs, hzs))
            if self.workers > 1:
                # tensors are independent once the skip decision is known; threads only spread them
                # over cores, the arithmetic per tensor is unchanged
                list(self._pool().map(one, work))
            else:
                for w in work:
                    one(w)

        next_scale = L.oracle_loss_scale_next(f32(loss_scale), skipped, C.byref(self.good_steps),
                                              f32(cfg.scale_backoff), f32(cfg.scale_growth),
                                              int(cfg.growth_interval))
        # (4) batch size from memory usage
        next_batch = L.oracle_batch_next(int(batch_size), int(mem_used), int(mem_total), cfg.rho_low, cfg.rho_high,
                                         cfg.delta_up, cfg.delta_down, cfg.b_min, cfg.b_max)
        return dict(skipped=skipped, step_index=self.step_index, next_loss_scale=float(next_scale),
                    next_batch_size=int(next_batch))
