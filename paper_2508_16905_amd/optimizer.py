"""Convenience wrapper that holds PyTorch-ROCm tensors and hands their device pointers to the
C ABI.  PyTorch is used for device memory and the stream only; no arithmetic happens here."""

from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as B

_TORCH_DTYPE = {B.FP16: torch.float16, B.BF16: torch.bfloat16, B.FP32: torch.float32}
_CODE = {v: k for k, v in _TORCH_DTYPE.items()}


class TriAccel:
    """State of one optimizer instance: per tensor a 4*numel-byte parameter buffer, curvature EMA,
    momentum buffer and bit mask, all on the GPU."""

    def __init__(self, hyper: dict, params: Sequence[torch.Tensor], grad_dtype=B.FP32,
                 stream: Optional[torch.cuda.Stream] = None):
        """``grad_dtype``: precision code of the gradients, one for all tensors or one per tensor."""
        if not torch.cuda.is_available():
            raise RuntimeError("TriAccel needs a GPU: the optimizer step runs only in the HIP library")
        B.load_library()
        self.hyper = dict(hyper)
        self.config = B.Config.from_hyper(hyper)
        self.device = params[0].device
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        self.n = len(params)
        self.numel = [int(p.numel()) for p in params]
        self.grad_dtype = ([int(grad_dtype)] * self.n if isinstance(grad_dtype, int)
                           else [int(d) for d in grad_dtype])
        if len(self.grad_dtype) != self.n:
            raise ValueError("grad_dtype: one code, or one per tensor")
        self.init_codes = [_CODE[p.dtype] for p in params]
        self.buf: List[torch.Tensor] = []
        for p, n in zip(params, self.numel):
            raw = torch.zeros(4 * n, dtype=torch.uint8, device=self.device)
            raw.view(p.dtype)[:n].copy_(p.reshape(-1))
            self.buf.append(raw)
        use_mom = hyper["momentum"] != 0.0
        self.curv = [torch.zeros(n, dtype=torch.float32, device=self.device) for n in self.numel]
        self.mom = [torch.zeros(n, dtype=torch.float32, device=self.device) if use_mom else None for n in self.numel]
        self.mask = [torch.zeros((n + 31) // 32, dtype=torch.int32, device=self.device) for n in self.numel]
        self._tensors = (B.Tensor * self.n)()
        for i in range(self.n):
            t = self._tensors[i]
            t.param = self.buf[i].data_ptr()
            t.curv = self.curv[i].data_ptr()
            t.mom = self.mom[i].data_ptr() if use_mom else None
            t.mask = self.mask[i].data_ptr()
            t.numel = self.numel[i]
            t.grad_dtype = self.grad_dtype[i]
            t.param_dtype = self.init_codes[i]
        # init validates grad pointers too: give it any valid address (the parameter buffer)
        for i in range(self.n):
            self._tensors[i].grad = self.buf[i].data_ptr()
        torch.cuda.synchronize(self.device)
        self.handle = B.triaccel_init(self.config, self._tensors, self.stream.cuda_stream)
        self._keep = None

    def step(self, grads: Sequence[torch.Tensor], zs: Optional[Sequence[Optional[torch.Tensor]]] = None,
             hzs: Optional[Sequence[Optional[torch.Tensor]]] = None, lr: float = 0.1, loss_scale: float = 1.0,
             batch_size: int = 0, mem_used_bytes: int = 0, mem_total_bytes: int = 0,
             update_curvature: bool = True) -> None:
        """Enqueue one step (asynchronous).  The caller keeps ``grads``/``zs``/``hzs`` alive until
        the stream has passed the step; a reference is also held here until the next call."""
        for i in range(self.n):
            t = self._tensors[i]
            t.grad = grads[i].data_ptr()
            z = None if zs is None else zs[i]
            t.z = None if z is None else z.data_ptr()
            t.hz = None if z is None else hzs[i].data_ptr()
        self._keep = (grads, zs, hzs)
        B.triaccel_step(self.handle, self._tensors, lr, loss_scale, batch_size, mem_used_bytes, mem_total_bytes,
                        update_curvature)

    def make_table(self, grads: Sequence[torch.Tensor], zs: Optional[Sequence[Optional[torch.Tensor]]] = None,
                   hzs: Optional[Sequence[Optional[torch.Tensor]]] = None):
        """The tensor table of ``step`` for one set of input buffers, marshalled once: a caller whose
        gradient and probe buffers stay where they are (the usual case in a training loop) passes it to
        ``step_table`` at every step instead of paying for the per-tensor marshalling again."""
        arr = (B.Tensor * self.n)()
        for i in range(self.n):
            src, t = self._tensors[i], arr[i]
            t.param, t.curv, t.mom, t.mask = src.param, src.curv, src.mom, src.mask
            t.numel, t.grad_dtype, t.param_dtype = src.numel, src.grad_dtype, src.param_dtype
            t.grad = grads[i].data_ptr()
            z = None if zs is None else zs[i]
            t.z = None if z is None else z.data_ptr()
            t.hz = None if z is None else hzs[i].data_ptr()
        return arr, (grads, zs, hzs)   # the buffers stay alive as long as the table does

    def step_table(self, table, lr: float = 0.1, loss_scale: float = 1.0, batch_size: int = 0,
                   mem_used_bytes: int = 0, mem_total_bytes: int = 0, update_curvature: bool = True) -> None:
        """``step`` with a table prepared by ``make_table``."""
        self._keep = table
        B.triaccel_step(self.handle, table[0], lr, loss_scale, batch_size, mem_used_bytes, mem_total_bytes,
                        update_curvature)

    def result(self) -> B.StepResult:
        return B.triaccel_result(self.handle)

    def layer_state(self):
        return B.triaccel_layer_state(self.handle, self.n)

    def power_iter(self, us: Sequence[torch.Tensor], hus: Sequence[torch.Tensor], k: int, latch: bool = False) -> None:
        """Enqueue one power iteration (asynchronous).  ``us[i]`` and ``hus[i]`` are fp32 tensors of
        shape (k, stride_i) with stride_i >= numel_i a multiple of 4; ``us[i]`` is overwritten."""
        arr = (B.PowerTensor * self.n)()
        for i in range(self.n):
            assert us[i].dtype == torch.float32 and hus[i].dtype == torch.float32
            assert us[i].shape == hus[i].shape and us[i].shape[0] >= k and us[i].is_contiguous() and hus[i].is_contiguous()
            arr[i].u = us[i].data_ptr()
            arr[i].hu = hus[i].data_ptr()
            arr[i].stride = us[i].shape[1]
        self._keep_power = (us, hus)
        B.triaccel_power_iter(self.handle, arr, k, latch)

    def power_state(self):
        return B.triaccel_power_state(self.handle, self.n)

    def power_times(self):
        """[Gram pass, per-layer kernel, apply pass] in ms of the last power_iter call (profiling on)."""
        return B.triaccel_power_times_get(self.handle)

    def get_state(self) -> bytes:
        """The library's own state (per-layer records, counters); the tensors are saved by the caller."""
        return B.triaccel_get_state(self.handle)

    def set_state(self, blob: bytes) -> None:
        B.triaccel_set_state(self.handle, blob)

    def param(self, i: int, code: int) -> torch.Tensor:
        """View of tensor ``i``'s stored parameters as precision ``code`` (take it from layer_state)."""
        return self.buf[i].view(_TORCH_DTYPE[code])[: self.numel[i]]

    def set_graph(self, on: bool) -> None:
        """Replay the step as a HIP graph instead of launching its kernels one by one."""
        B.triaccel_set_graph(self.handle, on)

    def set_profiling(self, level: int) -> None:
        """0 off; 1 a HIP event at every stage boundary; 2 events around the update kernel only."""
        B.triaccel_set_profiling(self.handle, int(level))

    def stage_times(self, steps_back: int = 0):
        return B.triaccel_stage_times_get(self.handle, steps_back)

    def close(self) -> None:
        if self.handle is not None:
            B.triaccel_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
