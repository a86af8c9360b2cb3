"""Lock-step driver: the HIP library and the CPU oracle consume the same seeded inputs and every
output is compared after every step.

Bars (written here once, used by every parity test):
  * masks, precision codes, skip / overflow flags, nnz: bit-exact;
  * theta, lambda, eta (order statistic / max / fixed fp32 operations): bit-exact;
  * curvature state h, momentum m, parameters (fp32 or the rounded bf16 / fp16 stores): bit-exact
    -- both sides use the same fp32 operation order, so the stricter bar is used instead of the
    1e-5 relative one;
  * mean, variance, variance EMA (reductions; fp64 on both sides, different summation order):
    |gpu - oracle| <= 1e-5 * max(|oracle|, sqrt(var)) for the mean and 1e-5 relative otherwise.
"""
import numpy as np
import torch

import paper_2508_16905_amd as ta
from _runner import make_oracle, to_numpy
from workloads.configs import TORCH_DTYPE

STAT_RTOL = 1e-5
DECISION_MARGIN = 1e-4  # ten times the tolerance of the statistics


def bits_equal(a: np.ndarray, b: np.ndarray) -> bool:
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    if a.dtype == np.float32:
        a, b = a.view(np.uint32), b.view(np.uint32)
    return a.shape == b.shape and bool(np.array_equal(a, b))


def same_or_both_nan(a: np.ndarray, b: np.ndarray) -> bool:
    """fp32 arrays equal bit for bit, except that any NaN matches any NaN."""
    if bits_equal(a, b):
        return True
    nan = np.isnan(a) & np.isnan(b)
    return bool(np.array_equal(a.view(np.uint32)[~nan], b.view(np.uint32)[~nan]))


class Pair:
    def __init__(self, wl, workers=8, device="cuda:0", graph=False, grad_dtypes=None):
        """``graph``: the library replays the step as a HIP graph (needs a stream of its own).
        ``grad_dtypes``: gradient precision per tensor (the workload's gradients are cast to it)."""
        self.wl = wl
        self.device = torch.device(device)
        self.grad_dtypes = grad_dtypes
        self.orc = make_oracle(wl, workers=workers, grad_dtypes=grad_dtypes)
        params = [wl.init_param(l).to(self.device) for l in range(wl.n_tensors)]
        self.stream = torch.cuda.Stream(device=self.device) if graph else None
        torch.cuda.synchronize()
        self.gpu = ta.TriAccel(wl.hyper, params, grad_dtype=wl.grad_dtype if grad_dtypes is None else grad_dtypes,
                               stream=self.stream)
        if graph:
            self.gpu.set_graph(True)
        self.scale = float(wl.hyper["loss_scale"])
        self.batch = int(wl.hyper["batch_size"])
        self.t = 0
        self.code_hist = []

    def close(self):
        self.gpu.close()

    def inputs(self, t, probe=True):
        wl = self.wl
        grads = [wl.grad(t, l, self.scale) for l in range(wl.n_tensors)]
        if self.grad_dtypes is not None:
            grads = [g.to(TORCH_DTYPE[d]) for g, d in zip(grads, self.grad_dtypes)]
        if probe:
            pr = [wl.probe(t, l, self.scale) for l in range(wl.n_tensors)]
            zs, hzs = [p[0] for p in pr], [p[1] for p in pr]
        else:
            zs = hzs = [None] * wl.n_tensors
        return grads, zs, hzs

    def step(self, grads, zs, hzs, lr=None, mem=(800, 1000), check=True, label="", update_curvature=True,
             margin_check=True):
        """One step on both sides from CPU torch tensors; returns the oracle's result dict.
        ``margin_check=False`` is for hand-made inputs whose statistics are exact on both sides."""
        wl = self.wl
        self.t += 1
        lr = wl.hyper["lr"] if lr is None else lr
        dev = self.device
        g_d = [g.to(dev) for g in grads]
        z_d = [None if z is None else z.to(dev) for z in zs]
        hz_d = [None if h is None else h.to(dev) for h in hzs]
        if self.stream is not None:
            torch.cuda.synchronize()  # the inputs were copied on the default stream
        self.gpu.step(g_d, z_d, hz_d, lr=lr, loss_scale=self.scale, batch_size=self.batch,
                      mem_used_bytes=mem[0], mem_total_bytes=mem[1], update_curvature=update_curvature)
        res_o = self.orc.step([to_numpy(g) for g in grads], [None if z is None else to_numpy(z) for z in zs],
                              [None if h is None else to_numpy(h) for h in hzs], lr, self.scale, self.batch,
                              mem[0], mem[1], update_curvature=update_curvature)
        res_g = self.gpu.result()
        where = f"{wl.name} step {self.t} {label}"
        if not res_o["skipped"] and margin_check:
            # decision stability: a reduction result within the statistics tolerance of a threshold could
            # legitimately give another code; such an input is a flaw of the generated case, not of either side
            for o in self.orc.tensors:
                for tau in (wl.hyper["tau_low"], wl.hyper["tau_high"]):
                    if tau > 0:
                        margin = abs(float(o.v) - float(np.float32(tau))) / float(np.float32(tau))
                        assert margin > DECISION_MARGIN, (where, "variance EMA too close to a threshold", float(o.v), tau)
        assert res_g.skipped == res_o["skipped"], where
        assert res_g.step_index == res_o["step_index"], where
        assert res_g.next_loss_scale == res_o["next_loss_scale"], where
        assert res_g.next_batch_size == res_o["next_batch_size"], where
        if check:
            self.compare(where)
        self.scale, self.batch = res_o["next_loss_scale"], res_o["next_batch_size"]
        self.code_hist.append([t.code for t in self.orc.tensors])
        return res_o

    def compare(self, where=""):
        st = self.gpu.layer_state()
        for l, (o, g) in enumerate(zip(self.orc.tensors, st)):
            w = f"{where} tensor {l} (n={o.numel})"
            assert (g.code, g.prev_code) == (o.code, o.prev_code), w
            assert (g.found_inf, g.curv_nonfinite) == (o.found_inf, o.curv_nonfinite), w
            assert g.nnz == o.nnz, (w, g.nnz, o.nnz)
            for name, gv, ov in (("theta", g.theta, o.theta), ("lambda", g.lambda_, o.lam),
                                 ("lambda_ctrl", g.lambda_ctrl, o.lam_ctrl), ("eta", g.eta, o.eta)):
                assert np.float32(gv).view(np.uint32) == np.float32(ov).view(np.uint32), (w, name, gv, ov)
            sd = float(np.sqrt(max(float(o.var), 0.0)))
            assert abs(g.mean - float(o.mean)) <= STAT_RTOL * max(abs(float(o.mean)), sd) + 1e-45, (w, g.mean, o.mean)
            assert abs(g.var - float(o.var)) <= STAT_RTOL * abs(float(o.var)) + 1e-45, (w, g.var, o.var)
            assert abs(g.v - float(o.v)) <= STAT_RTOL * abs(float(o.v)) + 1e-45, (w, g.v, o.v)
            assert bits_equal(self.gpu.mask[l].cpu().numpy().view(np.uint32), o.mask), w + " mask"
            assert bits_equal(self.gpu.curv[l].cpu().numpy(), o.curv), w + " curvature state"
            if o.mom is not None:
                assert same_or_both_nan(self.gpu.mom[l].cpu().numpy(), o.mom), w + " momentum"
            gp = to_numpy(self.gpu.param(l, g.code))
            op = o.param_view()
            if o.code == 2:
                assert same_or_both_nan(gp, op), w + " parameters"
            else:
                assert bits_equal(gp, op), w + " parameters (low-precision store)"

    def run(self, steps, probe_every=1, start=1):
        for t in range(start, start + steps):
            g, z, hz = self.inputs(t, probe=(t - 1) % probe_every == 0)
            self.step(g, z, hz)
        return self
