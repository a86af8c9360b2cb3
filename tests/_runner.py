"""Drive a workload through the CPU oracle (shared by the CPU tests and the GPU parity tests)."""
import numpy as np
import torch

import oracle


def to_numpy(t: torch.Tensor) -> np.ndarray:
    """Bit-preserving view of a (CPU or GPU) tensor as numpy: 2-byte floats become uint16."""
    t = t.detach().cpu().contiguous()
    if t.dtype in (torch.float16, torch.bfloat16):
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def make_oracle(wl, tensors=None, workers=1, grad_dtypes=None):
    """``grad_dtypes``: gradient precision per tensor of the workload (default: the workload's one)."""
    idx = list(range(wl.n_tensors)) if tensors is None else list(tensors)
    cfg = oracle.OracleConfig.from_hyper(wl.hyper)
    params = [to_numpy(wl.init_param(l)) for l in idx]
    return oracle.OracleTriAccel(cfg, params, [wl.init_dtype(l) for l in idx],
                                 [wl.grad_dtype if grad_dtypes is None else grad_dtypes[l] for l in idx], workers=workers)


def layer_record(t):
    return dict(mean=float(t.mean), var=float(t.var), v=float(t.v), theta=float(t.theta), nnz=int(t.nnz),
                lam=float(t.lam), eta=float(t.eta), code=int(t.code), prev_code=int(t.prev_code),
                found_inf=int(t.found_inf), curv_nonfinite=int(t.curv_nonfinite))


def run_oracle(wl, steps=None, probe_every=1, mem=(0.8, 1.0), workers=1):
    """Run ``steps`` steps; returns (oracle object, list of per-step dicts)."""
    orc = make_oracle(wl, workers=workers)
    steps = wl.steps if steps is None else steps
    scale = float(wl.hyper["loss_scale"])
    batch = int(wl.hyper["batch_size"])
    hist = []
    for t in range(1, steps + 1):
        grads = [to_numpy(wl.grad(t, l, scale)) for l in range(wl.n_tensors)]
        if (t - 1) % probe_every == 0:
            pr = [wl.probe(t, l, scale) for l in range(wl.n_tensors)]
            zs, hzs = [to_numpy(p[0]) for p in pr], [to_numpy(p[1]) for p in pr]
        else:
            zs = hzs = [None] * wl.n_tensors
        total = 1 << 30
        res = orc.step(grads, zs, hzs, wl.hyper["lr"], scale, batch, int(mem[0] * total), int(mem[1] * total))
        res["loss_scale"] = scale
        res["layers"] = [layer_record(x) for x in orc.tensors]
        hist.append(res)
        scale, batch = res["next_loss_scale"], res["next_batch_size"]
    return orc, hist


def decision_margin(hist, hyper, rel=1e-6):
    """Smallest relative distance of any smoothed variance to a precision threshold."""
    worst = np.inf
    for res in hist:
        if res["skipped"]:
            continue
        for rec in res["layers"]:
            for tau in (hyper["tau_low"], hyper["tau_high"]):
                worst = min(worst, abs(rec["v"] - np.float32(tau)) / float(np.float32(tau)))
    return worst
