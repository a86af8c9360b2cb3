"""Pins for the sequencing of one oracle step (the control loop of Sec. 3.4): skip-step leaves
every state byte untouched, carry-over without a probe, control interval, and the acceptance
checks of the synthetic workloads."""
import copy

import numpy as np
import pytest

import oracle
from workloads import get_workload
from _runner import decision_margin, make_oracle, run_oracle, to_numpy

FP16, BF16, FP32 = 0, 1, 2


def snapshot(orc):
    return [(t.buf.copy(), t.curv.copy(), None if t.mom is None else t.mom.copy(), t.mask.copy(),
             (t.v, t.code, t.prev_code, t.eta, t.theta, t.nnz, t.lam, t.lam_ctrl, t.mean, t.var, t.probes_seen))
            for t in orc.tensors]


def same(a, b):
    for (b1, c1, m1, k1, s1), (b2, c2, m2, k2, s2) in zip(a, b):
        if not (np.array_equal(b1, b2) and np.array_equal(c1, c2) and np.array_equal(k1, k2)):
            return False
        if (m1 is None) != (m2 is None) or (m1 is not None and not np.array_equal(m1, m2)):
            return False
        if s1 != s2:
            return False
    return True


def inputs(wl, t, scale=1.0):
    g = [to_numpy(wl.grad(t, l, scale)) for l in range(wl.n_tensors)]
    pr = [wl.probe(t, l, scale) for l in range(wl.n_tensors)]
    return g, [to_numpy(p[0]) for p in pr], [to_numpy(p[1]) for p in pr]


@pytest.mark.parametrize("bad", [np.inf, -np.inf, np.nan])
def test_skip_step_changes_no_state(bad):
    wl = get_workload("tiny_mlp")
    orc = make_oracle(wl)
    for t in (1, 2):
        g, z, hz = inputs(wl, t)
        assert orc.step(g, z, hz, 0.1, 1024.0, 96, 0, 100)["skipped"] == 0
    before = snapshot(orc)
    applied = orc.applied_steps
    g, z, hz = inputs(wl, 3)
    g[2][17] = bad
    res = orc.step(g, z, hz, 0.1, 1024.0, 96, 0, 100)
    assert res["skipped"] == 1 and res["next_loss_scale"] == 512.0
    assert [t.found_inf for t in orc.tensors] == [0, 0, 1, 0]
    assert same(before, snapshot(orc)) and orc.applied_steps == applied
    # the next clean step proceeds from the untouched state
    g, z, hz = inputs(wl, 3)
    res = orc.step(g, z, hz, 0.1, 512.0, 96, 0, 100)
    assert res["skipped"] == 0 and not same(before, snapshot(orc))


def test_loss_scale_grows_after_the_interval():
    wl = get_workload("tiny_mlp")
    wl.hyper = dict(wl.hyper, growth_interval=3)
    orc = make_oracle(wl)
    scale, seen = 8.0, []
    for t in range(1, 8):
        g, z, hz = inputs(wl, t, scale)
        scale = orc.step(g, z, hz, 0.1, scale, 96, 0, 100)["next_loss_scale"]
        seen.append(scale)
    assert seen == [8, 8, 16, 16, 16, 32, 32]


def test_without_a_probe_curvature_outputs_carry_over():
    wl = get_workload("tiny_mlp")
    orc = make_oracle(wl)
    g, z, hz = inputs(wl, 1)
    none = [None] * wl.n_tensors
    orc.step(g, none, none, 0.1, 1.0, 96, 0, 100)
    for t in orc.tensors:  # never probed: empty mask, theta = lambda = 0, eta = lr
        assert t.nnz == 0 and t.theta == 0 and t.lam == 0 and not t.mask.any() and t.eta == np.float32(0.1)
    orc.step(g, z, hz, 0.1, 1.0, 96, 0, 100)
    kept = [(t.curv.copy(), t.mask.copy(), t.theta, t.lam, t.nnz) for t in orc.tensors]
    assert all(k[4] > 0 for k in kept)
    g2, _, _ = inputs(wl, 2)
    orc.step(g2, none, none, 0.1, 1.0, 96, 0, 100)
    for t, k in zip(orc.tensors, kept):
        assert np.array_equal(t.curv, k[0]) and np.array_equal(t.mask, k[1]) and (t.theta, t.lam, t.nnz) == k[2:]


def test_first_probe_initialises_then_ema():
    wl = get_workload("tiny_mlp")
    orc = make_oracle(wl)
    g, z, hz = inputs(wl, 1)
    orc.step(g, z, hz, 0.1, 1.0, 96, 0, 100)
    t = orc.tensors[2]
    assert np.array_equal(t.curv, z[2] * hz[2])


def test_control_interval_latches_codes_and_curvature():
    wl = get_workload("tiny_mlp")
    wl.hyper = dict(wl.hyper, ctrl_interval=3)
    orc = make_oracle(wl)
    codes, etas = [], []
    for t in range(1, 8):
        g, z, hz = inputs(wl, t)
        orc.step(g, z, hz, 0.1 / t, 1.0, 96, 0, 100)
        codes.append([x.code for x in orc.tensors])
        etas.append([float(x.eta) for x in orc.tensors])
    assert codes[0] == codes[1] == [FP32] * 4          # initial storage dtype until the first control step
    assert etas[0] == [float(np.float32(0.1))] * 4      # no curvature latched yet: eta = lr
    assert codes[2] != codes[1] and codes[2] == codes[3] == codes[4]
    # the base learning rate of each step is used even between control steps
    lam3 = [x for x in [orc.tensors[i].lam_ctrl for i in range(4)]]
    L = oracle.lib()
    want = [L.oracle_eta(np.float32(0.1 / 7), np.float32(wl.hyper["alpha"]), l) for l in lam3]
    assert etas[6] == want


def test_batch_size_follows_memory():
    wl = get_workload("tiny_mlp")
    orc = make_oracle(wl)
    g, z, hz = inputs(wl, 1)
    assert orc.step(g, z, hz, 0.1, 1.0, 96, 10, 100)["next_batch_size"] == 112
    assert orc.step(g, z, hz, 0.1, 1.0, 112, 95, 100)["next_batch_size"] == 96
    assert orc.step(g, z, hz, 0.1, 1.0, 96, 80, 100)["next_batch_size"] == 96


def test_tiny_mlp_workload_acceptance():
    wl = get_workload("tiny_mlp")
    orc, hist = run_oracle(wl)
    assert len(hist) == 20 and not any(h["skipped"] for h in hist)
    codes = {rec["code"] for h in hist for rec in h["layers"]}
    assert codes == {FP16, BF16, FP32}
    assert decision_margin(hist, wl.hyper) > 1e-4
    # mask lies inside the support of the non-zero Hessian blocks (sparsity target 90 %)
    for l, t in enumerate(orc.tensors):
        diag = wl.hessian_diagonal(l)
        assert not (t.mask_bits() & (diag == 0)).any()
        assert t.nnz > 0
