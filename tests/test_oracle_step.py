"""Pins for the sequencing of one oracle step (the control loop of Sec. 3.4): skip-step leaves
every state byte untouched, carry-over without a probe, control interval, and the acceptance
checks of the synthetic workloads."""

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


# ---- sequencing pins on small hand-made cases (plain numpy beside the oracle) ----

def _small(cfg_kw, n=64, dtype=FP32, seed=0):
    rng = np.random.default_rng(seed)
    cfg = oracle.OracleConfig(**cfg_kw)
    p = rng.standard_normal(n).astype(np.float32)
    return oracle.OracleTriAccel(cfg, [p], [dtype], [FP32]), p, rng


def test_variance_ema_starts_at_the_first_applied_step_also_after_a_skipped_one():
    # constant per-step variance is a fixed point of the EMA from the first applied step on (Sec. 3.1)
    orc, _, rng = _small(dict(beta_var=0.9))
    g = rng.standard_normal(64).astype(np.float32)
    bad = g.copy()
    bad[3] = np.inf
    assert orc.step([bad], [None], [None], 0.1, 1.0, 96, 0, 100)["skipped"] == 1
    want = np.float32(np.var(g.astype(np.float64)))
    for _ in range(3):
        assert orc.step([g], [None], [None], 0.1, 1.0, 96, 0, 100)["skipped"] == 0
        assert orc.tensors[0].v == want and orc.tensors[0].var == want


def test_first_probe_initialises_whenever_it_arrives():
    # a diagonal Hessian gives z * Hz = diag(H) exactly; the first probe sets h to it even when the
    # run started without probes, the second one is a fixed point of the EMA
    orc, _, rng = _small(dict(beta_curv=0.9))
    g = rng.standard_normal(64).astype(np.float32)
    diag = rng.uniform(0.5, 2.0, 64).astype(np.float32)
    orc.step([g], [None], [None], 0.1, 1.0, 96, 0, 100)
    for _ in range(2):
        z = rng.choice([-1.0, 1.0], 64).astype(np.float32)
        orc.step([g], [z], [diag * z], 0.1, 1.0, 96, 0, 100)
        assert np.allclose(orc.tensors[0].curv, diag, rtol=2e-7, atol=0)
    orc2, _, _ = _small(dict(beta_curv=0.9))
    z = rng.choice([-1.0, 1.0], 64).astype(np.float32)
    orc2.step([g], [None], [None], 0.1, 1.0, 96, 0, 100)
    orc2.step([g], [z], [diag * z], 0.1, 1.0, 96, 0, 100)
    assert np.array_equal(orc2.tensors[0].curv, diag)


def test_loss_scale_divides_out():
    # a power-of-two loss scale is removed exactly: same state as the unscaled run
    kw = dict(alpha=0.5, tau_low=1e-3, tau_high=1e3)
    a, _, rng = _small(kw)
    b, _, _ = _small(kw)
    for _ in range(3):
        g = rng.standard_normal(64).astype(np.float32)
        z = rng.choice([-1.0, 1.0], 64).astype(np.float32)
        hz = rng.standard_normal(64).astype(np.float32)
        a.step([g], [z], [hz], 0.1, 1.0, 96, 0, 100)
        b.step([g * np.float32(1024)], [z], [hz * np.float32(1024)], 0.1, 1024.0, 96, 0, 100)
    assert same(snapshot(a), snapshot(b))


def test_stored_precision_of_the_previous_step_is_what_the_next_step_reads():
    # thresholds force FP16 storage from the first step on, although the tensor starts as FP32:
    # step 2 must widen FP16 values.  Plain SGD (no momentum, no decay, alpha = 0) beside it in numpy.
    orc, p, rng = _small(dict(tau_low=1e30, tau_high=2e30, tau_curv=1e30, alpha=0.0, momentum=0.0,
                              weight_decay=0.0))
    ref = p.copy()
    for step in range(3):
        g = rng.standard_normal(64).astype(np.float32)
        orc.step([g], [None], [None], 0.1, 1.0, 96, 0, 100)
        t = orc.tensors[0]
        assert (t.prev_code, t.code) == ((FP32 if step == 0 else FP16), FP16)
        ref = (ref - np.float32(0.1) * g).astype(np.float16).astype(np.float32)
        got = t.param_f32()
        # fma vs separate rounding may differ in the last fp16 place on rare elements
        assert np.max(np.abs(got - ref)) <= np.max(np.abs(ref)) * 2.0 ** -10
        assert np.mean(got == ref) > 0.95


def test_control_interval_counts_applied_steps():
    # T_ctrl = 2 with the second call skipped: the control steps are the 2nd and 4th APPLIED steps,
    # i.e. calls 3 and 5 (a skipped step changes no state, counters included)
    orc, _, rng = _small(dict(ctrl_interval=2, tau_low=1e30, tau_high=2e30, tau_curv=1e30))
    codes = []
    for call in range(1, 6):
        g = rng.standard_normal(64).astype(np.float32)
        if call == 2:
            g[0] = np.nan
        orc.step([g], [None], [None], 0.1, 1.0, 96, 0, 100)
        codes.append(orc.tensors[0].code)
    assert codes == [FP32, FP32, FP16, FP16, FP16]


def test_first_fisher_sample_initialises_whenever_it_arrives():
    # squared-gradient source with the curvature refresh switched off at the first step: the first
    # refresh sets h to the sample itself, the next one smooths
    orc, _, rng = _small(dict(curvature_source=1, beta_curv=0.9))
    g1, g2, g3 = (rng.standard_normal(64).astype(np.float32) for _ in range(3))
    orc.step([g1], [None], [None], 0.1, 1.0, 96, 0, 100, update_curvature=False)
    assert not orc.tensors[0].curv.any() and orc.tensors[0].nnz == 0
    orc.step([g2], [None], [None], 0.1, 1.0, 96, 0, 100, update_curvature=True)
    assert np.array_equal(orc.tensors[0].curv, g2 * g2)
    orc.step([g3], [None], [None], 0.1, 1.0, 96, 0, 100, update_curvature=True)
    want = 0.9 * (g2.astype(np.float64) ** 2) + 0.1 * (g3.astype(np.float64) ** 2)
    assert np.allclose(orc.tensors[0].curv, want, rtol=1e-6, atol=0)
