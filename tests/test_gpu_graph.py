"""The step replayed as a HIP graph must give what the kernels launched one by one give: every
replay is compared with the oracle, with the test's own eager work (copies, synchronisations)
between the replays."""
import pytest

import paper_2508_16905_amd as ta
from workloads import get_workload
from workloads.configs import BF16, FP16, FP32
from _gpu_harness import Pair
from test_gpu_parity import custom

pytestmark = pytest.mark.gpu


def test_resnet18_shaped_set_replayed():
    wl = get_workload("resnet18")
    p = Pair(wl, graph=True).run(12)
    assert {c for row in p.code_hist for c in row} == {FP16, BF16, FP32}
    p.close()


def test_both_graph_variants_alternate_with_control_interval():
    wl = custom([5000, 70000, 33], steps=12, ctrl_interval=3)
    Pair(wl, graph=True).run(12, probe_every=3).close()


def test_loss_scale_and_skips_change_between_replays():
    wl = get_workload("mixed_state", n_square=4, n_wide=8, rows=64)
    p = Pair(wl, graph=True)
    skipped = []
    for t in range(1, 23):
        g, z, hz = p.inputs(t)
        skipped.append(p.step(g, z, hz)["skipped"])
    assert sum(skipped) >= 3 and skipped[6] == 1
    p.close()


def test_precision_switches_and_learning_rate_schedule_replayed():
    sizes = [9000, 4096, 130000, 50]
    wl = custom(sizes, name="large_streaming", beta_var=0.0, tau_low=1e-4, tau_high=1e-2, tau_curv=1e30)
    p = Pair(wl, graph=True)
    mult = [0.1, 1.0, 10.0, 10.0, 0.1, 1.0, 0.1, 10.0]
    for t, m in enumerate(mult, start=1):
        g, z, hz = p.inputs(t)
        p.step([x * (m * 3.0) for x in g], z, hz, lr=0.1 / t)
    assert {row[0] for row in p.code_hist} == {FP16, BF16, FP32}
    p.close()


def test_elementwise_and_fisher_variants_replayed():
    sizes = [33, 4097, 70001]
    wl = custom(sizes, elementwise_scale=1, curvature_source=1, alpha=1e4, steps=6)
    p = Pair(wl, graph=True)
    none = [None] * len(sizes)
    for t in range(1, 7):
        g, _, _ = p.inputs(t, probe=False)
        p.step(g, none, none, update_curvature=(t != 4))
    p.close()


def test_switching_graph_mode_on_and_off_and_the_default_stream():
    wl = get_workload("tiny_mlp")
    p = Pair(wl, graph=True)
    for t in range(1, 9):
        p.gpu.set_graph(t % 3 != 0)
        g, z, hz = p.inputs(t)
        p.step(g, z, hz)
    p.close()
    opt = ta.TriAccel(wl.hyper, [wl.init_param(l).to("cuda:0") for l in range(wl.n_tensors)])
    if opt.stream.cuda_stream == 0:
        with pytest.raises(ta.TriAccelError):
            opt.set_graph(True)
    opt.close()
