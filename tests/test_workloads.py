"""The synthetic parameter sets have the shapes of the paper's two architectures (Sec. 4) and
the sizes the benchmark configurations name; generators are seeded and reproducible."""
import torch

from workloads import get_workload
from workloads.configs import BF16, FP16, FP32
from _runner import decision_margin, run_oracle


def test_tensor_and_parameter_counts():
    want = {"tiny_mlp": (4, 101770), "resnet18": (62, 11173962), "efficientnet_b0": (213, 4020358),
            "large_streaming": (64, 1073741824), "mixed_state": (96, 352321536)}
    for name, (nt, n) in want.items():
        wl = get_workload(name)
        assert (wl.n_tensors, wl.total_params) == (nt, n)
    eff = get_workload("efficientnet_b0")
    sizes = [eff.numel(l) for l in range(eff.n_tensors)]
    assert max(sizes) == 409600 and min(sizes) == 4 and sum(s < 1000 for s in sizes) == 121
    res = get_workload("resnet18")
    sizes = [res.numel(l) for l in range(res.n_tensors)]
    assert max(sizes) == 2359296 and min(sizes) == 10 and sum(s < 1000 for s in sizes) == 41


def test_generators_are_seeded():
    wl = get_workload("resnet18")
    a, b = wl.grad(3, 5), wl.grad(3, 5)
    assert torch.equal(a, b) and not torch.equal(a, wl.grad(4, 5))
    z, hz = wl.probe(2, 7)
    assert set(z.unique().tolist()) == {-1.0, 1.0}
    zeros = (wl.grad(1, 3) == 0).float().mean().item()
    assert 0.08 < zeros < 0.12


def test_mixed_state_split_and_injection():
    wl = get_workload("mixed_state")
    kinds = [wl.init_dtype(l) for l in range(wl.n_tensors)]
    assert (kinds.count(FP32), kinds.count(BF16), kinds.count(FP16)) == (38, 38, 20)
    small = get_workload("mixed_state", n_square=2, n_wide=10, rows=16)
    v = small.injected_tensor(7)
    assert v is not None and small.injected_tensor(8) is None
    g = small.grad(7, v, 32768.0)
    assert g.dtype == torch.float16 and not torch.isfinite(g).all()
    assert all(torch.isfinite(small.grad(7, l, 32768.0)).all() for l in range(small.n_tensors) if l != v)


def test_resnet18_first_steps_show_all_three_codes():
    wl = get_workload("resnet18")
    orc, hist = run_oracle(wl, steps=2, workers=8)
    codes = {rec["code"] for h in hist for rec in h["layers"]}
    assert codes == {FP16, BF16, FP32}
    assert decision_margin(hist, wl.hyper) > 1e-6
