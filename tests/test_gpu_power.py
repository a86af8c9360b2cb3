"""GPU parity of the power-iteration call (Sec. 3.2, third equation) against the CPU oracle.

Bars.  The new vectors are fp32 roundings of fp64 results that the two sides reach by different
routes (ordered Gram-Schmidt in the oracle; Cholesky of the Gram matrix in the kernels), so they
may differ in the last place: |gpu - oracle| <= 2 ulp(fp32) of the element + the conditioning
term 1e-15 * cond^2 (cond of the supplied products, computed in the test from their Gram matrix).  Rayleigh quotients
and norms: 2 ulp(fp32).  The residual is formed from sums on the GPU (G_jj - 2 lambda c + lambda^2
d), which cancels when the vector has converged: |gpu - oracle| <= 1e-6 * ||Hu|| / ||u||.
Flags: exact."""

import numpy as np
import pytest
import torch

import oracle
import paper_2508_16905_amd as ta
from paper_2508_16905_amd import binding as B
from workloads import get_workload
from _runner import to_numpy

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
ULP = 2.0 ** -23


def dense(x, n):
    """(k, stride) tensor -> contiguous numpy (k, n)."""
    return np.ascontiguousarray(to_numpy(x)[:, :n])


def make_pair(wl, **extra):
    hyper = dict(wl.hyper, **extra)
    cfg = oracle.OracleConfig.from_hyper(hyper)
    L = wl.n_tensors
    params = [to_numpy(wl.init_param(l)) for l in range(L)]
    orc = oracle.OracleTriAccel(cfg, params, [wl.init_dtype(l) for l in range(L)], [wl.grad_dtype] * L)
    gpu = ta.TriAccel(hyper, [wl.init_param(l).to(DEV) for l in range(L)], grad_dtype=wl.grad_dtype)
    return orc, gpu


def compare_step(wl, orc, gpu, us_cpu, hus_cpu, k, latch):
    """One call on both sides with the same inputs; returns the GPU's new vectors."""
    L = wl.n_tensors
    us_gpu = [u.to(DEV) for u in us_cpu]
    hus_gpu = [h.to(DEV) for h in hus_cpu]
    gpu.power_iter(us_gpu, hus_gpu, k, latch)
    info = gpu.power_state()
    uo = [dense(us_cpu[l][:k], wl.numel(l)).copy() for l in range(L)]
    ho = [dense(hus_cpu[l][:k], wl.numel(l)) for l in range(L)]
    orc.power_step(uo, ho, k, latch)
    for pos, l in enumerate(range(L)):
        n, t, g = wl.numel(l), orc.tensors[l], info[l]
        assert g.deficient == t.deficient, (l, g.deficient, t.deficient)
        ray = np.array(g.rayleigh[:k]); res = np.array(g.resid[:k]); hn = np.array(g.hnorm[:k])
        assert np.all(np.abs(ray - t.rayleigh) <= 2 * ULP * np.abs(t.rayleigh) + 1e-30), (l, ray, t.rayleigh)
        assert np.all(np.abs(hn - t.hnorm) <= 2 * ULP * np.abs(t.hnorm) + 1e-30), (l, hn, t.hnorm)
        unorm = np.linalg.norm(dense(us_cpu[l][:k], n).astype(np.float64), axis=1)
        tol = 1e-6 * t.hnorm / np.maximum(unorm, 1e-30) + 2 * ULP * np.abs(t.resid)
        assert np.all(np.abs(res - t.resid) <= tol), (l, res, t.resid, tol)
        assert list(g.rayleigh[k:]) == [0.0] * (8 - k)
        got = dense(us_gpu[l][:k], n)
        want = uo[pos].reshape(k, n)
        err = np.abs(got.astype(np.float64) - want.astype(np.float64))
        # conditioning of the independent supplied products (eigenvalue ratio of their Gram matrix = cond^2)
        keep = [j for j in range(k) if not (t.deficient >> j) & 1]
        cond2 = 1.0
        if keep:
            w64 = ho[pos].reshape(k, n)[keep].astype(np.float64)
            ev = np.linalg.eigvalsh(w64 @ w64.T)
            cond2 = float(ev[-1] / max(ev[0], 1e-300))
        bound = 2 * ULP * np.abs(want) + (1e-12 + 1e-15 * cond2) * np.max(np.abs(want))
        assert np.all(err <= bound), (l, float(err.max()), int(np.argmax(err - bound)))
        # padding columns stay untouched (zero)
        assert not to_numpy(us_gpu[l])[:k, n:].any()
        if latch:
            assert abs(g.lambda_latched - t.lam_power) <= 2 * ULP * abs(t.lam_power)
        assert abs(g.lambda_max - np.float32(np.max(np.abs(t.rayleigh)))) <= 2 * ULP * abs(g.lambda_max)
    return us_gpu


def test_one_iteration_on_every_small_workload_shape():
    for name in ("tiny_mlp", "resnet18"):
        wl = get_workload(name)
        orc, gpu = make_pair(wl, power_k=5)
        L = wl.n_tensors
        us = [wl.power_start(l, 5) for l in range(L)]
        hus = [wl.power_hessian_times(l, us[l].double()).float() for l in range(L)]
        compare_step(wl, orc, gpu, us, hus, 5, latch=True)
        gpu.close()


@pytest.mark.parametrize("k", [1, 2, 3, 4, 6, 7, 8])
def test_every_vector_count_and_ragged_sizes(k):
    wl = get_workload("large_streaming", n_tensors=9, side=64)
    sizes = [1, 3, 5, 4095, 4096, 4097, 8 * 4096 + 7, 70001, 3 * 8 * 4096]
    wl.tensors = [(f"t{i}", (n,)) for i, n in enumerate(sizes)]
    orc, gpu = make_pair(wl, power_k=8)
    us = [wl.power_start(l, k) for l in range(len(sizes))]
    hus = [wl.power_hessian_times(l, us[l].double()).float() for l in range(len(sizes))]
    compare_step(wl, orc, gpu, us, hus, k, latch=False)
    gpu.close()


def test_independent_chains_converge_to_the_same_top_eigenvalues():
    wl = get_workload("tiny_mlp")
    orc, gpu = make_pair(wl, power_k=5)
    L, k = wl.n_tensors, 5
    ug = [wl.power_start(l, k).to(DEV) for l in range(L)]
    uo = [dense(wl.power_start(l, k), wl.numel(l)).copy() for l in range(L)]
    for it in range(40):
        # the stand-in Hessian is generated on the CPU for both chains (device generators differ)
        hg = [wl.power_hessian_times(l, ug[l].cpu().double()).float().to(DEV) for l in range(L)]
        gpu.power_iter(ug, hg, k, latch=(it == 39))
        ho = []
        for l in range(L):
            n = wl.numel(l)
            pad = torch.zeros(k, (n + 3) // 4 * 4, dtype=torch.float64)
            pad[:, :n] = torch.from_numpy(uo[l].reshape(k, n)).double()
            ho.append(dense(wl.power_hessian_times(l, pad).float(), n))
        orc.power_step(uo, ho, k, latch=(it == 39))
    info = gpu.power_state()
    for l in range(L):
        t = orc.tensors[l]
        if wl.numel(l) < 100:
            continue   # fewer directions than spikes: the small tensors are covered by the one-step tests
        ray = np.array(info[l].rayleigh[:k])
        assert np.allclose(ray, t.rayleigh, rtol=1e-4), (l, ray, t.rayleigh)
        assert np.all(ray[:-1] > ray[1:])          # ordered: vector j holds the j-th eigenvalue
        assert info[l].lambda_latched == pytest.approx(float(t.lam_power), rel=1e-4)
    gpu.close()


def exact_pair(wl, k, seed):
    """Small-integer vectors: every sum is exact in fp64 whatever its order, so both sides get
    bit-identical quotients."""
    rs = np.random.default_rng(seed)
    us, hus = [], []
    for l in range(wl.n_tensors):
        n = wl.numel(l)
        stride = (n + 3) // 4 * 4
        u = np.zeros((k, stride), dtype=np.float32)
        h = np.zeros((k, stride), dtype=np.float32)
        u[:, :n] = rs.integers(-2, 3, (k, n))
        u[:, 0] = 1
        h[:, :n] = rs.integers(-3, 4, (k, n))
        h[np.arange(k), np.arange(k) % n] += 5
        us.append(torch.from_numpy(u))
        hus.append(torch.from_numpy(h))
    return us, hus


def test_latched_lambda_drives_step_size_and_promotion_bit_exactly():
    wl = get_workload("large_streaming", n_tensors=6, side=96)
    extra = dict(power_k=3, lambda_source=1, tau_curv=0.02, alpha=0.5)
    orc, gpu = make_pair(wl, **extra)
    L, k = wl.n_tensors, 3
    scale = float(wl.hyper["loss_scale"])
    for t in range(1, 6):
        if t in (2, 4):
            us, hus = exact_pair(wl, k, seed=t)
            compare_step(wl, orc, gpu, us, hus, k, latch=(t == 2))   # the call at t == 4 must change nothing
        grads = [wl.grad(t, l, scale) for l in range(L)]
        gpu.step([g.to(DEV) for g in grads], None, None, lr=0.1, loss_scale=scale, batch_size=64, mem_used_bytes=8,
                 mem_total_bytes=10)
        orc.step([to_numpy(g) for g in grads], [None] * L, [None] * L, 0.1, scale, 64, 8, 10)
        assert gpu.result().skipped == 0
        st = gpu.layer_state()
        for l in range(L):
            o = orc.tensors[l]
            assert st[l].code == o.code and st[l].prev_code == o.prev_code
            assert np.float32(st[l].lambda_) == o.lam and np.float32(st[l].eta) == o.eta, (t, l, st[l].lambda_, o.lam)
            got = to_numpy(gpu.param(l, st[l].code))
            assert np.array_equal(got.view(np.uint8), o.param_view().view(np.uint8)), (t, l)
            assert np.array_equal(to_numpy(gpu.mom[l]).view(np.uint32), o.mom.view(np.uint32)), (t, l)
    assert any(o.lam > 0 for o in orc.tensors) and len({o.code for o in orc.tensors}) >= 1
    gpu.close()


def test_dependent_and_zero_vectors():
    wl = get_workload("large_streaming", n_tensors=2, side=80)
    orc, gpu = make_pair(wl, power_k=4)
    us = [wl.power_start(l, 4) for l in range(2)]
    hus = [wl.power_hessian_times(l, us[l].double()).float() for l in range(2)]
    hus[0][2] = 2 * hus[0][0] - hus[0][1]
    hus[1][1] = 0
    us[1][3] = 0
    compare_step(wl, orc, gpu, us, hus, 4, latch=False)
    assert orc.tensors[0].deficient == 0b0100 and orc.tensors[1].deficient == 0b0010
    gpu.close()


def test_argument_errors():
    wl = get_workload("tiny_mlp")
    lib = ta.load_library()
    gpu = ta.TriAccel(dict(wl.hyper, power_k=2), [wl.init_param(l).to(DEV) for l in range(wl.n_tensors)])
    info = (B.PowerInfo * gpu.n)()
    assert lib.triaccel_power_state(gpu.handle, info, gpu.n) == -7          # nothing to report yet
    us = [wl.power_start(l, 2).to(DEV) for l in range(gpu.n)]
    arr = (B.PowerTensor * gpu.n)()
    for i in range(gpu.n):
        arr[i].u, arr[i].hu, arr[i].stride = us[i].data_ptr(), us[i].data_ptr(), us[i].shape[1]
    assert lib.triaccel_power_iter(gpu.handle, arr, gpu.n, 3, 0) == -1      # k above power_k
    assert lib.triaccel_power_iter(gpu.handle, arr, gpu.n, 0, 0) == -1
    assert lib.triaccel_power_iter(gpu.handle, arr, gpu.n - 1, 2, 0) == -3
    arr[1].stride = wl.numel(1) - 4
    assert lib.triaccel_power_iter(gpu.handle, arr, gpu.n, 2, 0) == -1      # stride below numel
    arr[1].stride = us[1].shape[1] + 2
    assert lib.triaccel_power_iter(gpu.handle, arr, gpu.n, 2, 0) == -1      # not a multiple of 4
    arr[1].stride = us[1].shape[1]
    arr[0].hu = None
    assert lib.triaccel_power_iter(gpu.handle, arr, gpu.n, 2, 0) == -4
    arr[0].hu = us[0].data_ptr() + 4
    assert lib.triaccel_power_iter(gpu.handle, arr, gpu.n, 2, 0) == -5
    gpu.close()
    # a handle without the workspace, and the config check
    gpu = ta.TriAccel(wl.hyper, [wl.init_param(l).to(DEV) for l in range(wl.n_tensors)])
    arr[0].hu = us[0].data_ptr()
    assert lib.triaccel_power_iter(gpu.handle, arr, gpu.n, 1, 0) == -1
    gpu.close()
    with pytest.raises(ta.TriAccelError):
        ta.TriAccel(dict(wl.hyper, lambda_source=1), [wl.init_param(l).to(DEV) for l in range(wl.n_tensors)])


def test_kernel_times_of_the_last_call_need_profiling():
    wl = get_workload("tiny_mlp")
    gpu = ta.TriAccel(dict(wl.hyper, power_k=2), [wl.init_param(l).to(DEV) for l in range(wl.n_tensors)])
    us = [wl.power_start(l, 2).to(DEV) for l in range(gpu.n)]
    hus = [u * 0.5 for u in us]
    with pytest.raises(ta.TriAccelError):
        gpu.power_times()            # no call yet
    gpu.power_iter(us, hus, 2)
    with pytest.raises(ta.TriAccelError):
        gpu.power_times()            # the call was not timed
    gpu.set_profiling(True)
    gpu.power_iter(us, hus, 2)
    times = gpu.power_times()
    assert len(times) == 3 and all(t > 0 for t in times)
    gpu.set_profiling(False)
    gpu.power_iter(us, hus, 2)
    with pytest.raises(ta.TriAccelError):
        gpu.power_times()            # times of an earlier call are not handed out for this one
    gpu.close()
