"""Parity at the full sizes of the two large workloads, in the launch configuration bench.py
times: the oracle follows a sample of whole tensors element by element (tensors are independent
once the skip decision is known), and every tensor is checked through properties that hold at
any size and are evaluated with plain PyTorch operations on the GPU."""
import numpy as np
import pytest
import torch

import oracle
import paper_2508_16905_amd as ta
from workloads import get_workload
from workloads.configs import FP32
from _gpu_harness import bits_equal, same_or_both_nan
from _runner import to_numpy

pytestmark = pytest.mark.gpu


def popcount_words(mask: torch.Tensor) -> int:
    b = mask.view(torch.uint8)
    table = torch.tensor([bin(i).count("1") for i in range(256)], dtype=torch.int64, device=mask.device)
    return int(table[b.long()].sum().item())


def check_properties(opt, l, st, k):
    """Invariants of the threshold / mask that need no oracle."""
    a = opt.curv[l].abs()
    theta = torch.tensor(st.theta, dtype=torch.float32, device=a.device)
    ge = int(((a >= theta) & (a > 0)).sum().item())
    gt = int((a > theta).sum().item())
    assert st.nnz == ge == popcount_words(opt.mask[l]), (l, st.nnz, ge)
    if st.theta > 0.0:
        assert gt < k <= ge, (l, gt, k, ge)  # theta is the k-th largest magnitude
    else:
        assert ge < k, (l, ge, k)            # fewer non-zero magnitudes than k: all of them are kept
    assert st.lambda_ == float(a.max().item())


def run_sampled(wl, sample, steps, dev, check_all_every=1, fisher=False):
    L = wl.n_tensors
    params = [wl.init_param(l, device=dev) for l in range(L)]
    opt = ta.TriAccel(wl.hyper, params, grad_dtype=wl.grad_dtype)
    opt.set_profiling(2)   # the launch configuration that bench.py times: kernel by kernel, events around the update
    cfg = oracle.OracleConfig.from_hyper(wl.hyper)
    orc = oracle.OracleTriAccel(cfg, [to_numpy(params[l]) for l in sample], [wl.init_dtype(l) for l in sample],
                                [wl.grad_dtype] * len(sample), workers=len(sample))
    del params
    scale, batch = float(wl.hyper["loss_scale"]), int(wl.hyper["batch_size"])
    skipped_steps = []
    run_sampled.band_steps = 0   # (sampled tensor, step) pairs that the predicted band settled
    for t in range(1, steps + 1):
        grads = [wl.grad(t, l, scale, device=dev) for l in range(L)]
        if fisher:
            zs = hzs = [None] * L
        else:
            pr = [wl.probe(t, l, scale, device=dev) for l in range(L)]
            zs, hzs = [p[0] for p in pr], [p[1] for p in pr]
            del pr
        opt.step(grads, zs, hzs, lr=wl.hyper["lr"], loss_scale=scale, batch_size=batch, mem_used_bytes=8,
                 mem_total_bytes=10)
        res = opt.result()
        # overflow in tensors the oracle does not hold, found with a library reduction
        elsewhere = any((not bool(torch.isfinite(grads[l]).all())) for l in range(L) if l not in sample)
        ro = orc.step([to_numpy(grads[l]) for l in sample], [None if fisher else to_numpy(zs[l]) for l in sample],
                      [None if fisher else to_numpy(hzs[l]) for l in sample], wl.hyper["lr"], scale, batch, 8, 10,
                      overflow_elsewhere=elsewhere)
        assert res.skipped == ro["skipped"], (t, res.skipped, ro["skipped"])
        assert res.next_loss_scale == ro["next_loss_scale"] and res.next_batch_size == ro["next_batch_size"]
        skipped_steps.append(res.skipped)
        st = opt.layer_state()
        run_sampled.band_steps += sum(1 for l in sample if st[l].sel_outcome == 1 and not res.skipped)
        for o, l in zip(orc.tensors, sample):
            g = st[l]
            w = f"{wl.name} step {t} tensor {l}"
            assert (g.code, g.prev_code, g.found_inf, g.nnz) == (o.code, o.prev_code, o.found_inf, o.nnz), w
            for gv, ov in ((g.theta, o.theta), (g.lambda_, o.lam), (g.eta, o.eta)):
                assert np.float32(gv).view(np.uint32) == np.float32(ov).view(np.uint32), w
            sd = float(np.sqrt(max(float(o.var), 0.0)))
            assert abs(g.mean - float(o.mean)) <= 1e-5 * max(abs(float(o.mean)), sd) + 1e-45, w
            assert abs(g.var - float(o.var)) <= 1e-5 * abs(float(o.var)) + 1e-45, w
            assert abs(g.v - float(o.v)) <= 1e-5 * abs(float(o.v)) + 1e-45, w
            assert bits_equal(opt.mask[l].cpu().numpy().view(np.uint32), o.mask), w + " mask"
            assert bits_equal(opt.curv[l].cpu().numpy(), o.curv), w + " curvature"
            assert same_or_both_nan(opt.mom[l].cpu().numpy(), o.mom), w + " momentum"
            gp, op = to_numpy(opt.param(l, g.code)), o.param_view()
            assert (same_or_both_nan(gp, op) if o.code == FP32 else bits_equal(gp, op)), w + " parameters"
        if not res.skipped and t % check_all_every == 0:
            for l in range(L):
                n = wl.numel(l)
                k = max(1, min(n, n - (n * int(wl.hyper["sparsity_ppm"])) // 1000000))
                check_properties(opt, l, st[l], k)
        print(f"{wl.name}: step {t} ok (skipped={res.skipped}, loss scale {scale})", flush=True)
        scale, batch = ro["next_loss_scale"], ro["next_batch_size"]
        del grads, zs, hzs
    codes = [s.code for s in opt.layer_state()]
    opt.close()
    return skipped_steps, codes


def test_large_streaming_full_size_sampled_tensors():
    wl = get_workload("large_streaming")
    assert wl.total_params == 1073741824
    # steps 1-3 go through the fallback selection (no prediction yet), the later ones through the
    # predicted band: both at the full size
    skipped, codes = run_sampled(wl, sample=[0, 37, 63], steps=6, dev=torch.device("cuda:0"))
    assert skipped == [0] * 6 and len(set(codes)) >= 2
    assert run_sampled.band_steps >= 3


def test_large_streaming_full_size_fisher_source_and_elementwise_step_size():
    wl = get_workload("large_streaming")
    wl.hyper = dict(wl.hyper, curvature_source=1, elementwise_scale=1, alpha=1e4)
    skipped, codes = run_sampled(wl, sample=[11, 50], steps=5, dev=torch.device("cuda:0"), fisher=True)
    assert skipped == [0] * 5


def test_mixed_state_full_size_sampled_tensors_with_overflow():
    wl = get_workload("mixed_state")
    assert wl.total_params == 352321536
    inj7, inj14 = wl.injected_tensor(7), wl.injected_tensor(14)
    sample = sorted({0, 1, 2, 5, 47, 95, inj7})  # both shapes, all three initial dtypes, one injected tensor
    assert wl.steps == 50
    skipped, codes = run_sampled(wl, sample=sample, steps=wl.steps, dev=torch.device("cuda:0"), check_all_every=5)
    assert all(skipped[t - 1] == 1 for t in range(7, 51, 7))
    assert inj14 not in sample  # the second injection hits a tensor the oracle does not hold
    assert set(codes) == {0, 1, 2}


def test_power_iteration_full_size_sampled_tensors():
    """64 x 4096 x 4096 with k = 5 vectors per tensor (43 GB of vectors): the oracle follows two
    whole tensors; every tensor's new vectors are checked for orthonormality with library
    reductions on the GPU, and its Rayleigh quotients against library dot products."""
    dev = torch.device("cuda:0")
    wl = get_workload("large_streaming")
    L, k = wl.n_tensors, 5
    opt = ta.TriAccel(dict(wl.hyper, power_k=k), [wl.init_param(l, device=dev) for l in range(L)],
                      grad_dtype=wl.grad_dtype)
    sample = [3, 41]
    us = [wl.power_start(l, k, device=dev) for l in range(L)]
    hus = [wl.power_hessian_times(l, us[l]) for l in range(L)]
    u_in = {l: to_numpy(us[l]).copy() for l in sample}
    # quotients from library reductions, before the call overwrites u
    want_ray = [((us[l].double() * hus[l].double()).sum(1) / (us[l].double() ** 2).sum(1)).cpu().numpy() for l in range(L)]
    opt.power_iter(us, hus, k, latch=True)
    info = opt.power_state()
    for l in range(L):
        assert info[l].deficient == 0
        assert np.allclose(np.array(info[l].rayleigh[:k]), want_ray[l], rtol=1e-6, atol=0), l
        g = (us[l].double() @ us[l].double().T).cpu().numpy()
        assert np.max(np.abs(g - np.eye(k))) < 1e-6, (l, g)
    cfg = oracle.OracleConfig.from_hyper(wl.hyper)
    orc = oracle.OracleTriAccel(cfg, [np.zeros(wl.numel(l), dtype=np.float32) for l in sample], [FP32] * len(sample),
                                [wl.grad_dtype] * len(sample))
    uo = [u_in[l] for l in sample]
    orc.power_step(uo, [to_numpy(hus[l]) for l in sample], k, True)
    for pos, l in enumerate(sample):
        t = orc.tensors[pos]
        assert np.all(np.abs(np.array(info[l].rayleigh[:k]) - t.rayleigh) <= 2 * 2.0 ** -23 * np.abs(t.rayleigh))
        assert np.all(np.abs(np.array(info[l].hnorm[:k]) - t.hnorm) <= 2 * 2.0 ** -23 * np.abs(t.hnorm))
        want = uo[pos].reshape(k, -1)
        got = to_numpy(us[l])
        err = np.abs(got.astype(np.float64) - want.astype(np.float64))
        assert np.all(err <= 2 * 2.0 ** -23 * np.abs(want) + 1e-11 * np.max(np.abs(want))), (l, float(err.max()))
        assert abs(info[l].lambda_latched - t.lam_power) <= 2 * 2.0 ** -23 * abs(t.lam_power)
    opt.close()


def test_single_tensor_of_maximum_size():
    """One tensor of 2^31 - 3 elements (the largest the ABI accepts, ragged in every granularity).
    The per-layer scalars the oracle needs are formed with library reductions on the GPU; the
    oracle then follows slices at the start, in the middle and at the very end element by element,
    and the threshold is checked by counting."""
    import ctypes as C

    dev = torch.device("cuda:0")
    n = (1 << 31) - 3
    hyper = dict(get_workload("large_streaming").hyper, tau_curv=1e30)
    lr, alpha = float(hyper["lr"]), float(hyper["alpha"])
    g0 = torch.Generator(device=dev)
    g0.manual_seed(12345)
    param = torch.randn(n, generator=g0, device=dev, dtype=torch.float32) * 0.1
    opt = ta.TriAccel(hyper, [param], grad_dtype=FP32)
    L = oracle.lib()
    spans = [(0, 1 << 20), (n // 2 - 12345, n // 2 - 12345 + (1 << 20)), (n - (1 << 20) - 1, n)]
    before = [(to_numpy(param[a:b]).copy(), np.zeros(b - a, np.float32)) for a, b in spans]
    del param
    v_prev = None
    for t in (1, 2):
        grad = torch.randn(n, generator=g0, device=dev, dtype=torch.float32) * 0.0316
        z = (torch.randint(0, 2, (n,), generator=g0, device=dev, dtype=torch.int8) * 2 - 1).to(torch.float32)
        hz = z * 0.37 + torch.randn(n, generator=g0, device=dev, dtype=torch.float32) * 0.19
        h_prev = opt.curv[0].clone() if t == 2 else None
        opt.step([grad], [z], [hz], lr=lr, loss_scale=1.0, batch_size=64, mem_used_bytes=8, mem_total_bytes=10)
        res = opt.result()
        st = opt.layer_state()[0]
        assert res.skipped == 0 and st.numel == n
        # curvature EMA with library element-wise operations (same fp32 operation order, no fma in torch:
        # the first probe is a product only, the second step is checked on the slices below)
        u = z * hz
        if t == 1:
            assert torch.equal(opt.curv[0], u)
        lam = float(opt.curv[0].abs().max().item())
        assert st.lambda_ == lam
        k = n - (n * int(hyper["sparsity_ppm"])) // 1000000
        check_properties(opt, 0, st, k)
        # statistics with library reductions in fp64, by parts to bound the temporary memory
        parts = torch.split(grad, 1 << 28)
        mean = sum(float(p.double().sum().item()) for p in parts) / n
        var = sum(float(((p.double() - mean) ** 2).sum().item()) for p in parts) / n
        assert abs(st.mean - mean) <= 1e-5 * max(abs(mean), var ** 0.5) and abs(st.var - var) <= 1e-5 * var
        v = np.float32(var) if v_prev is None else np.float32(L.oracle_var_ema(v_prev, var, np.float32(hyper["beta_var"]), 0))
        assert abs(st.v - float(v)) <= 1e-5 * float(v)
        for tau in (hyper["tau_low"], hyper["tau_high"]):
            assert abs(float(v) - tau) / tau > 1e-3
        v_prev = v
        code = int(L.oracle_precision_code(v, np.float32(lam), np.float32(hyper["tau_low"]), np.float32(hyper["tau_high"]),
                                           np.float32(hyper["tau_curv"])))
        eta = np.float32(L.oracle_eta(np.float32(lr), np.float32(alpha), np.float32(lam)))
        assert st.code == code and np.float32(st.eta) == eta
        # the oracle on the slices: update (and, at the second step, the EMA recurrence)
        prev_code = FP32 if t == 1 else prev_code_last
        for (a, b), (pbuf, mbuf) in zip(spans, before):
            m = b - a
            raw = np.zeros(4 * m, np.uint8)
            raw.view(pbuf.dtype)[:m] = pbuf
            gs = to_numpy(grad[a:b])
            L.oracle_update(raw.ctypes.data, prev_code, code, gs.ctypes.data, FP32, mbuf.ctypes.data, m, np.float32(1.0),
                            np.float32(hyper["weight_decay"]), np.float32(hyper["momentum"]), eta)
            view = raw.view(np.float32 if code == FP32 else np.uint16)[:m]
            got = to_numpy(opt.param(0, code)[a:b])
            assert np.array_equal(got.view(view.dtype), view), (t, a)
            assert np.array_equal(to_numpy(opt.mom[0][a:b]).view(np.uint32), mbuf.view(np.uint32)), (t, a)
            if t == 2:
                hs = to_numpy(h_prev[a:b]).copy()
                zs, hzs = to_numpy(z[a:b]), to_numpy(hz[a:b])   # held until the call returns
                flag = C.c_uint32(0)
                L.oracle_curv_ema(zs.ctypes.data, hzs.ctypes.data, hs.ctypes.data, m,
                                  np.float32(1.0), np.float32(hyper["beta_curv"]), 0, C.byref(flag))
                assert np.array_equal(to_numpy(opt.curv[0][a:b]).view(np.uint32), hs.view(np.uint32)), a
        before = [(view_of(opt, 0, code, a, b), mb) for (a, b), (_, mb) in zip(spans, before)]
        prev_code_last = code
        print(f"maximum-size tensor: step {t} ok (code {code}, theta {st.theta}, nnz {st.nnz})", flush=True)
        del grad, z, hz, u, parts
    opt.close()


def view_of(opt, l, code, a, b):
    """Stored parameters of a slice in their stored dtype (numpy, bit-preserving)."""
    return to_numpy(opt.param(l, code)[a:b]).copy()


def test_in_place_resize_through_every_phase():
    """Storage size changing in place on tensors of 4096 and 4099 chunks (the second one ragged and
    one phase deeper): every narrowing and widening pair, all phases of the rewrite, every element
    compared with the oracle.  No probes: only the statistics and the update run."""
    from _gpu_harness import Pair
    from test_gpu_parity import custom
    from workloads.configs import BF16, FP16

    sizes = [4096 * 4096, 4096 * 4096 + 2 * 4096 + 5]
    for init, target, (lo, hi) in ((FP16, FP32, (0.0, 0.0)), (BF16, FP32, (0.0, 0.0)),
                                   (FP32, FP16, (1e30, 1e31)), (FP32, BF16, (0.0, 1e30))):
        wl = custom(sizes, param_dtypes=[init] * len(sizes), tau_low=lo, tau_high=hi, tau_curv=1e30, steps=2)
        p = Pair(wl)
        for t in (1, 2):
            g, z, hz = p.inputs(t, probe=False)
            p.step(g, z, hz, label=f"{init}->{target} t={t}")
        assert [(o.prev_code, o.code) for o in p.orc.tensors] == [(target, target)] * 2
        p.close()
        print(f"in-place resize {init} -> {target} ok", flush=True)


def _switching_run(sizes, mult, workers=16):
    """Every tensor follows the same sequence of storage precisions (variance EMA off, the gradient
    scale picks the code); update-only steps, every element compared with the oracle."""
    from _gpu_harness import Pair
    from test_gpu_parity import custom

    wl = custom(sizes, name="large_streaming", beta_var=0.0, tau_low=1e-4, tau_high=1e-2, tau_curv=1e30)
    p = Pair(wl, workers=workers)
    for t, m in enumerate(mult, start=1):
        g, z, hz = p.inputs(t, probe=False)
        p.step([x * (m * 3.0) for x in g], z, hz, label=f"t={t}")
        print(f"step {t}: codes {sorted(set(p.code_hist[-1]))}", flush=True)
    seq = [row[0] for row in p.code_hist]
    p.close()
    return seq


def test_in_place_resize_with_more_work_items_than_workgroups():
    """65 tensors of 4097 chunks narrowing, widening and narrowing again together: 65 x 1024
    (tensor, subtree) work items in the widest launch of the rewrite, more than the 65536 workgroups a
    launch is given, so workgroups take several items each."""
    from workloads.configs import BF16, FP16

    assert _switching_run([4096 * 4096 + 7] * 65, [0.1, 10.0, 1.0]) == [FP16, FP32, BF16]


def test_in_place_resize_of_one_tensor_of_65540_chunks():
    """A single tensor of 2^28 + 12345 elements: four subtree stages, the deepest with 8192 roots."""
    from workloads.configs import BF16, FP16

    assert _switching_run([(1 << 28) + 12345, 5000], [0.1, 10.0, 1.0]) == [FP16, FP32, BF16]
