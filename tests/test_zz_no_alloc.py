"""The power iteration for callers that cannot allocate (triaccel_power_iter_static) against the
ordinary entry point (triaccel_power_iter), through the C ABI: new vectors and per-layer records
bit for bit, on two calls in a row, the second with a smaller input (the fixed device array keeps
the first call's tables and sums), then a third that is larger again."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2508_16905_amd as ta
from paper_2508_16905_amd import binding as B
from workloads import get_workload
from workloads.configs import FP32, Workload, _DEFAULT_HYPER

pytestmark = pytest.mark.gpu


def _workload(sizes, seed):
    tensors = [(f"t{i}", (n,)) for i, n in enumerate(sizes)]
    return Workload("large_streaming", 3, tensors, dict(_DEFAULT_HYPER), 1, seed=seed)


def _both(sizes, k, seed, dev):
    """One iteration through both entry points from identical inputs; returns nothing, asserts equality."""
    wl = _workload(sizes, seed)
    L = len(sizes)
    us = [wl.power_start(l, k, device=dev) for l in range(L)]
    hus = [wl.power_hessian_times(l, us[l]) for l in range(L)]
    us_static = [u.clone() for u in us]
    # existing entry point: a handle whose workspace triaccel_init allocated
    opt = ta.TriAccel(dict(wl.hyper, power_k=k), [wl.init_param(l, device=dev) for l in range(L)], grad_dtype=FP32)
    opt.power_iter(us, hus, k)
    want = opt.power_state()
    # the entry point that allocates nothing: raw ctypes call, outputs in caller-owned device memory
    info = torch.full((L * C.sizeof(B.PowerInfo),), 0xAB, dtype=torch.uint8, device=dev)
    arr = (B.PowerTensor * L)()
    for l in range(L):
        arr[l].u, arr[l].hu, arr[l].stride = us_static[l].data_ptr(), hus[l].data_ptr(), us_static[l].shape[1]
    numel = (C.c_int64 * L)(*sizes)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated(dev)
    lib = ta.load_library()
    rc = lib.triaccel_power_iter_static(arr, numel, L, k, C.c_void_p(info.data_ptr()),
                                        C.c_void_p(torch.cuda.current_stream(dev).cuda_stream))
    assert rc == 0, (rc, lib.triaccel_last_error())
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated(dev) == before
    got = (B.PowerInfo * L).from_buffer_copy(info.cpu().numpy().tobytes())
    for l in range(L):
        assert torch.equal(us_static[l].view(torch.int32), us[l].view(torch.int32)), (sizes, l)
        for name in ("rayleigh", "resid", "hnorm"):
            a = np.array(getattr(got[l], name), dtype=np.float32).view(np.uint32)
            b = np.array(getattr(want[l], name), dtype=np.float32).view(np.uint32)
            assert np.array_equal(a, b), (sizes, l, name)
        assert got[l].deficient == want[l].deficient
        assert np.float32(got[l].lambda_max).view(np.uint32) == np.float32(want[l].lambda_max).view(np.uint32)
        assert got[l].lambda_latched == 0.0
        assert any(got[l].rayleigh[j] != 0.0 for j in range(k))
    opt.close()


def test_static_entry_point_matches_the_allocating_one_on_consecutive_calls():
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    assert ta.load_library().triaccel_power_iter_static(None, None, 0, 1, None, None) == 0   # set-up only
    # several chunks and segments, ragged tails, a tensor below one vector; 70 tensors span two table batches
    big = [300007, 4096, 4097, 1, 33, 1100003, 8 * 4096, 8 * 4096 + 1] + [1000 + 37 * i for i in range(62)]
    _both(big, 5, 11, dev)
    _both([70001, 5, 40000], 3, 12, dev)          # smaller, right after: stale tables and sums must not leak
    _both([2 * 1024 * 1024 + 3, 9000], 8, 13, dev)


def test_static_entry_point_refuses_what_does_not_fit():
    dev = torch.device("cuda:0")
    lib = ta.load_library()
    u = torch.ones(8, dtype=torch.float32, device=dev)
    info = torch.zeros(C.sizeof(B.PowerInfo), dtype=torch.uint8, device=dev)
    one = (B.PowerTensor * 1)()
    one[0].u, one[0].hu, one[0].stride = u.data_ptr(), u.data_ptr(), 8

    def call(arr, numel, n, k):
        return lib.triaccel_power_iter_static(arr, (C.c_int64 * max(n, 1))(*numel), n, k, C.c_void_p(info.data_ptr()), None)

    assert call(one, [8], 1, 9) == -1 and call(one, [8], 1, 0) == -1        # k out of range
    assert call(one, [8], 257, 1) == -1                                      # too many tensors
    assert call(one, [9], 1, 1) == -1                                        # stride below numel
    many = (B.PowerTensor * 2)()
    for t in many:
        t.u, t.hu, t.stride = u.data_ptr(), u.data_ptr(), 1 << 30
    assert call(many, [65536 * 4096 // 2, 65536 * 4096 // 2 + 1], 2, 1) == -1  # one chunk beyond the fixed array
    assert b"65536" in lib.triaccel_last_error()
    torch.cuda.synchronize()
    assert torch.equal(u, torch.ones_like(u))
