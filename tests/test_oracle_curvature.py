"""Pins for the oracle's Hutchinson diagonal curvature EMA (the "sparse second-order
signal" of Sec. 3.2 in its diagonal form)."""
import ctypes as C
import itertools

import numpy as np

import oracle
from workloads import get_workload
from _exact import bits, fma32, mul32, sub32


def curv_ema(z, hz, h, inv_scale=1.0, beta=0.9, first=0):
    flag = C.c_uint32(0)
    oracle.lib().oracle_curv_ema(z.ctypes.data, hz.ctypes.data, h.ctypes.data, h.size, np.float32(inv_scale),
                                 np.float32(beta), first, C.byref(flag))
    return flag.value


def test_diagonal_hessian_is_recovered_exactly_by_one_probe():
    rs = np.random.default_rng(0)
    d = rs.uniform(-3, 3, size=257).astype(np.float32)
    for trial in range(5):
        z = rs.choice([-1.0, 1.0], size=d.size).astype(np.float32)
        hz = d * z
        h = np.full(d.size, 99.0, np.float32)
        assert curv_ema(z, hz, h, first=1) == 0
        assert np.array_equal(h, d)


def test_mean_over_all_sign_vectors_is_the_diagonal():
    # dense symmetric integer matrix: every product and sum below is exact in fp32
    n = 8
    rs = np.random.default_rng(1)
    a = rs.integers(-4, 5, size=(n, n))
    hmat = (a + a.T).astype(np.float64)
    acc = np.zeros(n)
    for signs in itertools.product((-1.0, 1.0), repeat=n):
        z = np.array(signs, np.float32)
        hz = (hmat @ z).astype(np.float32)
        h = np.zeros(n, np.float32)
        curv_ema(z, hz, h, first=1)
        acc += h
    assert np.array_equal(acc / 2 ** n, np.diag(hmat))


def test_block_diagonal_quadratic_converges_to_the_diagonal():
    wl = get_workload("tiny_mlp")
    l = 2  # 128 x 10 weight: 40 blocks of 32
    n = wl.numel(l)
    diag, off = wl.hessian_diagonal(l), wl.hessian_offdiag_sq(l)
    assert (diag != 0).any() and (diag == 0).any()
    beta = 0.9
    h = np.zeros(n, np.float32)
    tail = []
    for t in range(1, 401):
        z, hz = wl.probe(t, l)
        curv_ema(z.numpy(), hz.numpy(), h, beta=beta, first=int(t == 1))
        if t > 100:
            tail.append(h.astype(np.float64))
    # zero blocks: exactly zero at every step
    assert np.all(h[diag == 0] == 0.0)
    # steady state: E[h_i] = H_ii, Var[h_i] = (1-beta)/(1+beta) * sum_{j != i} H_ij^2
    sd = np.sqrt((1 - beta) / (1 + beta) * off)
    nz = diag != 0
    assert np.all(np.abs(h[nz] - diag[nz]) <= 6.0 * sd[nz] + 1e-6)
    # the time average is a much tighter estimate (about 300 / 19 independent samples)
    avg = np.mean(tail, axis=0)
    assert np.all(np.abs(avg[nz] - diag[nz]) <= 6.0 * sd[nz] / np.sqrt(300 / 19.0) + 1e-6)
    rel = np.linalg.norm(avg[nz] - diag[nz]) / np.linalg.norm(diag[nz])
    assert rel < 0.1


def test_recurrence_rounding_order():
    # h' = fma(beta, h, fp32((1 - beta) * u)), u = fp32(fp32(z * hz) * inv_scale)
    beta = np.float32(0.9)
    omb = sub32(1.0, beta)
    z = np.array([1.0, -1.0, 1.0], np.float32)
    hz = np.array([0.3, 1.7e-3, -5.1], np.float32)
    h0 = np.array([0.7, -2.2e-3, 1.0 / 3.0], np.float32)
    inv = np.float32(1.0) / np.float32(3.0)
    h = h0.copy()
    curv_ema(z, hz, h, inv_scale=inv, beta=beta)
    for i in range(3):
        u = mul32(mul32(z[i], hz[i]), inv)
        expect = fma32(beta, h0[i], mul32(omb, u))
        assert bits(h[i]) == bits(expect)


def test_loss_scale_is_removed():
    z = np.array([1.0, -1.0], np.float32)
    hz = np.array([2.0, -6.0], np.float32) * 1024.0
    h = np.zeros(2, np.float32)
    curv_ema(z, hz, h, inv_scale=1.0 / 1024.0, first=1)
    assert np.array_equal(h, np.array([2.0, 6.0], np.float32))


def test_nonfinite_sample_freezes_the_element_and_raises_the_flag():
    z = np.ones(4, np.float32)
    hz = np.array([1.0, np.inf, np.nan, 2.0], np.float32)
    h = np.array([5.0, 6.0, 7.0, 8.0], np.float32)
    assert curv_ema(z, hz, h, beta=0.5) == 1
    assert np.array_equal(h, np.array([3.0, 6.0, 7.0, 5.0], np.float32))
