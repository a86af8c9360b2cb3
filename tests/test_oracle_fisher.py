"""Pins for the empirical-Fisher source of the diagonal curvature EMA (Sec. 1 / 3.2: "Hessian or
Fisher" entries): the sample is the squared unscaled gradient."""
import ctypes as C

import numpy as np

import oracle
from _exact import fma32, mul32, sub32


def fisher_ema(g, h, dtype=2, inv_scale=1.0, beta=0.9, first=0):
    flag = C.c_uint32(0)
    oracle.lib().oracle_fisher_ema(g.ctypes.data, dtype, h.ctypes.data, h.size, np.float32(inv_scale),
                                   np.float32(beta), first, C.byref(flag))
    return flag.value


def hutchinson_ema(z, hz, h, inv_scale=1.0, beta=0.9, first=0):
    flag = C.c_uint32(0)
    oracle.lib().oracle_curv_ema(z.ctypes.data, hz.ctypes.data, h.ctypes.data, h.size, np.float32(inv_scale),
                                 np.float32(beta), first, C.byref(flag))
    return flag.value


def test_equals_the_hutchinson_estimate_of_a_diagonal_hessian_of_squared_gradients():
    # H = diag(g^2): z * (H z) = g^2 for any sign vector, so both sources must give the same h
    rs = np.random.default_rng(0)
    g = rs.standard_normal(1000).astype(np.float32)
    z = rs.choice([-1.0, 1.0], size=g.size).astype(np.float32)
    hz = (g * g) * z                      # fp32 square, exact sign flip
    h1 = np.zeros(g.size, np.float32)
    h2 = np.zeros(g.size, np.float32)
    for first in (1, 0, 0):
        assert fisher_ema(g, h1, first=first) == 0
        assert hutchinson_ema(z, hz, h2, first=first) == 0
        assert np.array_equal(h1.view(np.uint32), h2.view(np.uint32))


def test_first_sample_is_the_square_and_later_ones_follow_the_ema_exactly():
    g = np.array([3.0, -0.5, 0.0, 1e-3, 7.25], np.float32)
    h = np.full(5, 42.0, np.float32)
    fisher_ema(g, h, first=1)
    assert np.array_equal(h, g * g)
    g2 = np.array([1.0, 2.0, -4.0, 0.5, 0.0], np.float32)
    before = h.copy()
    fisher_ema(g2, h, beta=0.75)
    omb = sub32(1.0, 0.75)
    for i in range(5):
        u = mul32(g2[i], g2[i])
        assert h[i] == fma32(0.75, before[i], mul32(omb, u)), i


def test_loss_scale_is_removed_before_squaring():
    rs = np.random.default_rng(1)
    g = rs.standard_normal(300).astype(np.float32)
    h1 = np.zeros(300, np.float32)
    h2 = np.zeros(300, np.float32)
    fisher_ema(g, h1, first=1)
    fisher_ema(g * np.float32(1024.0), h2, inv_scale=1.0 / 1024.0, first=1)   # power of two: exact
    assert np.array_equal(h1, h2)
    # half-precision gradient storage is widened exactly first
    g16 = g.astype(np.float16)
    h3 = np.zeros(300, np.float32)
    fisher_ema(g16.view(np.uint16), h3, dtype=0, first=1)
    assert np.array_equal(h3, g16.astype(np.float32) ** 2)


def test_overflowing_square_freezes_the_element_and_raises_the_flag():
    g = np.array([1.0, 3e19, -2.0], np.float32)        # (3e19)^2 is beyond fp32
    h = np.array([5.0, 6.0, 7.0], np.float32)
    assert fisher_ema(g, h, beta=0.5) == 1
    assert h[1] == 6.0 and h[0] == np.float32(0.5 * 5.0 + 0.5 * 1.0) and h[2] == np.float32(0.5 * 7.0 + 0.5 * 4.0)


def test_step_uses_the_gradient_as_the_sample_and_needs_no_probe():
    rs = np.random.default_rng(2)
    n = 64
    cfg = oracle.OracleConfig(curvature_source=1, sparsity_ppm=750000, momentum=0.0, weight_decay=0.0, alpha=0.0)
    orc = oracle.OracleTriAccel(cfg, [np.zeros(n, np.float32)], [2], [2])
    g = rs.standard_normal(n).astype(np.float32)
    orc.step([g], [None], [None], 0.1, 1.0, 64, 8, 10)
    t = orc.tensors[0]
    assert np.array_equal(t.curv, g * g)
    k = n - (n * 750000) // 1000000
    assert t.nnz == k and t.theta == np.sort(g * g)[::-1][k - 1] and t.lam == np.max(g * g)
    # a step that does not refresh the curvature keeps h, theta and the mask
    keep = (t.curv.copy(), t.mask.copy(), t.theta)
    orc.step([rs.standard_normal(n).astype(np.float32)], [None], [None], 0.1, 1.0, 64, 8, 10, update_curvature=False)
    assert np.array_equal(t.curv, keep[0]) and np.array_equal(t.mask, keep[1]) and t.theta == keep[2]
