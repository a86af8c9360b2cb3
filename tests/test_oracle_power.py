"""Pins of the oracle's power-iteration step (Sec. 3.2, third equation) against things it does
not compute itself: a hand-worked example, matrices with a known spectrum (library
eigen-decomposition), a library QR factorisation, and invariants of an orthonormal basis."""
import ctypes as C

import numpy as np
import pytest

import oracle
from oracle.capi import lib


def power_step(u, hu):
    """u, hu: (k, n) fp32.  Returns (u_next, rayleigh, resid, hnorm, deficient)."""
    k, n = u.shape
    u = np.ascontiguousarray(u, dtype=np.float32)
    hu = np.ascontiguousarray(hu, dtype=np.float32)
    out = np.empty_like(u)
    ray, res, hn = (np.zeros(k) for _ in range(3))
    d = C.c_uint32(0)
    P = C.POINTER(C.c_double)
    lib().oracle_power_step(u.ctypes.data, hu.ctypes.data, out.ctypes.data, n, k, ray.ctypes.data_as(P),
                            res.ctypes.data_as(P), hn.ctypes.data_as(P), C.byref(d))
    return out, ray, res, hn, d.value


def spd_with_spectrum(rng, lams):
    n = len(lams)
    q, _ = np.linalg.qr(rng.standard_normal((n, n)))
    return (q * np.asarray(lams)) @ q.T, q


def test_single_vector_hand_example():
    # u = (1, 2, 2), Hu = (3, 0, 4): quotient 11/9, ||Hu|| = 5, next = (0.6, 0, 0.8),
    # Hu - (11/9) u = (16, -22, 14)/9, its norm sqrt(936)/9, divided by ||u|| = 3
    out, ray, res, hn, d = power_step(np.array([[1, 2, 2]]), np.array([[3, 0, 4]]))
    assert ray[0] == pytest.approx(11 / 9, rel=1e-15)
    assert hn[0] == pytest.approx(5.0, rel=1e-15)
    assert res[0] == pytest.approx(np.sqrt(936) / 27, rel=1e-14)
    assert np.array_equal(out, np.array([[0.6, 0.0, 0.8]], dtype=np.float32)) and d == 0


def test_two_vectors_hand_example():
    # Hu_0 = (3, 4, 0) -> q_0 = (0.6, 0.8, 0); Hu_1 = (5, 0, 2): q_0.Hu_1 = 3,
    # remainder (5, 0, 2) - 3 (0.6, 0.8, 0) = (3.2, -2.4, 2), norm sqrt(20)
    u = np.array([[1, 0, 0], [0, 1, 0]])
    hu = np.array([[3, 4, 0], [5, 0, 2]])
    out, ray, res, hn, d = power_step(u, hu)
    want = np.array([[0.6, 0.8, 0.0], np.array([3.2, -2.4, 2.0]) / np.sqrt(20.0)])
    assert np.array_equal(out, want.astype(np.float32))
    assert ray == pytest.approx([3.0, 0.0]) and hn == pytest.approx([5.0, np.sqrt(29.0)])
    # residuals: ||(3,4,0) - 3 (1,0,0)|| = 4 ; ||(5,0,2) - 0|| = sqrt(29)
    assert res == pytest.approx([4.0, np.sqrt(29.0)])


def test_converges_to_the_top_k_eigenpairs_of_a_known_spectrum():
    rng = np.random.default_rng(5)
    lams = [10.0, 7.0, 5.0, 3.0, 2.0] + list(rng.uniform(0.01, 1.0, 59))
    H, q = spd_with_spectrum(rng, lams)
    w, v = np.linalg.eigh(H)              # independent library routine
    top = w[::-1][:5]
    assert top == pytest.approx([10, 7, 5, 3, 2], rel=1e-12)
    u = rng.standard_normal((5, 64)).astype(np.float32)
    for _ in range(400):
        hu = (u.astype(np.float64) @ H).astype(np.float32)   # H symmetric: rows of u times H
        u, ray, res, hn, d = power_step(u, hu)
    assert d == 0
    assert ray == pytest.approx(top, rel=2e-6)
    assert np.all(res < 1e-4)
    for j in range(5):
        assert abs(float(u[j].astype(np.float64) @ v[:, ::-1][:, j])) > 1 - 1e-6


def test_negative_eigenvalues_keep_their_sign_in_the_quotient():
    rng = np.random.default_rng(6)
    H, _ = spd_with_spectrum(rng, [-9.0, 4.0, 1.0, 0.5, 0.1, 0.05])
    u = rng.standard_normal((2, 6)).astype(np.float32)
    for _ in range(200):
        u, ray, res, hn, d = power_step(u, (u.astype(np.float64) @ H).astype(np.float32))
    assert ray == pytest.approx([-9.0, 4.0], rel=1e-5)


def test_matches_a_library_qr_and_is_orthonormal():
    rng = np.random.default_rng(7)
    k, n = 5, 1000
    u = rng.standard_normal((k, n)).astype(np.float32)
    hu = (rng.standard_normal((k, n)) * rng.uniform(0.1, 10, (k, 1))).astype(np.float32)
    out, ray, res, hn, d = power_step(u, hu)
    qq, rr = np.linalg.qr(hu.astype(np.float64).T)          # columns = vectors
    qq = qq * np.sign(np.diag(rr))                           # the basis with positive diagonal of R
    assert np.max(np.abs(out.astype(np.float64).T - qq)) < 1e-7
    g = out.astype(np.float64) @ out.astype(np.float64).T
    assert np.max(np.abs(g - np.eye(k))) < 1e-6
    # definitions written out with library reductions
    u64, w64 = u.astype(np.float64), hu.astype(np.float64)
    lam = np.einsum("ji,ji->j", u64, w64) / np.einsum("ji,ji->j", u64, u64)
    assert ray == pytest.approx(lam, rel=1e-12)
    assert hn == pytest.approx(np.linalg.norm(w64, axis=1), rel=1e-12)
    assert res == pytest.approx(np.linalg.norm(w64 - lam[:, None] * u64, axis=1) / np.linalg.norm(u64, axis=1), rel=1e-12)


def test_exact_eigenvectors_are_fixed_points():
    # diagonal H: unit vectors are eigenvectors; values chosen exactly representable
    lams = np.array([8.0, -4.0, 2.0, 0.5])
    u = np.eye(4, dtype=np.float32)[:3]
    out, ray, res, hn, d = power_step(u, u * lams[:3, None].astype(np.float32))
    assert np.array_equal(ray, lams[:3]) and np.all(res == 0) and np.array_equal(hn, np.abs(lams[:3]))
    assert np.array_equal(out, u * np.sign(lams[:3, None]).astype(np.float32)) and d == 0


def test_dependent_and_zero_vectors_are_flagged_and_zeroed():
    rng = np.random.default_rng(8)
    hu = rng.standard_normal((4, 50)).astype(np.float32)
    hu[2] = 2 * hu[0] - hu[1]           # in the span of the first two (up to fp32 rounding of the sum)
    hu[3] = 0
    u = rng.standard_normal((4, 50)).astype(np.float32)
    u[3] = 0
    out, ray, res, hn, d = power_step(u, hu)
    assert d == 0b1100
    assert not out[2].any() and not out[3].any()
    assert ray[3] == 0 and res[3] == 0 and hn[3] == 0
    g = out[:2].astype(np.float64) @ out[:2].astype(np.float64).T
    assert np.max(np.abs(g - np.eye(2))) < 1e-6


def test_rank_threshold_separates_rounding_from_a_small_but_real_direction():
    # remainder^2 <= 1e-12 ||Hu||^2 means "no direction left".  A second vector that differs from the
    # first by a relative 1e-4 (remainder^2 / norm^2 = 1e-8) is nearly parallel but still carries a
    # direction and must be kept and orthonormalised; one that differs by 1e-7 (1e-14) must be flagged.
    n = 64
    e0, e1 = np.zeros(n), np.zeros(n)
    e0[0], e1[1] = 1.0, 1.0
    u = np.ones((2, n), dtype=np.float32)
    for eps, flagged in ((1e-4, False), (1e-7, True)):
        hu = np.stack([e0, e0 + eps * e1]).astype(np.float32)
        out, _, _, _, d = power_step(u, hu)
        assert d == (0b10 if flagged else 0)
        if flagged:
            assert not out[1].any()
        else:
            assert abs(abs(out[1][1]) - 1.0) < 1e-6 and abs(out[1][0]) < 1e-6


def test_latched_lambda_feeds_the_step_size_and_the_promotion():
    rng = np.random.default_rng(9)
    n = 40
    cfg = oracle.OracleConfig(lambda_source=1, alpha=0.5, tau_curv=3.0, tau_low=1e-5, tau_high=3e-5, momentum=0.0,
                              weight_decay=0.0)
    p = rng.standard_normal(n).astype(np.float32)
    orc = oracle.OracleTriAccel(cfg, [p], [2], [2])
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)    # variance 1e-6: FP16 by the variance rule
    u = np.zeros((2, n), dtype=np.float32)
    u[0, 0] = 1
    u[1, 1] = 1
    hu = np.zeros((2, n), dtype=np.float32)
    hu[0, 0] = -6.0                                            # quotients -6 and 2: lambda = 6
    hu[1, 1] = 2.0
    orc.power_step([u], [hu], 2, latch=True)
    t = orc.tensors[0]
    assert t.lam_power == np.float32(6.0) and list(t.rayleigh) == [-6.0, 2.0]
    orc.step([g], [None], [None], lr=0.1, loss_scale=1.0, batch_size=64, mem_used=8, mem_total=10)
    assert t.lam == np.float32(6.0) and t.eta == np.float32(np.float32(0.1) / np.float32(4.0))
    assert t.code == 1                                         # FP16 by variance, promoted once: 6 > 3
    # without latching the layer keeps its previous lambda
    hu[0, 0] = 1.0
    u[:] = 0
    u[0, 0] = 1
    u[1, 1] = 1
    orc.power_step([u], [hu], 2, latch=False)
    assert t.lam_power == np.float32(6.0)
