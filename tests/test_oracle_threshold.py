"""Pins for the oracle's magnitude threshold and sparsity mask ("top-k Hessian or Fisher
entries", Sec. 1 / 3.2)."""
import ctypes as C

import numpy as np
import pytest

import oracle


def select(h, s_ppm):
    h = np.ascontiguousarray(h, dtype=np.float32)
    mask = np.zeros((h.size + 31) // 32, np.uint32)
    theta, nnz, lam = C.c_float(), C.c_uint32(), C.c_float()
    oracle.lib().oracle_threshold_mask(h.ctypes.data, h.size, s_ppm, mask.ctypes.data, C.byref(theta),
                                       C.byref(nnz), C.byref(lam))
    bitsv = np.unpackbits(mask.view(np.uint8), bitorder="little")[: h.size].astype(bool)
    return theta.value, nnz.value, lam.value, bitsv, mask


def test_topk_count_formula():
    L = oracle.lib()
    assert L.oracle_topk_count(10, 900000) == 1
    assert L.oracle_topk_count(101, 950000) == 6          # 101 - floor(95.95)
    assert L.oracle_topk_count(100, 0) == 100
    assert L.oracle_topk_count(100, 1000000) == 1         # clamped from 0
    assert L.oracle_topk_count(1, 999999) == 1
    assert L.oracle_topk_count(16777216, 950000) == 16777216 - 15938355
    assert L.oracle_topk_count(1 << 40, 999999) == (1 << 40) - ((1 << 40) * 999999) // 1000000


def test_hand_case_five_elements():
    # magnitudes {1,5,3,0,2}; keep 2 of 5 (s = 60 %): theta = 3, bits for 5 and 3
    theta, nnz, lam, b, _ = select([1, -5, 3, 0, 2], 600000)
    assert (theta, nnz, lam) == (3.0, 2, 5.0)
    assert b.tolist() == [False, True, True, False, False]


def test_ties_are_all_kept():
    theta, nnz, lam, b, _ = select([2, -2, 2, 1, 2, 0.5], 500000)  # k = 3, but four entries tie at 2
    assert (theta, nnz, lam) == (2.0, 4, 2.0)
    assert b.tolist() == [True, True, True, False, True, False]


def test_all_equal_all_zero_single():
    theta, nnz, lam, b, _ = select([3.0] * 7, 900000)
    assert (theta, nnz) == (3.0, 7) and b.all()
    theta, nnz, lam, b, _ = select([0.0, -0.0, 0.0], 0)
    assert (theta, nnz, lam) == (0.0, 0, 0.0) and not b.any()
    theta, nnz, lam, b, _ = select([-4.0], 999999)
    assert (theta, nnz, lam) == (4.0, 1, 4.0) and b.all()


def test_zeros_never_enter_the_mask_even_when_theta_is_zero():
    theta, nnz, lam, b, _ = select([0, 0, 1.5, 0, -0.25, 0], 0)  # k = n = 6 > number of non-zeros
    assert (theta, nnz, lam) == (0.0, 2, 1.5)
    assert b.tolist() == [False, False, True, False, True, False]


def test_bit_layout():
    h = np.zeros(70, np.float32)
    h[[0, 31, 32, 69]] = [1, 2, 3, 4]
    theta, nnz, lam, b, mask = select(h, 0)
    assert mask.tolist() == [(1 << 0) | (1 << 31), 1 << 0, 1 << 5]


def test_subnormal_and_sign():
    tiny = np.float32(1e-45)
    theta, nnz, lam, b, _ = select([tiny, -3 * tiny, 0, 2 * tiny], 500000)  # k = 2
    assert theta == float(2 * tiny) and nnz == 2 and b.tolist() == [False, True, False, True]


@pytest.mark.parametrize("n,s_ppm", [(1, 0), (31, 500000), (32, 950000), (1000, 950000), (4097, 900000),
                                      (100001, 999000), (65536, 0)])
def test_invariants_and_numpy_partition(n, s_ppm):
    rs = np.random.default_rng(n)
    h = (rs.standard_normal(n) * rs.choice([1e-3, 1.0, 50.0], size=n)).astype(np.float32)
    h[rs.uniform(size=n) < 0.2] = 0.0
    h[rs.uniform(size=n) < 0.1] = 0.5  # ties
    theta, nnz, lam, b, _ = select(h, s_ppm)
    a = np.abs(h)
    k = n - (n * s_ppm) // 1000000
    k = min(max(k, 1), n)
    assert theta == float(np.partition(a, n - k)[n - k])      # k-th largest via a library routine
    assert np.array_equal(b, (a >= theta) & (a > 0))
    assert nnz == int(b.sum())
    assert np.count_nonzero(a > theta) < k
    assert nnz >= min(k, np.count_nonzero(a > 0))
    assert lam == (float(a.max()) if nnz else 0.0)


def select_k(h, k):
    h = np.ascontiguousarray(h, dtype=np.float32)
    mask = np.zeros((h.size + 31) // 32, np.uint32)
    theta, nnz, lam = C.c_float(), C.c_uint32(), C.c_float()
    oracle.lib().oracle_threshold_mask_k(h.ctypes.data, h.size, k, mask.ctypes.data, C.byref(theta), C.byref(nnz),
                                         C.byref(lam))
    bitsv = np.unpackbits(mask.view(np.uint8), bitorder="little")[: h.size].astype(bool)
    return theta.value, nnz.value, lam.value, bitsv


def test_fixed_k_keeps_the_k_largest_magnitudes():
    # the paper's top-k with k = 5 (Sec. 4.1): threshold = fifth largest magnitude
    h = np.array([0.5, -9.0, 3.0, 7.5, -1.0, 0.0, 2.0, -4.0, 6.0, 0.25], np.float32)
    theta, nnz, lam, b = select_k(h, 5)
    assert (theta, nnz, lam) == (3.0, 5, 9.0)
    assert b.tolist() == [False, True, True, True, False, False, False, True, True, False]
    # against a library partial sort on random data
    rs = np.random.default_rng(4)
    x = rs.standard_normal(5000).astype(np.float32)
    for k in (1, 5, 64, 4999, 5000):
        theta, nnz, lam, b = select_k(x, k)
        want = np.partition(np.abs(x), x.size - k)[x.size - k]
        assert theta == want and nnz == k and b.sum() == k and lam == np.abs(x).max()
    # clamps: k above n keeps every non-zero entry, k below 1 keeps the largest
    assert select_k([1, 0, -2], 10)[1] == 2 and select_k([1, 0, -2], 0)[:2] == (2.0, 1)
    # same function as the fractional form when the counts agree
    for s_ppm in (900000, 500000):
        k = oracle.lib().oracle_topk_count(x.size, s_ppm)
        assert select_k(x, k)[:3] == select(x, s_ppm)[:3]
