"""Pins for the oracle's gradient statistics and the variance EMA (Sec. 3.1, first equation)."""
import ctypes as C
import itertools
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from _exact import frac

FP16, BF16, FP32 = 0, 1, 2


def stats(g, dtype=FP32, inv_scale=1.0):
    L = oracle.lib()
    mean, var = C.c_double(), C.c_double()
    L.oracle_grad_stats(g.ctypes.data, dtype, g.size, np.float32(inv_scale), C.byref(mean), C.byref(var))
    return mean.value, var.value


def test_brute_force_small_integer_tensors():
    # every tensor of length 1..4 with entries in {-2..2}: exact rational mean / variance
    for n in range(1, 5):
        for vals in itertools.product(range(-2, 3), repeat=n):
            g = np.array(vals, dtype=np.float32)
            m = Fraction(sum(vals), n)
            v = sum((Fraction(x) - m) ** 2 for x in vals) / n
            mean, var = stats(g)
            assert mean == pytest.approx(float(m), rel=0, abs=1e-15)
            assert var == pytest.approx(float(v), rel=1e-15, abs=1e-15)


def test_population_not_sample_variance():
    mean, var = stats(np.array([1, 2, 3, 4], np.float32))
    assert mean == 2.5 and var == 1.25  # divide by n (sample variance would be 5/3)
    assert stats(np.array([7.5], np.float32)) == (7.5, 0.0)  # n = 1 is defined


@pytest.mark.parametrize("n", [1, 2, 33, 1000, 100003])
def test_matches_numpy_population_variance(n):
    rs = np.random.default_rng(n)
    g = (rs.standard_t(3, size=n) * 1e-3).astype(np.float32)
    mean, var = stats(g)
    g64 = g.astype(np.float64)
    assert mean == pytest.approx(g64.mean(), rel=1e-12, abs=1e-18)
    assert var == pytest.approx(g64.var(ddof=0), rel=1e-12)


def test_exact_rational_with_large_offset():
    # Var[x + c] at c = 1e4 sigma: compare with exact rational arithmetic on the rounded inputs
    rs = np.random.default_rng(3)
    g = (rs.standard_normal(500) * 1e-3 + 10.0).astype(np.float32)
    xs = [frac(v) for v in g]
    m = sum(xs) / len(xs)
    v = sum((x - m) ** 2 for x in xs) / len(xs)
    mean, var = stats(g)
    assert mean == pytest.approx(float(m), rel=1e-14)
    assert var == pytest.approx(float(v), rel=1e-9)
    assert var == pytest.approx(1e-6, rel=0.2)


def test_unscaling_is_one_fp32_multiply():
    # 3 * fp32(1/3) rounds to exactly 1 in fp32; a double multiply would give 1.0000000298
    inv = np.float32(1.0) / np.float32(3.0)
    mean, var = stats(np.array([3.0, 3.0], np.float32), inv_scale=inv)
    assert mean == 1.0 and var == 0.0


def test_half_precision_gradients():
    rs = np.random.default_rng(11)
    x = rs.standard_normal(4097).astype(np.float32) * 300.0
    for dtype, tdt in ((FP16, torch.float16), (BF16, torch.bfloat16)):
        stored = torch.from_numpy(x).to(tdt)
        raw = stored.view(torch.int16).numpy().view(np.uint16)
        inv = np.float32(1.0 / 1024.0)
        mean, var = stats(raw, dtype, inv)
        ref = (stored.to(torch.float32).numpy() * inv).astype(np.float64)
        assert mean == pytest.approx(ref.mean(), rel=1e-12)
        assert var == pytest.approx(ref.var(), rel=1e-12)


def test_found_nonfinite():
    L = oracle.lib()
    g = np.zeros(100, np.float32)
    assert L.oracle_found_nonfinite(g.ctypes.data, FP32, 100) == 0
    for bad in (np.inf, -np.inf, np.nan):
        h = g.copy()
        h[57] = bad
        assert L.oracle_found_nonfinite(h.ctypes.data, FP32, 100) == 1
    big = np.full(10, np.finfo(np.float32).max, np.float32)
    assert L.oracle_found_nonfinite(big.ctypes.data, FP32, 10) == 0
    h16 = np.zeros(10, np.uint16)
    h16[3] = 0x7C00
    assert L.oracle_found_nonfinite(h16.ctypes.data, FP16, 10) == 1
    h16[3] = 0x7BFF
    assert L.oracle_found_nonfinite(h16.ctypes.data, FP16, 10) == 0
    h16[3] = 0x7F80  # bf16 inf (a finite number when read as binary16... and vice versa)
    assert L.oracle_found_nonfinite(h16.ctypes.data, BF16, 10) == 1
    h16[3] = 0xFFC1  # bf16 NaN
    assert L.oracle_found_nonfinite(h16.ctypes.data, BF16, 10) == 1


# ---- variance EMA ----------------------------------------------------------------------

def ema(v_prev, var, beta, first=0):
    return oracle.lib().oracle_var_ema(np.float32(v_prev), float(var), np.float32(beta), first)


def test_ema_first_step_is_the_variance():
    assert ema(123.0, 0.25, 0.9, first=1) == 0.25


def test_ema_constant_input_is_a_fixed_point():
    v = 0.125
    for _ in range(50):
        v = ema(v, 0.125, 0.9)
    assert v == 0.125


def test_ema_beta_zero_tracks_the_variance():
    assert ema(5.0, 0.75, 0.0) == 0.75


def test_ema_closed_form_geometric_response():
    # v(t) = beta^(t-1) v(1) + (1 - beta^(t-1)) c   for constant variance c after the first step
    beta, v1, c = 0.5, 8.0, 2.0  # dyadic numbers: every step is exact
    v = ema(0.0, v1, beta, first=1)
    for t in range(2, 12):
        v = ema(v, c, beta)
        assert v == beta ** (t - 1) * v1 + (1 - beta ** (t - 1)) * c


def test_ema_weights():
    # one step from v=1 with var=0, beta=0.9f: result is fp32(beta) exactly (weights beta, 1-beta)
    b = np.float32(0.9)
    assert ema(1.0, 0.0, b) == float(b)
    assert ema(0.0, 1.0, b) == float(np.float32(1.0 - float(b)))
