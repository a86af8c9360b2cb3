"""Pins for the oracle's parameter update: reduction to textbook SGD with momentum and L2
decay (the FP32 baseline optimizer of Sec. 4.1), exact rounding order, low-precision stores."""
import numpy as np
import pytest
import torch

import oracle
from _exact import bits, fma32, mul32

FP16, BF16, FP32 = 0, 1, 2


def update(buf, prev, new, g, gdt, m, inv_scale, wd, mu, eta):
    oracle.lib().oracle_update(buf.ctypes.data, prev, new, g.ctypes.data, gdt,
                               None if m is None else m.ctypes.data, g.size, np.float32(inv_scale),
                               np.float32(wd), np.float32(mu), np.float32(eta))


@pytest.mark.parametrize("mu,wd", [(0.9, 5e-4), (0.0, 0.0), (0.9, 0.0), (0.0, 1e-2)])
def test_reduces_to_library_sgd(mu, wd):
    rs = np.random.default_rng(0)
    n, lr = 1000, 0.05
    p0 = rs.standard_normal(n).astype(np.float32)
    tp = torch.nn.Parameter(torch.from_numpy(p0.copy()))
    opt = torch.optim.SGD([tp], lr=lr, momentum=mu, weight_decay=wd)
    buf = np.zeros(4 * n, np.uint8)
    buf.view(np.float32)[:] = p0
    m = np.zeros(n, np.float32) if mu else None
    for step in range(5):
        g = (rs.standard_normal(n) * 0.1).astype(np.float32)
        tp.grad = torch.from_numpy(g.copy())
        opt.step()
        update(buf, FP32, FP32, g, FP32, m, 1.0, wd, mu, lr)
        np.testing.assert_allclose(buf.view(np.float32), tp.detach().numpy(), rtol=2e-6, atol=1e-7)


def test_three_element_hand_calculation():
    theta = np.array([1.0, -0.5, 0.3], np.float32)
    g = np.array([0.25, 1.7, -3.1], np.float32) * np.float32(8.0)
    m0 = np.array([0.1, -0.2, 0.05], np.float32)
    inv, wd, mu, eta = np.float32(0.125), np.float32(5e-4), np.float32(0.9), np.float32(0.037)
    buf = np.zeros(12, np.uint8)
    buf.view(np.float32)[:] = theta
    m = m0.copy()
    update(buf, FP32, FP32, g, FP32, m, inv, wd, mu, eta)
    for i in range(3):
        gt = mul32(g[i], inv)
        d = fma32(wd, theta[i], gt)
        mm = fma32(mu, m0[i], d)
        th = fma32(-eta, mm, theta[i])
        assert bits(m[i]) == bits(mm)
        assert bits(buf.view(np.float32)[i]) == bits(th)


def test_no_momentum_buffer_means_m_equals_d():
    theta = np.array([2.0], np.float32)
    g = np.array([0.5], np.float32)
    buf = np.zeros(4, np.uint8)
    buf.view(np.float32)[:] = theta
    update(buf, FP32, FP32, g, FP32, None, 1.0, 0.0, 0.0, 0.5)
    assert buf.view(np.float32)[0] == 1.75


@pytest.mark.parametrize("prev,new", [(FP32, BF16), (FP32, FP16), (BF16, FP32), (FP16, FP32), (BF16, FP16),
                                      (FP16, BF16), (BF16, BF16), (FP16, FP16)])
def test_precision_transitions_store_the_rounded_fp32_result(prev, new):
    L = oracle.lib()
    rs = np.random.default_rng(prev * 3 + new)
    n = 257
    tdt = {FP16: torch.float16, BF16: torch.bfloat16, FP32: torch.float32}
    stored = torch.from_numpy(rs.standard_normal(n).astype(np.float32)).to(tdt[prev])
    wide = stored.to(torch.float32).numpy()
    g = (rs.standard_normal(n) * 0.01).astype(np.float32)
    buf = np.zeros(4 * n, np.uint8)
    raw = stored.view(torch.int16).numpy().view(np.uint16) if prev != FP32 else stored.numpy()
    buf.view(raw.dtype)[:n] = raw
    m = np.zeros(n, np.float32)
    update(buf, prev, new, g, FP32, m, 1.0, 0.0, 0.9, 0.1)
    # expected fp32 value: m = g (buffer was zero, decay zero), theta' = fma(-eta, g, theta)
    expect32 = np.array([fma32(-np.float32(0.1), g[i], wide[i]) for i in range(n)], np.float32)
    if new == FP32:
        assert np.array_equal(buf.view(np.float32)[:n], expect32)
    else:
        lib_cast = torch.from_numpy(expect32).to(tdt[new]).view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(buf.view(np.uint16)[:n], lib_cast)


def test_fp16_gradients_are_widened_then_unscaled():
    g16 = torch.tensor([1024.0, -3.0, 65504.0], dtype=torch.float16)
    raw = g16.view(torch.int16).numpy().view(np.uint16)
    buf = np.zeros(12, np.uint8)
    update(buf, FP32, FP32, raw, FP16, None, 1.0 / 1024.0, 0.0, 0.0, 1.0)
    assert buf.view(np.float32).tolist() == [-1.0, 3.0 / 1024.0, -65504.0 / 1024.0]
