"""Pins for the element-wise form of the curvature-scaled step size (Sec. 3.2, fourth equation
applied per entry of the sparsified curvature)."""
import numpy as np
import pytest

import oracle
from _exact import div32, fma32, mul32

FP16, BF16, FP32 = 0, 1, 2


def update(buf, prev, new, g, gdt, m, inv_scale, wd, mu, eta):
    oracle.lib().oracle_update(buf.ctypes.data, prev, new, g.ctypes.data, gdt,
                               None if m is None else m.ctypes.data, g.size, np.float32(inv_scale),
                               np.float32(wd), np.float32(mu), np.float32(eta))


def update_elem(buf, prev, new, g, gdt, m, h, mask, inv_scale, wd, mu, lr, alpha):
    oracle.lib().oracle_update_elementwise(buf.ctypes.data, prev, new, g.ctypes.data, gdt,
                                           None if m is None else m.ctypes.data, h.ctypes.data, mask.ctypes.data,
                                           g.size, np.float32(inv_scale), np.float32(wd), np.float32(mu),
                                           np.float32(lr), np.float32(alpha))


def pack(bits):
    n = len(bits)
    words = np.zeros((n + 31) // 32, np.uint32)
    for i, b in enumerate(bits):
        if b:
            words[i // 32] |= np.uint32(1 << (i % 32))
    return words


def fresh(n, rs, code=FP32):
    p = rs.standard_normal(n).astype(np.float32)
    buf = np.zeros(4 * n, np.uint8)
    if code == FP32:
        buf.view(np.float32)[:n] = p
    else:
        import torch
        t = torch.from_numpy(p).to(torch.bfloat16 if code == BF16 else torch.float16)
        buf.view(np.uint16)[:n] = t.view(torch.int16).numpy().view(np.uint16)
    return buf


@pytest.mark.parametrize("prev,new", [(FP32, FP32), (FP32, BF16), (BF16, FP16), (FP16, FP32)])
def test_constant_curvature_and_full_mask_is_the_per_layer_rule(prev, new):
    rs = np.random.default_rng(0)
    n, lr, alpha, c = 777, 0.1, 0.3, 2.5
    g = (rs.standard_normal(n) * 0.1).astype(np.float32)
    a, b = fresh(n, rs, prev), None
    b = a.copy()
    ma, mb = np.full(n, 0.01, np.float32), np.full(n, 0.01, np.float32)
    h = np.full(n, -c, np.float32)                   # the magnitude counts, not the sign
    eta = oracle.lib().oracle_eta(np.float32(lr), np.float32(alpha), np.float32(c))
    update(a, prev, new, g, FP32, ma, 1.0, 5e-4, 0.9, eta)
    update_elem(b, prev, new, g, FP32, mb, h, pack([1] * n), 1.0, 5e-4, 0.9, lr, alpha)
    assert np.array_equal(a, b) and np.array_equal(ma, mb)


def test_unmasked_entries_take_the_base_learning_rate():
    rs = np.random.default_rng(1)
    n, lr = 100, 0.05
    g = rs.standard_normal(n).astype(np.float32)
    a = fresh(n, rs)
    b = a.copy()
    h = (rs.standard_normal(n) * 100).astype(np.float32)
    update(a, FP32, FP32, g, FP32, None, 1.0, 0.0, 0.0, lr)
    update_elem(b, FP32, FP32, g, FP32, None, h, pack([0] * n), 1.0, 0.0, 0.0, lr, 7.0)
    assert np.array_equal(a, b)


def test_hand_example_with_a_mixed_mask():
    theta = np.array([1.0, -2.0, 0.5, 4.0], np.float32)
    g = np.array([0.5, 0.25, -1.0, 2.0], np.float32)
    h = np.array([3.0, -1.0, 8.0, 0.125], np.float32)
    bits = [1, 1, 0, 1]
    lr, alpha = np.float32(0.1), np.float32(0.5)
    buf = np.zeros(16, np.uint8)
    buf.view(np.float32)[:] = theta
    update_elem(buf, FP32, FP32, g, FP32, None, h, pack(bits), 1.0, 0.0, 0.0, lr, alpha)
    got = buf.view(np.float32)
    # denominators 1 + 0.5 * {3, 1, 0, 0.125} = {2.5, 1.5, 1, 1.0625}
    for i, den in enumerate([2.5, 1.5, 1.0, 1.0625]):
        eta = div32(lr, np.float32(den))
        assert got[i] == fma32(-eta, g[i], theta[i]), i
    # a masked entry with more curvature moves less for the same gradient
    buf2 = np.zeros(8, np.uint8)
    buf2.view(np.float32)[:] = [1.0, 1.0]
    update_elem(buf2, FP32, FP32, np.array([1.0, 1.0], np.float32), FP32, None, np.array([0.5, 50.0], np.float32),
                pack([1, 1]), 1.0, 0.0, 0.0, lr, alpha)
    step = 1.0 - buf2.view(np.float32)
    assert step[0] > step[1] > 0


def test_momentum_and_decay_enter_as_in_the_per_layer_update():
    theta = np.array([1.5], np.float32)
    g = np.array([8.0], np.float32)      # stored with loss scale 16
    m = np.array([0.25], np.float32)
    h = np.array([-2.0], np.float32)
    wd, mu, lr, alpha = np.float32(0.01), np.float32(0.9), np.float32(0.2), np.float32(0.25)
    buf = np.zeros(4, np.uint8)
    buf.view(np.float32)[:] = theta
    update_elem(buf, FP32, FP32, g, FP32, m, h, pack([1]), 1.0 / 16.0, wd, mu, lr, alpha)
    d = fma32(wd, theta[0], mul32(g[0], np.float32(1.0 / 16.0)))
    mm = fma32(mu, np.float32(0.25), d)
    eta = div32(lr, fma32(alpha, np.float32(2.0), np.float32(1.0)))
    assert m[0] == mm and buf.view(np.float32)[0] == fma32(-eta, mm, theta[0])


def test_step_uses_this_steps_curvature_and_mask():
    rs = np.random.default_rng(3)
    n = 96
    cfg = oracle.OracleConfig(elementwise_scale=1, sparsity_ppm=500000, momentum=0.0, weight_decay=0.0, alpha=2.0,
                              tau_low=0.0, tau_high=0.0)
    p = rs.standard_normal(n).astype(np.float32)
    orc = oracle.OracleTriAccel(cfg, [p.copy()], [FP32], [FP32])
    g = rs.standard_normal(n).astype(np.float32)
    z = rs.choice([-1.0, 1.0], n).astype(np.float32)
    d = rs.uniform(0.1, 5.0, n).astype(np.float32)
    orc.step([g], [z], [d * z], 0.1, 1.0, 64, 8, 10)
    t = orc.tensors[0]
    assert np.array_equal(t.curv, d) and t.nnz == 48
    kept = t.mask_bits()
    den = np.where(kept, np.float32(1.0) + np.float32(2.0) * d, np.float32(1.0)).astype(np.float32)
    want = p - (np.float32(0.1) / den) * g
    np.testing.assert_allclose(t.param_f32(), want, rtol=1e-6)
    assert np.all(np.abs(t.param_f32() - p)[kept] < np.abs(np.float32(0.1) * g)[kept])
