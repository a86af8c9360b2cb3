"""Pins for the oracle's per-layer decisions: precision rule and promotion (Sec. 3.1 / 3.2),
step-size scaling (Sec. 3.2), batch rule (Sec. 3.3), loss-scale schedule."""
import ctypes as C
import os

import numpy as np

import oracle
from _exact import bits, div32, fma32

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rows(name):
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                yield line.split()


def test_precision_rule_golden_cases():
    L = oracle.lib()
    n = 0
    for v, lam, tl, th, tc, want in rows("precision_rule_cases.txt"):
        got = L.oracle_precision_code(np.float32(v), np.float32(lam), np.float32(tl), np.float32(th), np.float32(tc))
        assert got == int(want), (v, lam, tl, th, tc)
        n += 1
    assert n >= 15


def test_precision_rule_is_monotone():
    L = oracle.lib()
    vs = np.geomspace(1e-8, 1.0, 200).astype(np.float32)
    for lam in (0.0, 2.0):
        codes = [L.oracle_precision_code(v, np.float32(lam), np.float32(1e-5), np.float32(3e-5), np.float32(1.0))
                 for v in vs]
        assert codes == sorted(codes) and set(codes) <= {0, 1, 2}
    assert all(L.oracle_precision_code(v, np.float32(2.0), 1e-5, 3e-5, 1.0)
               >= L.oracle_precision_code(v, np.float32(0.0), 1e-5, 3e-5, 1.0) for v in vs)


def test_eta_closed_forms():
    L = oracle.lib()
    lr = np.float32(0.1)
    assert L.oracle_eta(lr, np.float32(0.0), np.float32(123.0)) == float(lr)        # alpha = 0
    assert L.oracle_eta(lr, np.float32(0.7), np.float32(0.0)) == float(lr)          # lambda = 0
    assert L.oracle_eta(lr, np.float32(0.25), np.float32(4.0)) == float(lr) / 2      # lambda = 1/alpha
    lams = np.linspace(0, 50, 101).astype(np.float32)
    etas = [L.oracle_eta(lr, np.float32(0.1), l) for l in lams]
    assert all(a >= b for a, b in zip(etas, etas[1:])) and etas[-1] > 0
    # rounding: one fma for the denominator, one correctly rounded division
    a, lam = np.float32(0.1), np.float32(3.3333333)
    assert bits(L.oracle_eta(lr, a, lam)) == bits(div32(lr, fma32(a, lam, 1.0)))


def test_batch_rule_golden_trace():
    L = oracle.lib()
    n = 0
    for b, used, want in rows("batch_rule_trace.txt"):
        got = L.oracle_batch_next(int(b), int(used), 1000, 0.70, 0.90, 16, 32, 16, 160)
        assert got == int(want), (b, used)
        n += 1
    assert n >= 13


def test_loss_scale_schedule():
    L = oracle.lib()
    good = C.c_int32(0)
    s = 1024.0
    trace = []
    for skipped in (0, 0, 0, 1, 0, 0, 0, 0, 1, 1, 0):
        s = L.oracle_loss_scale_next(np.float32(s), skipped, C.byref(good), np.float32(0.5), np.float32(2.0), 3)
        trace.append((s, good.value))
    assert trace == [(1024, 1), (1024, 2), (2048, 0), (1024, 0), (1024, 1), (1024, 2), (2048, 0), (2048, 1),
                     (1024, 0), (512, 0), (512, 1)]
