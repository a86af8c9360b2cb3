"""Pins for the oracle's number-format conversions.

The oracle rounds by the formats' definition (scale, round-half-even, rescale).  It is
compared, over all 2^32 binary32 patterns, with independent library conversions on the CPU
(PyTorch's float16 and bfloat16 casts), and on a random sample with numpy's float16.  NaNs
are compared by NaN-ness only.
"""
import multiprocessing as mp

import numpy as np
import torch

import oracle

BATCH = 1 << 24


def _check_batch(b):
    torch.set_num_threads(1)
    L = oracle.lib()
    bits = np.arange(BATCH, dtype=np.uint32) + np.uint32(b * BATCH)
    x = bits.view(np.float32)
    nan = np.isnan(x)
    got = np.empty(BATCH, np.uint16)
    L.oracle_f32_to_f16_array(x.ctypes.data, got.ctypes.data, BATCH)
    ref = torch.from_numpy(x).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    bad16 = int(np.count_nonzero((got != ref) & ~nan))
    nan_ok16 = bool(np.all(((got[nan] & 0x7C00) == 0x7C00) & ((got[nan] & 0x03FF) != 0)))
    L.oracle_f32_to_bf16_array(x.ctypes.data, got.ctypes.data, BATCH)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    badb = int(np.count_nonzero((got != ref) & ~nan))
    nan_okb = bool(np.all(((got[nan] & 0x7F80) == 0x7F80) & ((got[nan] & 0x007F) != 0)))
    return bad16, badb, nan_ok16, nan_okb


def test_f32_to_f16_and_bf16_exhaustive():
    oracle.lib()  # build before forking
    with mp.get_context("fork").Pool(8) as pool:
        res = pool.map(_check_batch, range((1 << 32) // BATCH), chunksize=4)
    assert sum(r[0] for r in res) == 0
    assert sum(r[1] for r in res) == 0
    assert all(r[2] for r in res) and all(r[3] for r in res)


def test_f32_to_f16_vs_numpy_sample():
    L = oracle.lib()
    rs = np.random.default_rng(5)
    bits = rs.integers(0, 1 << 32, size=1 << 22, dtype=np.uint64).astype(np.uint32)
    x = bits.view(np.float32)
    got = np.empty(x.size, np.uint16)
    L.oracle_f32_to_f16_array(x.ctypes.data, got.ctypes.data, x.size)
    with np.errstate(over="ignore", invalid="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    nan = np.isnan(x)
    assert np.array_equal(got[~nan], ref[~nan])


def test_f16_to_f32_exhaustive():
    L = oracle.lib()
    h = np.arange(1 << 16, dtype=np.uint32).astype(np.uint16)
    out = np.empty(1 << 16, np.float32)
    L.oracle_f16_to_f32_array(h.ctypes.data, out.ctypes.data, 1 << 16)
    ref = h.view(np.float16).astype(np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(out[~nan].view(np.uint32), ref[~nan].view(np.uint32))
    assert np.all(np.isnan(out[nan]))


def test_hand_cases():
    L = oracle.lib()
    # binary16: 1 + 2^-11 is a tie between 1 and 1 + 2^-10 -> even (1.0)
    assert L.oracle_f32_to_f16(1.0 + 2.0 ** -11) == 0x3C00
    assert L.oracle_f32_to_f16(1.0 + 3 * 2.0 ** -11) == 0x3C02  # tie -> even (up)
    assert L.oracle_f32_to_f16(65504.0) == 0x7BFF
    assert L.oracle_f32_to_f16(65519.996) == 0x7BFF
    assert L.oracle_f32_to_f16(65520.0) == 0x7C00  # tie at the top rounds to infinity
    assert L.oracle_f32_to_f16(2.0 ** -24) == 0x0001  # smallest subnormal
    assert L.oracle_f32_to_f16(2.0 ** -25) == 0x0000  # tie with zero -> even (zero)
    assert L.oracle_f32_to_f16(-(2.0 ** -25) * 1.0000001) == 0x8001
    assert L.oracle_f32_to_f16(-0.0) == 0x8000
    # bfloat16: 8 significant bits
    assert L.oracle_f32_to_bf16(1.0 + 2.0 ** -8) == 0x3F80  # tie -> even
    assert L.oracle_f32_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82
    tie_top = float(np.array([0x7F7F8000], np.uint32).view(np.float32)[0])  # max bf16 + half an ulp
    below = float(np.array([0x7F7F7FFF], np.uint32).view(np.float32)[0])
    assert L.oracle_f32_to_bf16(tie_top) == 0x7F80  # tie at the top rounds to infinity
    assert L.oracle_f32_to_bf16(below) == 0x7F7F
    assert L.oracle_f32_to_bf16(float("inf")) == 0x7F80
    assert L.oracle_f32_to_bf16(float("-inf")) == 0xFF80
