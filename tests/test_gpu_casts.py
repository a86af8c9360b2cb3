"""GPU parity of the round-to-nearest-even stores: every one of the 2^32 binary32 patterns (visited
as int32 values from -2^31 upward) is
converted by the HIP library (the store path of the update kernel) and by the CPU oracle; the
16-bit results must be identical (NaNs compared by NaN-ness only)."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import oracle
import paper_2508_16905_amd as ta

pytestmark = pytest.mark.gpu

BATCH = 1 << 26


def _oracle_slice(args):
    x, got16, gotb = args
    L = oracle.lib()
    n = x.size
    ref = np.empty(n, np.uint16)
    nan = np.isnan(x)
    L.oracle_f32_to_f16_array(x.ctypes.data, ref.ctypes.data, n)
    bad16 = int(np.count_nonzero((ref != got16) & ~nan))
    nan16 = bool(np.all(((got16[nan] & 0x7C00) == 0x7C00) & ((got16[nan] & 0x03FF) != 0)))
    L.oracle_f32_to_bf16_array(x.ctypes.data, ref.ctypes.data, n)
    badb = int(np.count_nonzero((ref != gotb) & ~nan))
    nanb = bool(np.all(((gotb[nan] & 0x7F80) == 0x7F80) & ((gotb[nan] & 0x007F) != 0)))
    return bad16, badb, nan16, nanb


def test_all_fp32_patterns_round_like_the_oracle():
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream(dev).cuda_stream
    out16 = torch.empty(BATCH, dtype=torch.int16, device=dev)
    outb = torch.empty(BATCH, dtype=torch.int16, device=dev)
    bad16 = badb = 0
    ok = True
    with ThreadPoolExecutor(16) as pool:
        for b in range((1 << 32) // BATCH):
            bits = (torch.arange(BATCH, dtype=torch.int64, device=dev) + (b * BATCH - (1 << 31))).to(torch.int32)
            x = bits.view(torch.float32)
            ta.triaccel_cast_f32(x.data_ptr(), out16.data_ptr(), BATCH, ta.FP16, stream)
            ta.triaccel_cast_f32(x.data_ptr(), outb.data_ptr(), BATCH, ta.BF16, stream)
            torch.cuda.synchronize()
            xh = x.cpu().numpy()
            g16 = out16.cpu().numpy().view(np.uint16)
            gb = outb.cpu().numpy().view(np.uint16)
            parts = 16
            step = BATCH // parts
            res = list(pool.map(_oracle_slice, [(xh[i * step:(i + 1) * step], g16[i * step:(i + 1) * step],
                                                 gb[i * step:(i + 1) * step]) for i in range(parts)]))
            bad16 += sum(r[0] for r in res)
            badb += sum(r[1] for r in res)
            ok = ok and all(r[2] and r[3] for r in res)
            if b % 8 == 7:
                print(f"cast batch {b + 1}/64 done", flush=True)
    assert bad16 == 0 and badb == 0 and ok


def test_fp32_target_copies_and_ragged_length():
    dev = torch.device("cuda:0")
    x = torch.randn(1003, device=dev)
    y = torch.zeros(1004, device=dev)
    ta.triaccel_cast_f32(x.data_ptr(), y.data_ptr(), 1003, ta.FP32)
    torch.cuda.synchronize()
    assert torch.equal(y[:1003], x) and y[1003] == 0
    h = torch.zeros(1004, dtype=torch.float16, device=dev)
    ta.triaccel_cast_f32(x.data_ptr(), h.data_ptr(), 1003, ta.FP16)
    torch.cuda.synchronize()
    assert torch.equal(h[:1003], x.to(torch.float16)) and h[1003] == 0
