"""The schedule of the in-place 2 <-> 4-byte rewrite of a tensor, replayed on the host on a byte map.

The kernels take the order of chunks, the grouping into launches and workgroups and the barrier
points from ``csrc/resize_schedule.h``; the same header is compiled here with g++ and its event
list is checked against the one rule that makes the rewrite correct: a store may only land on
bytes whose old contents have been loaded -- by an earlier launch, or by the same workgroup before
a barrier that precedes the store.  Loads by other workgroups of the same launch do not count
(no workgroup waits for another)."""
import ctypes as C
import os
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
E = 8  # elements per chunk in the replay: the schedule is in units of chunks


@pytest.fixture(scope="module")
def lib(tmp_path_factory):
    so = tmp_path_factory.mktemp("resize") / "libresize_replay.so"
    subprocess.run(["g++", "-std=c++17", "-O1", "-fPIC", "-shared", "-fsanitize=undefined", "-fno-sanitize-recover=all",
                    "-o", str(so), os.path.join(ROOT, "tests", "resize_replay.cpp")], check=True)
    L = C.CDLL(str(so))
    L.resize_replay.restype = C.c_int64
    L.resize_replay.argtypes = [C.c_uint32, C.c_uint32, C.c_uint32, C.c_int, C.c_void_p, C.c_int64]
    L.resize_plan.argtypes = [C.c_uint32, C.c_uint32, C.c_void_p]
    return L


def events(lib, max_chunks, total_chunks, n_chunks, narrowing):
    cap = 4 * n_chunks + 64
    buf = np.zeros((cap, 5), np.int32)
    n = lib.resize_replay(max_chunks, total_chunks, n_chunks, int(narrowing), buf.ctypes.data, cap)
    assert n <= cap
    return buf[:n]


def replay(ev, n_chunks, numel, narrowing):
    """Checks the event list on a byte map; returns the number of launches used."""
    s_old, s_new = (4, 2) if narrowing else (2, 4)
    old_bytes = s_old * numel
    never = np.iinfo(np.int32).max
    load_launch = np.full(4 * numel, never, np.int32)   # per byte: when its old contents were loaded
    load_wg = np.full(4 * numel, -1, np.int32)
    load_epoch = np.full(4 * numel, -1, np.int32)
    loaded = np.zeros(n_chunks, bool)
    stored = np.zeros(n_chunks, bool)
    epoch = {}                                           # (launch, wg) -> barriers passed
    last_launch = -1
    for launch, wg, kind, c, stage in ev:
        assert launch >= last_launch                     # launches are listed in order
        last_launch = launch
        key = (int(launch), int(wg))
        e = epoch.get(key, 0)
        if kind == 1:
            epoch[key] = e + 1
            continue
        lo, hi = c * E, min((c + 1) * E, numel)
        assert 0 <= c < n_chunks and lo < hi
        if kind == 0:
            assert not loaded[c] and not stored[c], ("chunk loaded twice or after its store", c)
            loaded[c] = True
            b0, b1 = s_old * lo, s_old * hi
            load_launch[b0:b1], load_wg[b0:b1], load_epoch[b0:b1] = launch, wg, e
        else:
            assert loaded[c] and not stored[c], c
            stored[c] = True
            b0, b1 = s_new * lo, min(s_new * hi, old_bytes)   # bytes beyond the old data hold nothing
            if b0 < b1:
                ok = (load_launch[b0:b1] < launch) | ((load_launch[b0:b1] == launch) & (load_wg[b0:b1] == wg)
                                                      & (load_epoch[b0:b1] < e))
                assert ok.all(), ("store onto bytes not yet loaded", dict(chunk=int(c), launch=int(launch), wg=int(wg),
                                                                          stage=int(stage), narrowing=narrowing))
    assert loaded.all() and stored.all()
    return last_launch + 1


SIZES = [1, 2, 3, 4, 15, 16, 17, 31, 32, 33, 63, 64, 65, 100, 127, 128, 129, 130, 255, 256, 257, 511, 513, 576, 1000,
         1023, 1024, 1025, 2047, 2049, 4095, 4096, 4097, 4099, 5000, 8191, 8193, 33000, 70001]


@pytest.mark.parametrize("narrowing", [True, False])
def test_no_store_lands_on_bytes_not_yet_loaded(lib, narrowing):
    rs = np.random.default_rng(5)
    for n_chunks in SIZES:
        for total in (n_chunks, 1 << 20):                # a small set (deep subtrees) and a large one (shallow)
            for tail in sorted({1, int(rs.integers(1, E + 1)), E}):
                numel = (n_chunks - 1) * E + tail
                ev = events(lib, n_chunks, total, n_chunks, narrowing)
                replay(ev, n_chunks, numel, narrowing)


@pytest.mark.parametrize("narrowing", [True, False])
def test_smaller_tensors_follow_the_plan_of_the_largest(lib, narrowing):
    rs = np.random.default_rng(6)
    for max_chunks in (129, 576, 4099, 70001):
        for n_chunks in sorted({1, 2, 16, 17, 128, 129, max_chunks // 2 + 1, max_chunks - 1} | set(rs.integers(1, max_chunks, 6).tolist())):
            n_chunks = int(n_chunks)
            for total in (max_chunks, 1 << 20):
                numel = (n_chunks - 1) * E + int(rs.integers(1, E + 1))
                replay(events(lib, max_chunks, total, n_chunks, narrowing), n_chunks, numel, narrowing)


def test_the_check_itself_rejects_a_wrong_order(lib):
    # widening in the narrowing order must be caught: the replay is not vacuous
    ev = events(lib, 300, 300, 300, True)
    with pytest.raises(AssertionError):
        replay(ev, 300, 300 * E, False)
    ev = events(lib, 300, 300, 300, False)
    with pytest.raises(AssertionError):
        replay(ev, 300, 300 * E, True)
    # a barrier taken out of a subtree walk must be caught as well
    ev = events(lib, 5000, 1 << 20, 5000, True)
    stage1 = np.nonzero((ev[:, 2] == 1) & (ev[:, 4] >= 1))[0]
    broken = np.delete(ev, stage1[:1], axis=0)
    with pytest.raises(AssertionError):
        replay(broken, 5000, 5000 * E, True)


def test_number_of_launches(lib):
    def plan(max_chunks, total):
        out = np.zeros(18, np.uint32)
        lib.resize_plan(max_chunks, total, out.ctypes.data)
        return int(out[0]), int(out[1]), out[2:10].tolist(), out[10:18].tolist()

    assert plan(25, 25)[0] == 1 and plan(100, 982)[0] == 1 and plan(128, 128)[0] == 1    # stage 0 alone
    assert plan(576, 2800)[0] == 2                       # ResNet-18-shaped set: one subtree stage
    n, top, root, depth = plan(4096, 262144)             # 64 x 4096 x 4096: 16 -> 256 -> 4096
    assert (n, top, root[1:3], depth[1:3]) == (3, 16, [16, 256], [4, 4])
    n, top, root, depth = plan(524287, 524287)           # the largest tensor the library accepts
    assert n <= 8 and (root[n - 1] << depth[n - 1]) >= 524287
