"""GPU tests of the C ABI's contract: argument errors change no state, pointers may change from
call to call, results are deterministic, several handles coexist, profiling returns stage times."""
import ctypes as C

import pytest
import torch

import paper_2508_16905_amd as ta
from paper_2508_16905_amd import binding as B
from workloads import get_workload

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def make(wl, seed_shift=0):
    params = [wl.init_param(l).to(DEV) for l in range(wl.n_tensors)]
    return ta.TriAccel(wl.hyper, params, grad_dtype=wl.grad_dtype)


def inputs(wl, t):
    g = [wl.grad(t, l).to(DEV) for l in range(wl.n_tensors)]
    pr = [wl.probe(t, l) for l in range(wl.n_tensors)]
    return g, [p[0].to(DEV) for p in pr], [p[1].to(DEV) for p in pr]


def snapshot(opt):
    torch.cuda.synchronize()
    return [(opt.buf[i].clone(), opt.curv[i].clone(), opt.mom[i].clone(), opt.mask[i].clone()) for i in range(opt.n)]


def equal(a, b):
    return all(torch.equal(x, y) for ta_, tb in zip(a, b) for x, y in zip(ta_, tb))


def test_argument_errors_are_reported_and_change_nothing():
    wl = get_workload("tiny_mlp")
    opt = make(wl)
    g, z, hz = inputs(wl, 1)
    opt.step(g, z, hz)
    opt.result()
    before = snapshot(opt)
    lib = ta.load_library()
    args = B.StepArgs(C.sizeof(B.StepArgs), 0.1, 1.0, 96, 8, 10)

    def call(mutate, n=None):
        arr = (B.Tensor * opt.n)()
        for i in range(opt.n):
            C.memmove(C.byref(arr[i]), C.byref(opt._tensors[i]), C.sizeof(B.Tensor))
        mutate(arr)
        return lib.triaccel_step(opt.handle, arr, opt.n if n is None else n, C.byref(args))

    assert call(lambda a: setattr(a[1], "grad", a[1].grad + 4)) == -5          # misaligned
    assert call(lambda a: setattr(a[0], "param", None)) == -4                  # NULL pointer
    assert call(lambda a: setattr(a[2], "hz", None)) == -4                     # z without hz
    assert call(lambda a: setattr(a[2], "numel", a[2].numel + 1)) == -3        # shape changed
    assert call(lambda a: setattr(a[3], "grad_dtype", 1)) == -3                # dtype changed
    assert call(lambda a: None, n=opt.n - 1) == -3                             # wrong count
    bad = B.StepArgs(C.sizeof(B.StepArgs), 0.1, 0.0, 96, 8, 10)                # loss scale must be > 0
    assert lib.triaccel_step(opt.handle, opt._tensors, opt.n, C.byref(bad)) == -1
    bad = B.StepArgs(4, 0.1, 1.0, 96, 8, 10)                                   # wrong struct_size
    assert lib.triaccel_step(opt.handle, opt._tensors, opt.n, C.byref(bad)) == -1
    res = opt.result()
    assert res.step_index == 1 and equal(before, snapshot(opt))
    # init-time errors
    cfg = B.Config.from_hyper(wl.hyper)
    cfg.beta_var = 1.0
    handle = C.c_void_p()
    assert lib.triaccel_init(C.byref(handle), C.byref(cfg), opt._tensors, opt.n, None) == -1 and not handle
    cfg = B.Config.from_hyper(wl.hyper)
    arr = (B.Tensor * opt.n)()
    for i in range(opt.n):
        C.memmove(C.byref(arr[i]), C.byref(opt._tensors[i]), C.sizeof(B.Tensor))
    arr[0].param_dtype = 7
    assert lib.triaccel_init(C.byref(handle), C.byref(cfg), arr, opt.n, None) == -2
    opt.close()


def test_result_before_any_step_and_profiling_calls():
    wl = get_workload("tiny_mlp")
    opt = make(wl)
    lib = ta.load_library()
    res = B.StepResult()
    res.struct_size = C.sizeof(B.StepResult)
    assert lib.triaccel_result(opt.handle, C.byref(res)) == -7
    g, z, hz = inputs(wl, 1)
    opt.step(g, z, hz)
    with pytest.raises(ta.TriAccelError):
        opt.stage_times()  # profiling was off
    opt.set_profiling(True)
    opt.step(g, z, hz)
    times = opt.stage_times()
    assert len(times) == len(ta.STAGE_NAMES) and all(t >= 0 for t in times) and sum(times) > 0
    assert times[0] > 0 and times[4] > 0
    opt.set_profiling(2)              # only the update kernel is bracketed
    opt.step(g, z, hz)
    times = opt.stage_times()
    assert times[4] > 0 and sum(times) == times[4]
    assert lib.triaccel_set_profiling(opt.handle, 3) == -1
    opt.close()


def test_two_runs_are_bit_identical_and_pointers_may_change():
    # determinism (no floating-point atomics, fixed merge orders) and fresh input buffers every step
    wl = get_workload("resnet18")
    a, b = make(wl), make(wl)
    for t in range(1, 5):
        ga, za, hza = inputs(wl, t)
        gb, zb, hzb = [x.clone() for x in ga], [x.clone() for x in za], [x.clone() for x in hza]
        a.step(ga, za, hza)
        b.step(gb, zb, hzb)
        ra, rb = a.result(), b.result()
        assert (ra.skipped, ra.next_loss_scale) == (rb.skipped, rb.next_loss_scale)
        sa, sb = a.layer_state(), b.layer_state()
        for x, y in zip(sa, sb):
            assert bytes(x) == bytes(y)
    assert equal(snapshot(a), snapshot(b))
    a.close()
    b.close()


@pytest.mark.parametrize("graph", [False, True], ids=["kernel_by_kernel", "graph_replay"])
def test_prepared_tables_of_resident_buffers_revisited_in_any_order(graph):
    """Eleven resident sets of input buffers, each marshalled once (make_table) and revisited in an
    irregular order with and without a probe: more distinct pointer tables than the library keeps
    device copies of, so tables are found again, evicted and uploaded again.  Every step is compared
    with the oracle, the steps are enqueued without a wait in between (the copies are ordered on the
    stream), and a second handle fed the same sequence through plain ``step`` ends bit-identical.
    With ``graph`` the first handle replays the step as a HIP graph (one captured step per device copy
    of the table and variant) on a stream of its own."""
    import sys, os
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    from _runner import make_oracle, to_numpy
    from _gpu_harness import bits_equal

    wl = get_workload("resnet18")
    R = 11
    b = make(wl)
    if graph:
        stream = torch.cuda.Stream(device=DEV)
        params = [wl.init_param(l).to(DEV) for l in range(wl.n_tensors)]
        with torch.cuda.stream(stream):
            a = ta.TriAccel(wl.hyper, params, grad_dtype=wl.grad_dtype, stream=stream)
        a.set_graph(True)
    else:
        a = make(wl)
    orc = make_oracle(wl, workers=16)
    sets = [inputs(wl, t) for t in range(1, R + 1)]
    torch.cuda.synchronize()  # the inputs were made on the default stream
    with_probe = [a.make_table(g, z, hz) for g, z, hz in sets]
    without = [a.make_table(g) for g, _, _ in sets]
    order = [0, 1, 0, 2, 3, 4, 5, 6, 7, 8, 9, 10, 0, 0, 5, 1, 10, 9, 2, 2, 7, 3, 0, 8]
    lr, scale = float(wl.hyper["lr"]), float(wl.hyper["loss_scale"])
    for step, j in enumerate(order):
        probe = step % 3 != 2
        a.step_table((with_probe if probe else without)[j], lr=lr, loss_scale=scale, batch_size=96,
                     mem_used_bytes=8, mem_total_bytes=10)
        g, z, hz = sets[j]
        b.step(g, z if probe else None, hz if probe else None, lr=lr, loss_scale=scale, batch_size=96,
               mem_used_bytes=8, mem_total_bytes=10)
        none = [None] * wl.n_tensors
        orc.step([to_numpy(x) for x in g], [to_numpy(x) for x in z] if probe else none,
                 [to_numpy(x) for x in hz] if probe else none, lr, scale, 96, 8, 10)
    assert a.result().step_index == len(order)
    assert equal(snapshot(a), snapshot(b))
    st = a.layer_state()
    for l, o in enumerate(orc.tensors):
        assert (st[l].code, st[l].nnz) == (o.code, o.nnz), l
        assert bits_equal(a.curv[l].cpu().numpy(), o.curv) and bits_equal(a.mask[l].cpu().numpy().view("uint32"), o.mask), l
        assert bits_equal(to_numpy(a.param(l, st[l].code)), o.param_view()), l
    a.close()
    b.close()


def test_step_on_a_side_stream():
    wl = get_workload("tiny_mlp")
    stream = torch.cuda.Stream(device=DEV)
    params = [wl.init_param(l).to(DEV) for l in range(wl.n_tensors)]
    ref = make(wl)
    with torch.cuda.stream(stream):
        opt = ta.TriAccel(wl.hyper, params, grad_dtype=wl.grad_dtype, stream=stream)
    for t in range(1, 4):
        g, z, hz = inputs(wl, t)
        torch.cuda.synchronize()
        opt.step(g, z, hz)
        ref.step(g, z, hz)
        opt.result()
        ref.result()
    assert equal(snapshot(opt), snapshot(ref))
    opt.close()
    ref.close()


def test_memory_numbers_from_the_runtime_when_not_supplied():
    wl = get_workload("tiny_mlp")
    opt = make(wl)
    g, z, hz = inputs(wl, 1)
    opt.step(g, z, hz, batch_size=96, mem_used_bytes=0, mem_total_bytes=0)
    res = opt.result()
    free, total = torch.cuda.mem_get_info()
    used = total - free
    want = 112 if used < 0.7 * total else (80 if used > 0.9 * total else 96)
    assert res.next_batch_size == want
    opt.close()


def test_state_round_trip_resumes_bit_identically():
    wl = get_workload("resnet18")
    n = wl.n_tensors
    a = make(wl)
    for t in range(1, 9):
        a.step(*inputs(wl, t))
    saved = snapshot(a)
    blob = a.get_state()
    assert len(blob) == ta.load_library().triaccel_state_size(a.handle)
    for t in range(9, 15):
        a.step(*inputs(wl, t))
    want = snapshot(a)
    want_layers = [(s.code, s.theta, s.v, s.eta, s.nnz) for s in a.layer_state()]
    # a new handle, the caller's tensors restored, the library state restored
    b = make(wl)
    for i in range(n):
        for dst, src in zip((b.buf[i], b.curv[i], b.mom[i], b.mask[i]), saved[i]):
            dst.copy_(src)
    b.set_state(blob)
    with pytest.raises(ta.TriAccelError):
        b.result()                                   # no step since the restore
    for t in range(9, 15):
        b.step(*inputs(wl, t))
    assert b.result().step_index == 14
    assert equal(want, snapshot(b))
    assert want_layers == [(s.code, s.theta, s.v, s.eta, s.nnz) for s in b.layer_state()]
    # blobs that do not belong to the handle are refused
    lib = ta.load_library()
    bad = bytearray(blob)
    bad[0] ^= 1
    assert lib.triaccel_set_state(b.handle, bytes(bad), len(bad)) == -1
    assert lib.triaccel_set_state(b.handle, blob, len(blob) - 8) == -3
    other = make(get_workload("tiny_mlp"))
    assert lib.triaccel_set_state(other.handle, blob, len(blob)) == -3
    c = ta.TriAccel(dict(wl.hyper, alpha=0.25), [wl.init_param(l).to(DEV) for l in range(n)], grad_dtype=wl.grad_dtype)
    assert lib.triaccel_set_state(c.handle, blob, len(blob)) == -1     # other hyper-parameters
    for o in (a, b, other, c):
        o.close()


def test_example_training_loop_reduces_the_loss():
    # the caller's side of the contract (autograd, loss scaling, Hessian-vector products, reading the
    # parameters back in the stored precision) around the library: the fit must improve markedly
    from paper_2508_16905_amd.examples.train_mlp import train

    losses = train(steps=150, verbose=False)
    first, last = sum(losses[:5]) / 5, sum(losses[-10:]) / 10
    assert last < 0.35 * first, (first, last)


def test_create_and_destroy_release_the_workspace():
    wl = get_workload("resnet18")
    params = [wl.init_param(l).to(DEV) for l in range(wl.n_tensors)]
    g, z, hz = inputs(wl, 1)

    def cycle(hyper):
        opt = ta.TriAccel(hyper, params, grad_dtype=wl.grad_dtype)
        opt.step(g, z, hz)
        opt.result()
        opt.close()

    cycle(wl.hyper)
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for i in range(40):
        cycle(dict(wl.hyper, power_k=5) if i % 2 else wl.hyper)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    # the wrapper's own tensors return to PyTorch's cache; the library's hipMalloc'ed workspace must come back
    assert free0 - free1 < 64 * 2**20, (free0, free1)
