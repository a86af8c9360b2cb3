#!/usr/bin/env python3
"""Benchmark of the fused Tri-Accel optimizer step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--all-fp32] [--no-variants]

One "step" is one pass of the whole hot path (gradient statistics, curvature EMA, threshold and
mask, per-layer assignment, update + cast) over every tensor of the workload, with inputs already
resident in HBM.  Prints ONE JSON line: whole-step throughput in params/s, the HBM roofline of the
dominant kernel (update + cast) from HIP-event timings taken inside the timed region, per-stage
figures, the same set measured in its other regimes (`variants`: every layer FP32, steps without a
probe, a probe every 200th step, the first steps of a run, every layer changing its storage size at
every step, the mixed-state set), and the CPU oracle timed on bounded samples as a baseline.

Two byte counts are reported for a step.  `moved`: what the kernels of that step have to move given
what they did (a threshold settled by its predicted band costs no second pass over the curvature).
`credited`: the method's traffic with the re-read of |h| that an exact order statistic needs in
general (4.125 B/param on probed steps) counted whether or not the prediction let the kernels skip
it.  Fractions of the HBM peak are given for both; `step.frac_of_peak` is the moved one.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak

# HBM bytes one launch of the dominant kernel moved on the default workload, from two
# `rocprofv3 --pmc` runs (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch, scaled by what the same
# counters read for the library's plain copy kernel; see the summaries under profiles/).  They belong
# to the kernel sources with the digest below: when the sources differ, `traffic` is null.
STEP_SOURCES = ("update.hip", "update_body.h", "resize_body.h", "resize_schedule.h", "device_util.h", "numerics.h")
POWER_SOURCES = ("power.hip", "power.h", "numerics.h")
MEASURED_TRAFFIC = {
    # k_update<false>, default run of the large_streaming workload
    "step": {"sources_sha256": "16a0fc49e758ec5b6e4b2ab216d26cd137125df31f6cbaf06a31275dd758259e", "workload": "large_streaming",
             "alg_bytes": 18991808512, "fetch_bytes": 11.677e9, "write_bytes": 7.348e9,
             "from": "profiles/fused_step_large_streaming_hbm_counters.md"},
    # k_power_apply<5> / k_power_gram<5>, --mode power on the large_streaming workload
    "power": {"sources_sha256": "1bf257dfb3af1e77ee28322071abf703d828084ae8edeb4fa6b9f98da079a634", "workload": "large_streaming",
              "k_power_apply": {"fetch_bytes": 21.51e9, "write_bytes": 21.47e9},
              "k_power_gram": {"fetch_bytes": 42.95e9, "write_bytes": 0.01e9},
              "from": "profiles/power_iteration_large_streaming_k5.md"},
}


def sources_digest(files):
    import hashlib
    h = hashlib.sha256()
    for f in files:
        with open(os.path.join(ROOT, "paper_2508_16905_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def measured_traffic(workload, plain_run, alg_bytes):
    """Counter-measured HBM bytes per launch of k_update (taken in a separate rocprofv3 run, not in this
    one), or None if they do not apply: another workload or variant, launches that do other work than
    those of the counter run (e.g. mask passes of tensors that fell back), or changed kernel sources."""
    m = MEASURED_TRAFFIC["step"]
    if workload != m["workload"] or not plain_run or int(alg_bytes) != m["alg_bytes"]:
        return None
    if sources_digest(STEP_SOURCES) != m["sources_sha256"]:
        return None
    return m["fetch_bytes"] + m["write_bytes"]


def measured_power_traffic(workload, k, kernel, n_tensors_limit):
    m = MEASURED_TRAFFIC["power"]
    if workload != m["workload"] or k != 5 or n_tensors_limit or sources_digest(POWER_SOURCES) != m["sources_sha256"]:
        return None
    return m[kernel]["fetch_bytes"] + m[kernel]["write_bytes"]


def step_bytes(numel, grad_size, prev_codes, codes, sel_passes, probed, momentum, fisher=False, elem=False):
    """Bytes of one step per kernel stage, from the definitions of the stages: statistics read g; the EMA
    reads z, Hz, h and writes h; the mask is one bit per element; the update reads g, the stored parameter
    and m, and writes the parameter and m.  Returns (moved, credited): `moved` charges every pass over h
    that the threshold selection of this step made (`sel_passes` per tensor, 0 when the predicted band
    settled it), `credited` charges exactly one re-read of |h| per probed tensor, made or not."""
    size = lambda c: 4 if c == 2 else 2
    moved = dict(grad_stats=0.0, curv_ema=0.0, select_refine=0.0, update=0.0, update_resize=0.0)
    reread_credit = 0.0
    for n, pc, c, extra in zip(numel, prev_codes, codes, sel_passes):
        moved["grad_stats"] += n * grad_size
        if probed:
            # Hutchinson source: z, Hz, h read, h written; Fisher source: g, h read, h written
            moved["curv_ema"] += n * ((grad_size + 8) if fisher else 16)
            if extra:
                # histogram passes read h; the last extra pass is the mask pass, which rides in the update kernel
                moved["select_refine"] += n * 4.0 * (extra - 1)
                moved["update"] += n * 4.0 + n / 8.0
            else:
                moved["curv_ema"] += n / 8.0
            reread_credit += n * 4.0 + n / 8.0
        # the element-wise form of the step size reads h once more in the update
        upd = n * (grad_size + size(pc) + size(c) + (8 if momentum else 0) + (4 if elem else 0))
        moved["update" if size(pc) == size(c) else "update_resize"] += upd
    base = sum(n * grad_size for n in numel)
    if probed:
        base += sum(n * ((grad_size + 8) if fisher else 16) for n in numel)
    base += sum(n * (grad_size + size(pc) + size(c) + (8 if momentum else 0) + (4 if elem else 0))
                for n, pc, c in zip(numel, prev_codes, codes))
    return moved, base + reread_credit


def build_sets(wl, R, scale, dev, fisher=False, mult=None):
    """R input batches resident on the GPU: (gradients, z, Hz) per batch.  Generator steps with injected
    inf/NaN are left out (a skipped step does no work and would flatter the average)."""
    L = wl.n_tensors
    gen_steps = [t for t in range(1, 4 * R + 2) if not (wl.inject_every and t % wl.inject_every == 0)][:R]
    sets = []
    for j, t in enumerate(gen_steps):
        grads = [wl.grad(t, l, scale, device=dev) for l in range(L)]
        if mult is not None:
            for gten in grads:
                gten.mul_(mult[j % len(mult)])
        if fisher:
            sets.append((grads, None, None))
            continue
        pr = [wl.probe(t, l, scale, device=dev) for l in range(L)]
        sets.append((grads, [p[0] for p in pr], [p[1] for p in pr]))
    return sets


class Runner:
    """One optimizer instance driven over cycled input batches."""

    def __init__(self, wl, hyper, sets, dev, graph=False, own_stream=False):
        import torch

        import paper_2508_16905_amd as ta

        self.ta, self.torch, self.wl, self.hyper, self.sets, self.dev = ta, torch, wl, hyper, sets, dev
        L = wl.n_tensors
        stream = torch.cuda.Stream(device=dev) if (graph or own_stream) else None
        self.opt = ta.TriAccel(hyper, [wl.init_param(l, device=dev) for l in range(L)], grad_dtype=wl.grad_dtype,
                               stream=stream)
        if graph:
            self.opt.set_graph(True)
        self.graph = graph
        self.i = 0
        self.probes = 0
        self.tables = {}
        self.scale = float(hyper["loss_scale"])
        self.lr = float(hyper["lr"])
        self.numel = [wl.numel(l) for l in range(L)]
        self.grad_size = 4 if wl.grad_dtype == 2 else 2
        self.fisher = hyper.get("curvature_source", 0) == 1
        self.elem = hyper.get("elementwise_scale", 0) == 1

    def one(self, probe=True):
        # gradients cycle with the steps, probe pairs with the probed steps: a probe after a stretch of
        # steps without one continues the sequence of samples where the last probe left it.  The tensor
        # table of every combination is marshalled once (the buffers are resident and never move).
        gi = self.i % len(self.sets)
        self.i += 1
        pi = None
        if probe:
            pi = self.probes % len(self.sets)
            self.probes += 1
        if self.fisher:
            pi = None   # the curvature sample is the gradient itself: no probe pairs in this mode
        table = self.tables.get((gi, pi))
        if table is None:
            z = hz = None
            if pi is not None:
                _, z, hz = self.sets[pi]
            table = self.tables[(gi, pi)] = self.opt.make_table(self.sets[gi][0], z, hz)
        self.opt.step_table(table, lr=self.lr, loss_scale=self.scale, batch_size=int(self.hyper["batch_size"]),
                            mem_used_bytes=8, mem_total_bytes=10, update_curvature=probe)

    def run(self, n, probe=True):
        for _ in range(n):
            self.one(probe)

    def timed(self, n, probe=True):
        """n steps bracketed by device synchronisation; returns ms per step."""
        self.torch.cuda.synchronize()
        t0 = time.perf_counter()
        self.run(n, probe)
        self.torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n

    def bytes_of_last_step(self, probed):
        state = self.opt.layer_state()
        moved, credited = step_bytes(self.numel, self.grad_size, [s.prev_code for s in state], [s.code for s in state],
                                     [s.sel_passes if probed else 0 for s in state], probed,
                                     self.hyper["momentum"] != 0.0, fisher=self.fisher, elem=self.elem)
        return state, moved, credited

    def figures(self, ms, probed):
        """Throughput and both bandwidth figures of a step that took `ms`, with the bytes of the last step."""
        N = sum(self.numel)
        state, moved, credited = self.bytes_of_last_step(probed)
        mv = sum(moved.values())
        return {
            "ms_per_step": ms,
            "params_per_s": N / (ms / 1e3),
            "moved_bytes_per_param": mv / N,
            "GBps": mv / 1e9 / (ms / 1e3),
            "frac_of_peak": mv / 1e9 / (ms / 1e3) / HBM_PEAK_GBPS,
            "credited_bytes_per_param": credited / N,
            "credited_frac_of_peak": credited / 1e9 / (ms / 1e3) / HBM_PEAK_GBPS,
            "codes": {"fp16": sum(s.code == 0 for s in state), "bf16": sum(s.code == 1 for s in state),
                      "fp32": sum(s.code == 2 for s in state)},
            "tensors_needing_extra_passes_over_h_last_step": sum(1 for s in state if probed and s.sel_passes),
        }

    def close(self):
        self.opt.close()
        self.tables.clear()
        self.opt._keep = None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--workload", default="large_streaming")
    ap.add_argument("--all-fp32", action="store_true", help="thresholds that keep every layer in FP32")
    ap.add_argument("--fisher", action="store_true",
                    help="curvature sample = squared gradient (no probe pairs) instead of the Hutchinson pair")
    ap.add_argument("--elementwise", action="store_true",
                    help="step size scaled per element by the masked |h_i| instead of per layer")
    ap.add_argument("--graph", action="store_true",
                    help="replay the step as a HIP graph in the timed region (stage times then come from "
                         "the same number of steps launched kernel by kernel afterwards)")
    ap.add_argument("--own-stream", action="store_true", help="run the steps on a stream of their own, not the default one")
    ap.add_argument("--switch-stress", action="store_true",
                    help="variance EMA off and a gradient scale cycling over three decades: every layer changes "
                         "its storage precision at every step (all updates go through the in-place resize)")
    ap.add_argument("--no-probe", action="store_true",
                    help="timed steps carry no curvature probe (the ordinary step between two curvature refreshes, "
                         "Sec. 4.1: T = 200); settle and warm-up steps still probe")
    ap.add_argument("--settle", type=int, default=64,
                    help="the optimizer state is first brought to at least this many steps into the run (untimed, "
                         "before the warm-up steps): the exact threshold needs no second pass over the curvature "
                         "once its prediction has converged, about 40 steps in; 0 measures the first steps of a run")
    ap.add_argument("--input-sets", type=int, default=8, help="distinct pre-generated input batches (cycled)")
    ap.add_argument("--cpu-sample-tensors", type=int, default=8)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-variants", action="store_true",
                    help="only the headline measurement (profiler runs); by default the large_streaming run also "
                         "measures the set in its other regimes, a few steps each, into `variants`")
    ap.add_argument("--tensors", type=int, default=0, help="use only the first N tensors of the workload (tuning runs)")
    ap.add_argument("--mode", choices=["step", "power", "placements"], default="step",
                    help="step: the fused optimizer step (default, the headline); power: one power iteration; "
                         "placements: the update kernel's time over several placements of the optimizer state in "
                         "memory (the state is released to the driver and allocated anew behind a junk allocation "
                         "of random size, inside this one process; steps without a probe)")
    ap.add_argument("--placements", type=int, default=12, help="--mode placements: how many placements to time")
    ap.add_argument("--power-k", type=int, default=5, help="vectors per layer in --mode power (the paper's top-k = 5)")
    ap.add_argument("--power-stage-times", action="store_true",
                    help="--mode power: read the kernel times after every call (synchronises each call)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run the library's plain fp32 copy kernel on 1 GiB (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(a sharded job would run one such step per rank on its own tensors)", file=sys.stderr)
        sys.exit(2)
    if args.steps < 1 or args.warmup < 0:
        print("bench.py: --steps must be at least 1 and --warmup at least 0", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2508_16905_amd as ta
    from workloads import get_workload

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = get_workload(args.workload)
    if args.tensors:
        wl.tensors = wl.tensors[: args.tensors]
    hyper = dict(wl.hyper)
    if args.all_fp32:
        hyper.update(tau_low=0.0, tau_high=0.0)
    if args.fisher:
        hyper.update(curvature_source=1)
    if args.elementwise:
        hyper.update(elementwise_scale=1)
    if args.switch_stress:
        hyper.update(beta_var=0.0, tau_curv=1e30)
        args.input_sets = 6  # a multiple of the three-step cycle of the gradient scale
    K, W = args.steps, args.warmup
    if args.mode == "power":
        return bench_power(args, wl, hyper, dev)
    if args.mode == "placements":
        return bench_placements(args, wl, hyper, dev)
    L, N = wl.n_tensors, wl.total_params
    scale = float(hyper["loss_scale"])
    R = max(1, min(args.input_sets, K + max(W, args.settle)))
    # unscaled standard deviation 0.0316 x {0.3, 3, 30}: variance below tau_low, between, above tau_high
    sets = build_sets(wl, R, scale, dev, fisher=args.fisher, mult=SWITCH_MULT if args.switch_stress else None)
    torch.cuda.synchronize()
    print(f"[bench] {wl.name}: {L} tensors, {N} params, {R} input sets resident, "
          f"{torch.cuda.memory_allocated() / 2**30:.1f} GiB allocated", file=sys.stderr, flush=True)

    if args.calibrate_copy:
        # 2^28 floats: reads 1 GiB, writes 1 GiB, five launches
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            ta.triaccel_cast_f32(src.data_ptr(), dst.data_ptr(), src.numel(), ta.FP32,
                                 torch.cuda.current_stream(dev).cuda_stream)
        torch.cuda.synchronize()
        del src, dst

    run = Runner(wl, hyper, sets, dev, graph=args.graph, own_stream=args.own_stream)
    opt = run.opt
    # In the timed region only the dominant kernel (update + cast) is bracketed by HIP events: every
    # recorded event costs the stream a few microseconds.  A graph replay carries no events at all.
    # On the small sets (a step of ~0.1 ms) the two events would be a tenth of what is measured: their
    # timed region carries none, and the kernel time comes from the breakdown steps afterwards.
    events_in_timed_region = not args.graph and N >= 67_000_000
    if events_in_timed_region:
        opt.set_profiling(1 if args.switch_stress else 2)

    # bring the run to its steady state first when the warm-up alone is shorter than that takes
    P = max(0, args.settle - W)
    run.run(P + W)
    if P + W > 0:
        res = opt.result()
        assert not res.skipped
    codes_before = [s.code for s in opt.layer_state()]
    probed = not args.no_probe
    ms_per_step = run.timed(K, probed)
    res = opt.result()
    assert not res.skipped and res.step_index == P + W + K
    KP = min(K, 63)  # the library keeps the event times of the last 64 steps
    upd_ms_timed = sum(opt.stage_times(back)[4] for back in range(KP)) / KP if events_in_timed_region else None
    resize_ms_timed = sum(opt.stage_times(back)[5] for back in range(KP)) / KP if args.switch_stress and events_in_timed_region else None
    timed_stage_ms = [opt.stage_times(back) for back in range(KP)] if resize_ms_timed is not None else []
    # stage breakdown: the same number of steps again, launched kernel by kernel with an event at
    # every stage boundary (not part of the timed region)
    opt.set_profiling(1)
    run.run(KP, probed)
    opt.result()
    stage_ms = [opt.stage_times(back) for back in range(KP)]
    mean_ms = {name: sum(s[i] for s in stage_ms) / KP for i, name in enumerate(ta.STAGE_NAMES)}

    # traffic of the last step (codes are stationary over the timed region unless a layer switched;
    # the count of switches is reported)
    fig = run.figures(ms_per_step, probed)
    state, moved, credited = run.bytes_of_last_step(probed)
    codes = [s.code for s in state]
    switched = sum(1 for a, b in zip(codes_before, codes) if a != b)
    stages = {}
    for name in ta.STAGE_NAMES:
        entry = {"ms": round(mean_ms[name], 4)}
        if moved.get(name):
            entry["GB"] = round(moved[name] / 1e9, 4)
            entry["GBps"] = round(moved[name] / 1e9 / (mean_ms[name] / 1e3), 1) if mean_ms[name] > 0 else None
        stages[name] = entry
    upd_ms = mean_ms["update"] if upd_ms_timed is None else upd_ms_timed
    upd_gbps = moved["update"] / 1e9 / (upd_ms / 1e3)
    dominant, dominant_bytes = "k_update (fused update + cast)", moved["update"]
    grad_size = run.grad_size
    if args.switch_stress:
        # every step of the cycle sends all tensors through the update, in place at the same or at another
        # element size (2 -> 2, 2 -> 4, 4 -> 2 bytes per stored parameter); the first launch of the in-place
        # resize is part of the update kernel's launch, so both stages are reported as one figure
        dominant = "k_update + k_update_resize (update of every tensor, two of three steps in place at another element size)"
        both = lambda t: t[4] + t[5]
        upd_ms = (mean_ms["update"] + mean_ms["update_resize"] if resize_ms_timed is None
                  else sum(both(opt_times) for opt_times in timed_stage_ms) / len(timed_stage_ms))
        dominant_bytes = N * (grad_size + (8 if hyper["momentum"] != 0.0 else 0)) + N * (4 + 6 + 6) / 3.0
        upd_gbps = dominant_bytes / 1e9 / (upd_ms / 1e3)
    plain_run = not (args.all_fp32 or args.tensors or args.fisher or args.elementwise or args.switch_stress)
    traffic = measured_traffic(wl.name, plain_run, dominant_bytes)

    out = {
        "metric": "fused Tri-Accel step params/sec and achieved HBM GB/s (% of peak), 1 GPU",
        "value": N / (ms_per_step / 1e3),
        "unit": "params/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{wl.name}: {L} tensors, {N} params, fp{8 * grad_size} gradients, "
                        f"{'probe every step' if probed else 'no probe in the timed steps'}, "
                        f"momentum {hyper['momentum']}, sparsity {hyper['sparsity_ppm'] / 1e4:.0f}%",
            "all_fp32": bool(args.all_fp32),
            "step_size": "per element" if args.elementwise else "per layer",
            "curvature_source": "empirical Fisher (squared gradient)" if args.fisher else "Hutchinson pair (z, Hz)",
            "codes": fig["codes"],
            "layers_switched_in_timed_region": switched,
            "tensors_needing_extra_passes_over_h_last_step": fig["tensors_needing_extra_passes_over_h_last_step"],
            "input_sets": R,
            "settle_steps_before_warmup": P,
            "launch": "HIP graph replay" if args.graph else "kernel by kernel",
            "switch_stress": bool(args.switch_stress),
        },
        "roofline": {
            "bound": "hbm",
            "kernel": dominant,
            "kernel_ms": upd_ms,
            "kernel_ms_from": "HIP events in the steps after the timed region (the timed region of a graph replay or of a "
                              "small set carries none)"
                              if upd_ms_timed is None else "HIP events around the kernel in the timed region",
            "achieved": upd_gbps,
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": upd_gbps / HBM_PEAK_GBPS,
            "alg_bytes_per_launch": dominant_bytes,
            "traffic": traffic,
            "traffic_from": None if traffic is None else
                            "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, summarised in "
                            + MEASURED_TRAFFIC["step"]["from"] + " (not counters of this run)",
        },
        "step": {
            # bytes the kernels of the step had to move, and the same with the re-read of |h| credited
            "moved_bytes_per_param": fig["moved_bytes_per_param"],
            "moved_GB": fig["moved_bytes_per_param"] * N / 1e9,
            "GBps": fig["GBps"],
            "frac_of_peak": fig["frac_of_peak"],
            "credited_bytes_per_param": fig["credited_bytes_per_param"],
            "credited_GB": credited / 1e9,
            "credited_GBps": credited / 1e9 / (ms_per_step / 1e3),
            "credited_frac_of_peak": fig["credited_frac_of_peak"],
            # HIP-event time from the first to the last kernel of a step, median over the steps of
            # the stage breakdown (an event at every stage boundary costs the stream a few microseconds)
            "ms_events_median": sorted(sum(s) for s in stage_ms)[KP // 2],
        },
        "stages": stages,
    }

    want_variants = (not args.no_variants and plain_run and wl.name == "large_streaming" and not args.graph
                     and not args.no_probe and len(sets) >= 6)
    if want_variants:
        out["variants"] = variants(run, wl, hyper, sets, dev, min(K, 10))
    else:
        run.close()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, hyper, args.cpu_sample_tensors, scale)
        if want_variants:
            out["cpu_baseline"]["per_config"] = cpu_per_config()
    print(json.dumps(out))


SWITCH_MULT = (0.3, 3.0, 30.0)


def variants(run, wl, hyper, sets, dev, K):
    """The same parameter set in its other regimes, K timed steps each (same process, same resident
    inputs); the mixed-state set last, on inputs of its own.  `run` is the headline's runner in steady
    state; it is closed here."""
    import torch

    from workloads import get_workload

    N = wl.total_params
    v = {}
    # (1) the ordinary step between two curvature refreshes
    run.opt.set_profiling(2)
    run.run(3, probe=False)
    ms = run.timed(K, probe=False)
    v["no_probe"] = run.figures(ms, probed=False)
    v["no_probe"]["k_update_ms"] = sum(run.opt.stage_times(b)[4] for b in range(K)) / K

    # (2) the paper's refresh schedule (Sec. 4.1: T = 200): two periods, a probe on the first step of each
    outcomes = {}
    extra = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for period in range(2):
        run.one(probe=True)
        for s in run.opt.layer_state():       # synchronises: two of the 400 steps pay for it
            outcomes[int(s.sel_outcome)] = outcomes.get(int(s.sel_outcome), 0) + 1
            extra += int(s.sel_passes)
        run.run(199, probe=False)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / 400
    v["probe_every_200"] = {
        "ms_per_step": ms, "params_per_s": N / (ms / 1e3), "steps": 400, "probe_steps": 2,
        "band_check_outcomes_over_probe_steps_x_tensors": {str(k): n for k, n in sorted(outcomes.items())},
        "extra_passes_over_h": extra,
        "note": "outcome 1 = the predicted band settled the threshold in the EMA pass; the predictor only sees "
                "probed steps, so its state after P probes is the same whatever the spacing of the probes",
    }
    run.close()

    # (3) every layer stored in FP32: the 44.125 B/param case (the worked example prints 40.125)
    r = Runner(wl, dict(hyper, tau_low=0.0, tau_high=0.0), sets, dev)
    r.opt.set_profiling(2)
    r.run(64)
    ms = r.timed(K)
    f = r.figures(ms, True)
    f["k_update_ms"] = sum(r.opt.stage_times(b)[4] for b in range(K)) / K
    f["frac_of_peak_at_40.125_bytes_per_param"] = 40.125 * N / 1e9 / (ms / 1e3) / HBM_PEAK_GBPS
    v["all_fp32"] = f
    r.close()

    # (3b) the other curvature source and the other form of the step size (same inputs)
    for name, extra in (("fisher", dict(curvature_source=1)), ("elementwise", dict(elementwise_scale=1))):
        r = Runner(wl, dict(hyper, **extra), sets, dev)
        r.opt.set_profiling(2)
        r.run(64)
        ms = r.timed(K)
        v[name] = r.figures(ms, True)
        v[name]["k_update_ms"] = sum(r.opt.stage_times(b)[4] for b in range(K)) / K
        r.close()

    # (4) the first steps of a run: no threshold prediction yet, every tensor goes through the fallback
    r = Runner(wl, hyper, sets, dev)
    first = []
    for t in range(1, 7):
        ms = r.timed(1)
        st = r.opt.layer_state()
        first.append({"step": t, "ms": ms, "tensors_with_extra_passes": sum(1 for s in st if s.sel_passes),
                      "extra_passes_over_h": sum(int(s.sel_passes) for s in st)})
    v["first_steps"] = first
    r.close()

    # (5) every layer changes its storage size at (two of three) steps: the in-place resize
    for j, (grads, _, _) in enumerate(sets[:6]):
        for g in grads:
            g.mul_(SWITCH_MULT[j % 3])
    r = Runner(wl, dict(hyper, beta_var=0.0, tau_curv=1e30), sets[:6], dev)
    r.opt.set_profiling(1)
    r.run(60)
    K3 = max(3, (K // 3) * 3)
    ms = r.timed(K3)
    resize_ms = sum(r.opt.stage_times(b)[5] for b in range(K3)) / K3
    update_ms = sum(r.opt.stage_times(b)[4] for b in range(K3)) / K3
    gs = r.grad_size
    mom = 8 if hyper["momentum"] != 0.0 else 0
    # bytes of all updates of an average step of the cycle (2 -> 2, 2 -> 4 and 4 -> 2 bytes per stored parameter);
    # the first launch of the in-place resize is part of the update kernel's launch, so the two stages are one figure
    upd_bytes = N * (gs + mom) + N * (4 + 6 + 6) / 3.0
    avg_bytes = N * (gs + 16.125) + upd_bytes
    v["switch_stress"] = {
        "ms_per_step": ms, "params_per_s": N / (ms / 1e3),
        "moved_bytes_per_param": avg_bytes / N, "GBps": avg_bytes / 1e9 / (ms / 1e3),
        "frac_of_peak": avg_bytes / 1e9 / (ms / 1e3) / HBM_PEAK_GBPS,
        "update_and_resize_ms_avg": update_ms + resize_ms, "of_which_later_resize_launches_ms": resize_ms,
        "update_and_resize_GBps": upd_bytes / 1e9 / ((update_ms + resize_ms) / 1e3),
        "update_and_resize_frac_of_peak": upd_bytes / 1e9 / ((update_ms + resize_ms) / 1e3) / HBM_PEAK_GBPS,
        "note": "two of three steps rewrite every tensor in place at another element size; an event at every stage "
                "boundary in the timed steps",
    }
    r.close()
    del r
    sets.clear()
    torch.cuda.empty_cache()

    # (5b) one power iteration on k = 5 vectors per tensor (Sec. 3.2; 43 GB of vectors)
    v["power_iteration_k5"] = power_variant(wl, hyper, dev, 5, max(3, K // 2))

    # (6) the mixed-state set: fp16 gradients, three storage formats
    wm = get_workload("mixed_state")
    hm = dict(wm.hyper)
    sm = build_sets(wm, 8, float(hm["loss_scale"]), dev)
    r = Runner(wm, hm, sm, dev)
    r.opt.set_profiling(2)
    r.run(64)
    ms = r.timed(max(K, 20))
    v["mixed_state"] = r.figures(ms, True)
    v["mixed_state"]["workload"] = f"{wm.n_tensors} tensors, {wm.total_params} params, fp16 gradients"
    r.close()
    return v


PLACEMENT_WARM, PLACEMENT_TIMED = 4, 12


def bench_placements(args, wl, hyper, dev):
    """The update kernel has a faster and a slower regime, and which one a run gets depends on where the
    arrays it streams lie in memory: same process, same kernel, same inputs, only the optimizer state
    allocated anew.  Each placement launches the kernel PLACEMENT_WARM + PLACEMENT_TIMED times (steps
    without a probe: statistics, per-layer kernel, update), so the dispatches of a profiler's counter file
    can be grouped by placement."""
    import random

    import torch

    N = wl.total_params
    sets = build_sets(wl, 4, float(hyper["loss_scale"]), dev, fisher=True)   # gradients only
    rs = random.Random(os.getpid())
    junk, rows = None, []
    for k in range(args.placements):
        run = Runner(wl, hyper, sets, dev)
        run.opt.set_profiling(2)
        run.run(PLACEMENT_WARM, probe=False)
        run.run(PLACEMENT_TIMED, probe=False)
        run.opt.result()
        ms = sorted(run.opt.stage_times(b)[4] for b in range(PLACEMENT_TIMED))
        state = run.opt.layer_state()
        size = lambda c: 4 if c == 2 else 2
        nbytes = sum(n * (run.grad_size + size(s.prev_code) + size(s.code) + 8) for n, s in zip(run.numel, state))
        rows.append({"placement": k, "k_update_ms_median": ms[len(ms) // 2], "GBps": nbytes / 1e9 / (ms[len(ms) // 2] / 1e3),
                     "junk_bytes_before": 0 if junk is None else junk.numel(),
                     "param0": hex(run.opt.buf[0].data_ptr()), "grad0": hex(sets[0][0][0].data_ptr())})
        run.close()
        del run, junk
        torch.cuda.empty_cache()
        junk = torch.empty(rs.randrange(1, 4000) * (1 << 20) + rs.randrange(0, 512) * 4096, dtype=torch.uint8, device=dev)
    t = sorted(r["k_update_ms_median"] for r in rows)
    print(json.dumps({
        "metric": "k_update time over placements of the optimizer state in memory (ms, steps without a probe)",
        "workload": f"{wl.name}: {wl.n_tensors} tensors, {N} params" + (", every layer FP32" if args.all_fp32 else ""),
        "launches_of_k_update_per_placement": PLACEMENT_WARM + PLACEMENT_TIMED,
        "min_ms": t[0], "median_ms": t[len(t) // 2], "max_ms": t[-1], "mean_ms": sum(t) / len(t),
        "placements": rows}))


def power_variant(wl, hyper, dev, k, K):
    """Short form of --mode power for the `variants` record: ms per iteration and the two passes."""
    import torch

    import paper_2508_16905_amd as ta

    L, N = wl.n_tensors, wl.total_params
    opt = ta.TriAccel(dict(hyper, power_k=k), [wl.init_param(l, device=dev) for l in range(L)], grad_dtype=wl.grad_dtype)
    us = [wl.power_start(l, k, device=dev) for l in range(L)]
    hus = []
    for l in range(L):
        g = torch.Generator(device=dev)
        g.manual_seed(1000 + l)
        h = torch.zeros_like(us[l])
        h[:, : wl.numel(l)] = torch.randn(k, wl.numel(l), generator=g, device=dev) * float(wl.layer_consts(l).get("d", 1.0))
        hus.append(h)
    opt.set_profiling(True)
    for _ in range(2):
        opt.power_iter(us, hus, k)
    torch.cuda.synchronize()
    stage = [0.0, 0.0, 0.0]
    t0 = time.perf_counter()
    for _ in range(K):
        opt.power_iter(us, hus, k)
        stage = [a + b for a, b in zip(stage, opt.power_times())]   # synchronises each call
    ms = (time.perf_counter() - t0) * 1e3 / K
    stage = [x / K for x in stage]
    opt.close()
    pass_bytes = 8.0 * k * N
    return {"ms_per_iteration": ms, "params_per_s": N / (ms / 1e3), "bytes_per_param": 16.0 * k,
            "gram_ms": stage[0], "gram_frac_of_peak": pass_bytes / 1e9 / (stage[0] / 1e3) / HBM_PEAK_GBPS,
            "apply_ms": stage[2], "apply_frac_of_peak": pass_bytes / 1e9 / (stage[2] / 1e3) / HBM_PEAK_GBPS,
            "frac_of_peak": 2 * pass_bytes / 1e9 / ((stage[0] + stage[1] + stage[2]) / 1e3) / HBM_PEAK_GBPS}


def bench_power(args, wl, hyper, dev):
    """One call = one power iteration (Sec. 3.2) on k vectors for every tensor of the workload."""
    import torch

    import paper_2508_16905_amd as ta

    K, W, k = args.steps, min(args.warmup, 5), args.power_k
    L, N = wl.n_tensors, wl.total_params
    opt = ta.TriAccel(dict(hyper, power_k=k), [wl.init_param(l, device=dev) for l in range(L)], grad_dtype=wl.grad_dtype)
    us = [wl.power_start(l, k, device=dev) for l in range(L)]
    # stand-in products with the scale structure of H u (fixed over the timed calls)
    hus = []
    for l in range(L):
        g = torch.Generator(device=dev)
        g.manual_seed(1000 + l)
        h = torch.zeros_like(us[l])
        h[:, : wl.numel(l)] = torch.randn(k, wl.numel(l), generator=g, device=dev) * float(wl.layer_consts(l).get("d", 1.0))
        hus.append(h)
    torch.cuda.synchronize()
    print(f"[bench] power iteration, {wl.name}: {L} tensors, {N} params, k = {k}, "
          f"{torch.cuda.memory_allocated() / 2**30:.1f} GiB allocated", file=sys.stderr, flush=True)
    opt.set_profiling(True)
    for _ in range(W):
        opt.power_iter(us, hus, k)
    torch.cuda.synchronize()
    stage = [0.0, 0.0, 0.0]
    t0 = time.perf_counter()
    for _ in range(K):
        opt.power_iter(us, hus, k)
        if args.power_stage_times:
            stage = [a + b for a, b in zip(stage, opt.power_times())]
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / K
    if not args.power_stage_times:
        stage = [x * K for x in opt.power_times()]   # the last call only
    stage = [x / K for x in stage]
    info = opt.power_state()
    assert all(i.deficient == 0 for i in info)
    pass_bytes = 8.0 * k * N   # each pass: k vectors read + k vectors read or written, 4 bytes each
    gram_gbps, apply_gbps = pass_bytes / 1e9 / (stage[0] / 1e3), pass_bytes / 1e9 / (stage[2] / 1e3)
    dom = ("k_power_gram", stage[0], gram_gbps) if stage[0] >= stage[2] else ("k_power_apply", stage[2], apply_gbps)
    traffic = measured_power_traffic(wl.name, k, dom[0], args.tensors)
    out = {
        "metric": "power-iteration throughput (params/s per iteration on k vectors per layer)",
        "value": N / (ms / 1e3), "unit": "params/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {L} tensors, {N} params, one power iteration on k = {k} fp32 vectors per tensor"},
        "roofline": {"bound": "hbm", "kernel": dom[0], "achieved": dom[2], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": dom[2] / HBM_PEAK_GBPS, "alg_bytes_per_launch": pass_bytes,
                     "traffic": traffic,
                     "traffic_from": None if traffic is None else MEASURED_TRAFFIC["power"]["from"] + " (not counters of this run)"},
        "step": {"alg_bytes_per_param": 16.0 * k, "alg_GB": 2 * pass_bytes / 1e9,
                 "GBps": 2 * pass_bytes / 1e9 / (ms / 1e3), "frac_of_peak": 2 * pass_bytes / 1e9 / (ms / 1e3) / HBM_PEAK_GBPS},
        "stages": {"gram": {"ms": round(stage[0], 4), "GBps": round(gram_gbps, 1)}, "layer": {"ms": round(stage[1], 4)},
                   "apply": {"ms": round(stage[2], 4), "GBps": round(apply_gbps, 1)}},
    }
    if not args.no_cpu_baseline:
        import oracle
        from _runner import to_numpy

        idx = [0]
        cfg = oracle.OracleConfig.from_hyper(hyper)
        orc = oracle.OracleTriAccel(cfg, [to_numpy(wl.init_param(l)) for l in idx], [wl.init_dtype(l) for l in idx],
                                    [wl.grad_dtype] * len(idx))
        uo = [to_numpy(us[l])[:, : wl.numel(l)].copy() for l in idx]
        ho = [to_numpy(hus[l])[:, : wl.numel(l)].copy() for l in idx]
        t0 = time.perf_counter()
        orc.power_step(uo, ho, k, False)
        dt = time.perf_counter() - t0
        n = sum(wl.numel(l) for l in idx)
        out["cpu_baseline"] = {"value": n / dt, "unit": "params/s", "cores": 1, "kind": "oracle",
                               "sample": f"first tensor ({n} params, k = {k}) of the workload, 1 iteration, {dt:.2f} s wall"}
    opt.close()
    print(json.dumps(out))


def _oracle_timed(orc, gs, zs, hzs, args, budget_s):
    steps, t0 = 0, time.perf_counter()
    while True:
        orc.step(gs, zs, hzs, *args)
        steps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or steps >= 2000:
            return steps, dt


def cpu_baseline(wl, hyper, n_sample, scale):
    """The CPU oracle, as it stands, timed on a bounded sample of the same workload: the first tensors
    up to about 1.5e8 parameters (the whole workload when it is smaller), as many steps as fit in
    about six seconds of wall time (twice: all cores, then one thread)."""
    import oracle
    from _runner import to_numpy

    idx = list(range(wl.n_tensors if wl.total_params <= 150_000_000 else min(n_sample, wl.n_tensors)))
    while len(idx) > 1 and sum(wl.numel(l) for l in idx) > 150_000_000:
        idx.pop()
    cores = max(1, min(len(idx), 16, os.cpu_count() or 1))
    cfg = oracle.OracleConfig.from_hyper(hyper)
    params = [to_numpy(wl.init_param(l)) for l in idx]
    # inputs of the first generator step, drawn again (the resident batches may have been released)
    dev = "cuda:0"
    g = [to_numpy(wl.grad(1, l, scale, device=dev)) for l in idx]
    if hyper.get("curvature_source", 0) == 1:
        z = hz = [None] * len(idx)
    else:
        pr = [wl.probe(1, l, scale, device=dev) for l in idx]
        z, hz = [to_numpy(p[0]) for p in pr], [to_numpy(p[1]) for p in pr]
    args = (float(hyper["lr"]), scale, int(hyper["batch_size"]), 8, 10)
    orc = oracle.OracleTriAccel(cfg, params, [wl.init_dtype(l) for l in idx], [wl.grad_dtype] * len(idx), workers=cores)
    steps, dt = _oracle_timed(orc, g, z, hz, args, 6.0)
    n = sum(wl.numel(l) for l in idx)
    # the same oracle on one thread, largest tensor of the sample only
    big = max(range(len(idx)), key=lambda i: wl.numel(idx[i]))
    one = oracle.OracleTriAccel(cfg, [params[big]], [wl.init_dtype(idx[big])], [wl.grad_dtype], workers=1)
    steps1, dt1 = _oracle_timed(one, [g[big]], [z[big]], [hz[big]], args, 6.0)
    return {
        "value": n * steps / dt,
        "unit": "params/s",
        "cores": cores,
        "kind": "oracle",
        "sample": f"first {len(idx)} tensors ({n} params) of the workload, {steps} step(s), {dt:.2f} s wall",
        "single_thread_value": wl.numel(idx[big]) * steps1 / dt1,
        "single_thread_sample": f"one tensor ({wl.numel(idx[big])} params), {steps1} step(s), {dt1:.2f} s wall",
    }


def cpu_per_config():
    """The oracle on the other four configurations, about two seconds each, all cores (the largest of them
    on its first tensors up to about 2e7 parameters)."""
    import oracle
    from _runner import to_numpy
    from workloads import get_workload

    out = {}
    for name in ("tiny_mlp", "resnet18", "efficientnet_b0", "mixed_state"):
        wl = get_workload(name)
        idx = list(range(wl.n_tensors))
        while len(idx) > 1 and sum(wl.numel(l) for l in idx) > 20_000_000:
            idx.pop()
        scale = float(wl.hyper["loss_scale"])
        cores = max(1, min(len(idx), 16, os.cpu_count() or 1))
        cfg = oracle.OracleConfig.from_hyper(wl.hyper)
        params = [to_numpy(wl.init_param(l)) for l in idx]
        g = [to_numpy(wl.grad(1, l, scale)) for l in idx]
        pr = [wl.probe(1, l, scale) for l in idx]
        z, hz = [to_numpy(p[0]) for p in pr], [to_numpy(p[1]) for p in pr]
        orc = oracle.OracleTriAccel(cfg, params, [wl.init_dtype(l) for l in idx], [wl.grad_dtype] * len(idx), workers=cores)
        steps, dt = _oracle_timed(orc, g, z, hz, (float(wl.hyper["lr"]), scale, int(wl.hyper["batch_size"]), 8, 10), 2.0)
        n = sum(wl.numel(l) for l in idx)
        out[name] = {"value": n * steps / dt, "unit": "params/s", "cores": cores,
                     "sample": f"{len(idx)} of {wl.n_tensors} tensors ({n} params), {steps} step(s), {dt:.2f} s wall"}
    return out


if __name__ == "__main__":
    main()
