"""Mutation check of the oracle's pins (CPU only; not collected by pytest -- run it by hand:
``python tests/oracle_mutants.py [-j 8] [--gpu] [--logdir DIR] [indices...]``, about twenty minutes on eight cores).

Each entry plants ONE plausible mistake in a private copy of the oracle (a dropped term, a wrong
sign or comparison, swapped operands, an off-by-one, a wrong counter) and runs the CPU tests of the
oracle against that copy.  A mutant that no test notices points at a missing pin.  The
repository's own files are never modified.

With ``--gpu`` (on a machine with an MI355X) the mutated oracle is instead put beside the
UNCHANGED HIP library and the GPU parity tests are run: every mutant must make them fail, which
shows that those tests really compare what the oracle computes (the mistake is in the oracle, on
the CPU; the GPU code runs as built)."""
import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.abspath(os.path.join(os.path.dirname(__file__), ".."))
C = "oracle/triaccel_oracle.c"
S = "oracle/step.py"
M = [
 (C, "double d = (double)(widen(g, dtype, i) * inv_scale) - mean;", "double d = (double)(widen(g, dtype, i) * inv_scale) + mean;"),
 (C, "*var_out = q / (double)n;", "*var_out = q / (double)(n > 1 ? n - 1 : 1);"),
 (C, "double mean = s / (double)n;", "double mean = s / (double)(n + 1);"),
 (C, "for (int64_t i = 0; i < n; ++i) s += (double)(widen(g, dtype, i) * inv_scale);", "for (int64_t i = 0; i < n; ++i) s += (double)(widen(g, dtype, i));"),
 (C, "return (float)((double)beta * (double)v_prev + (1.0 - (double)beta) * var);", "return (float)((1.0 - (double)beta) * (double)v_prev + (double)beta * var);"),
 (C, "return (float)((double)beta * (double)v_prev + (1.0 - (double)beta) * var);", "return (float)((double)beta * (double)v_prev + var);"),
 (C, "if (first) return (float)var;", "if (first) return (float)((1.0 - (double)beta) * var);"),
 (C, "        float u = z[i] * hz[i];\n        u = u * inv_scale;", "        float u = hz[i];\n        u = u * inv_scale;"),
 (C, "        float u = z[i] * hz[i];\n        u = u * inv_scale;", "        float u = z[i] * hz[i];"),
 (C, "        float p = omb * u;\n        h[i] = fmaf(beta_h, h[i], p);\n    }\n}\n\n/* Empirical", "        float p = beta_h * u;\n        h[i] = fmaf(omb, h[i], p);\n    }\n}\n\n/* Empirical"),
 (C, "        if (first) { h[i] = u; continue; }\n        float p = omb * u;\n        h[i] = fmaf(beta_h, h[i], p);\n    }\n}\n\n/* Empirical", "        if (first) { h[i] = omb * u; continue; }\n        float p = omb * u;\n        h[i] = fmaf(beta_h, h[i], p);\n    }\n}\n\n/* Empirical"),
 (C, "if (!isfinite(u)) { *nonfinite = 1; continue; }\n        if (first) { h[i] = u; continue; }\n        float p = omb * u;\n        h[i] = fmaf(beta_h, h[i], p);\n    }\n}\n\n/* Empirical", "if (!isfinite(u)) { *nonfinite = 1; h[i] = 0.0f; continue; }\n        if (first) { h[i] = u; continue; }\n        float p = omb * u;\n        h[i] = fmaf(beta_h, h[i], p);\n    }\n}\n\n/* Empirical"),
 (C, "float u = x * x;", "float u = fabsf(x);"),
 (C, "float x = widen(g, g_dtype, i) * inv_scale;\n        float u = x * x;", "float x = widen(g, g_dtype, i);\n        float u = x * x;"),
 (C, "int64_t k = n - (int64_t)(((__int128)n * (int64_t)s_ppm) / 1000000);", "int64_t k = (int64_t)(((__int128)n * (int64_t)s_ppm) / 1000000);"),
 (C, "int64_t k = n - (int64_t)(((__int128)n * (int64_t)s_ppm) / 1000000);", "int64_t k = n - (int64_t)(((__int128)n * (int64_t)s_ppm + 999999) / 1000000);"),
 (C, "uint32_t theta = sorted[k - 1];", "uint32_t theta = sorted[k < n ? k : n - 1];"),
 (C, "if (a[i] >= theta && a[i] > 0) {", "if (a[i] > theta && a[i] > 0) {"),
 (C, "if (a[i] >= theta && a[i] > 0) {", "if (a[i] >= theta) {"),
 (C, "a[i] = bits_of(h[i]) & 0x7fffffffu;", "a[i] = bits_of(h[i]);"),
 (C, "return (x < y) - (x > y);", "return (x > y) - (x < y);"),
 (C, "mask[i >> 5] |= 1u << (i & 31);", "mask[i >> 5] |= 1u << (31 - (i & 31));"),
 (C, "if (a[i] > lam) lam = a[i];", "if (a[i] < lam || lam == 0) lam = a[i];"),
 (C, "int base = (v < tau_low) ? ORC_FP16 : (v < tau_high) ? ORC_BF16 : ORC_FP32;", "int base = (v <= tau_low) ? ORC_FP16 : (v < tau_high) ? ORC_BF16 : ORC_FP32;"),
 (C, "int base = (v < tau_low) ? ORC_FP16 : (v < tau_high) ? ORC_BF16 : ORC_FP32;", "int base = (v < tau_low) ? ORC_FP16 : (v <= tau_high) ? ORC_BF16 : ORC_FP32;"),
 (C, "int base = (v < tau_low) ? ORC_FP16 : (v < tau_high) ? ORC_BF16 : ORC_FP32;", "int base = (v < tau_low) ? ORC_BF16 : (v < tau_high) ? ORC_FP16 : ORC_FP32;"),
 (C, "if (lambda > tau_curv && base < ORC_FP32) base += 1;", "if (lambda >= tau_curv && base < ORC_FP32) base += 1;"),
 (C, "if (lambda > tau_curv && base < ORC_FP32) base += 1;", "if (lambda > tau_curv) base = ORC_FP32;"),
 (C, "float den = fmaf(alpha, lambda, 1.0f);\n    return lr / den;", "float den = fmaf(alpha, lambda, 0.0f);\n    return lr / den;"),
 (C, "float den = fmaf(alpha, lambda, 1.0f);\n    return lr / den;", "float den = fmaf(alpha, lambda, 1.0f);\n    return lr * den;"),
 (C, "        float d = fmaf(wd, th, gt);\n        float mm;\n        if (m) { m[i] = fmaf(mu, m[i], d); mm = m[i]; } else { mm = d; }\n        next[i] = fmaf(neg_eta, mm, th);", "        float d = fmaf(-wd, th, gt);\n        float mm;\n        if (m) { m[i] = fmaf(mu, m[i], d); mm = m[i]; } else { mm = d; }\n        next[i] = fmaf(neg_eta, mm, th);"),
 (C, "        if (m) { m[i] = fmaf(mu, m[i], d); mm = m[i]; } else { mm = d; }\n        next[i] = fmaf(neg_eta, mm, th);", "        if (m) { m[i] = fmaf(mu, m[i], d); mm = m[i]; } else { mm = d; }\n        next[i] = fmaf(eta, mm, th);"),
 (C, "        if (m) { m[i] = fmaf(mu, m[i], d); mm = m[i]; } else { mm = d; }\n        next[i] = fmaf(neg_eta, mm, th);", "        if (m) { mm = m[i]; m[i] = fmaf(mu, m[i], d); } else { mm = d; }\n        next[i] = fmaf(neg_eta, mm, th);"),
 (C, "        if (m) { m[i] = fmaf(mu, m[i], d); mm = m[i]; } else { mm = d; }\n        next[i] = fmaf(neg_eta, mm, th);", "        if (m) { m[i] = fmaf(mu, m[i], d); mm = d; } else { mm = d; }\n        next[i] = fmaf(neg_eta, mm, th);"),
 (C, "        if (m) { m[i] = fmaf(mu, m[i], d); mm = m[i]; } else { mm = d; }\n        next[i] = fmaf(neg_eta, mm, th);", "        if (m) { m[i] = fmaf(mu, m[i], (1.0f - mu) * d); mm = m[i]; } else { mm = d; }\n        next[i] = fmaf(neg_eta, mm, th);"),
 (C, "        float gt = widen(g, grad_dtype, i) * inv_scale;\n        float d = fmaf(wd, th, gt);\n        float mm;\n        if (m) { m[i] = fmaf(mu, m[i], d); mm = m[i]; } else { mm = d; }\n        next[i] = fmaf(neg_eta, mm, th);", "        float gt = widen(g, grad_dtype, i);\n        float d = fmaf(wd, th, gt);\n        float mm;\n        if (m) { m[i] = fmaf(mu, m[i], d); mm = m[i]; } else { mm = d; }\n        next[i] = fmaf(neg_eta, mm, th);"),
 (C, "float a = ((mask[i >> 5] >> (i & 31)) & 1u) ? fabsf(h[i]) : 0.0f;", "float a = fabsf(h[i]);"),
 (C, "float a = ((mask[i >> 5] >> (i & 31)) & 1u) ? fabsf(h[i]) : 0.0f;", "float a = ((mask[i >> 5] >> (i & 31)) & 1u) ? h[i] : 0.0f;"),
 (C, "float a = ((mask[i >> 5] >> (i & 31)) & 1u) ? fabsf(h[i]) : 0.0f;", "float a = ((mask[i >> 5] >> (i & 31)) & 1u) ? 0.0f : fabsf(h[i]);"),
 (C, "if (skipped) { *good_steps = 0; return scale * backoff; }", "if (skipped) { return scale * backoff; }"),
 (C, "if (*good_steps >= growth_interval) { *good_steps = 0; return scale * growth; }", "if (*good_steps > growth_interval) { *good_steps = 0; return scale * growth; }"),
 (C, "if (*good_steps >= growth_interval) { *good_steps = 0; return scale * growth; }", "if (*good_steps >= growth_interval) { return scale * growth; }"),
 (C, "if (used < rho_low * total) b += delta_up;", "if (used <= rho_low * total) b += delta_up;"),
 (C, "else if (used > rho_high * total) b -= delta_down;", "else if (used >= rho_high * total) b -= delta_down;"),
 (C, "else if (used > rho_high * total) b -= delta_down;", "else if (used > rho_high * total) b -= delta_up;"),
 (C, "if (b < b_min) b = b_min;", "if (b < b_min) b = b_min + 1;"),
 (C, "lam = uw / uu;", "lam = uw / sqrt(uu);"),
 (C, "lam = uw / uu;", "lam = ww / uw;"),
 (C, "rr = sqrt(rr) / sqrt(uu);", "rr = sqrt(rr);"),
 (C, "for (int64_t i = 0; i < n; ++i) v[i] -= dot * qp[i];", "for (int64_t i = 0; i < n; ++i) v[i] += dot * qp[i];"),
 (C, "for (int32_t p = 0; p < j; ++p) {", "for (int32_t p = 0; p + 1 < j; ++p) {"),
 (C, "for (int64_t i = 0; i < n; ++i) v[i] = v[i] / nv;", "for (int64_t i = 0; i < n; ++i) v[i] = v[i] / vv;"),
 (C, "for (int64_t i = 0; i < n; ++i) v[i] = (double)wj[i];", "for (int64_t i = 0; i < n; ++i) v[i] = (double)uj[i];"),
 (C, "hnorm[j] = sqrt(ww);", "hnorm[j] = ww;"),
 (C, "if (vv <= 1e-12 * ww) {", "if (vv <= 1e-3 * ww) {"),
 (S, "t.v = f32(L.oracle_var_ema(t.v, var.value, f32(cfg.beta_var), int(first)))", "t.v = f32(L.oracle_var_ema(t.v, var.value, f32(cfg.beta_var), 0))"),
 (S, "int(t.probes_seen == 0), C.byref(flag))\n            else:", "int(first), C.byref(flag))\n            else:"),
 (S, "f32(cfg.beta_curv), int(t.probes_seen == 0), C.byref(flag))\n            t.curv_nonfinite", "f32(cfg.beta_curv), int(first), C.byref(flag))\n            t.curv_nonfinite"),
 (S, "t.prev_code = t.code\n", "\n"),
 (S, "        if control_step:\n            t.lam_ctrl = t.lam\n", "        t.lam_ctrl = t.lam\n        if control_step:\n"),
 (S, "t.eta = f32(L.oracle_eta(f32(lr), f32(cfg.alpha), t.lam_ctrl))", "t.eta = f32(L.oracle_eta(f32(lr), f32(cfg.alpha), t.lam))"),
 (S, "L.oracle_update(t.buf.ctypes.data, t.prev_code, t.code,", "L.oracle_update(t.buf.ctypes.data, t.prev_code, t.prev_code,"),
 (S, "skipped = int(any(t.found_inf for t in self.tensors) or overflow_elsewhere)", "skipped = int(all(t.found_inf for t in self.tensors) or overflow_elsewhere)"),
 (S, "control_step = self.applied_steps % cfg.ctrl_interval == 0", "control_step = self.step_index % cfg.ctrl_interval == 0"),
 (S, "control_step = self.applied_steps % cfg.ctrl_interval == 0", "control_step = self.applied_steps % cfg.ctrl_interval == 1 % cfg.ctrl_interval"),
 (S, "first = self.applied_steps == 1", "first = self.step_index == 1"),
 (S, "inv_scale = f32(1.0) / f32(loss_scale)", "inv_scale = f32(loss_scale)"),
 (S, "t.lam_power = np.float32(np.max(np.abs(ray)))", "t.lam_power = np.float32(np.max(ray))"),
 (S, "        if cfg.lambda_source == 1:\n            t.lam = t.lam_power\n", ""),
 (S, "        if not skipped:\n            self.applied_steps += 1", "        if True:\n            self.applied_steps += 1"),
 (S, "t.theta, t.nnz, t.lam = f32(theta.value), int(nnz.value), f32(lam.value)", "t.theta, t.nnz, t.lam = f32(theta.value), int(nnz.value), f32(theta.value)"),
]


GPU = False
LOGDIR = None


def check(idx):
    f, a, b = M[idx]
    src = open(os.path.join(ROOT, f)).read()
    label = (b.strip().splitlines() or ["<lines deleted>"])[0][:90]
    if src.count(a) < 1:
        return idx, "PATTERN NOT FOUND", label, ""
    tree = tempfile.mkdtemp(prefix="oracle_mutant_")
    try:
        for d in ("oracle", "tests", "workloads", "include"):
            shutil.copytree(os.path.join(ROOT, d), os.path.join(tree, d),
                            ignore=shutil.ignore_patterns("__pycache__", "*.so"))
        with open(os.path.join(tree, f), "w") as fh:
            fh.write(src.replace(a, b, 1))
        if GPU:
            os.symlink(os.path.join(ROOT, "paper_2508_16905_amd"), os.path.join(tree, "paper_2508_16905_amd"))
            # the quick parity tests (each a few seconds) that between them touch every part of the step
            quick = ("tiny_mlp or ragged or mixed_state or control_interval or no_momentum or half_precision or "
                     "skip_step or nonfinite_probe or fisher or elementwise_step or exact_thresholds or fixed_top_k or "
                     "batch_rule_trace or arrives_after or skipped_first_call")
            tests = ["-m", "gpu", "--timeout", "300", "--timeout-method", "thread", "-k", quick + " or power",
                     "tests/test_gpu_parity.py", "tests/test_gpu_power.py"]
        else:
            tests = sorted("tests/" + t for t in os.listdir(os.path.join(tree, "tests"))
                           if t.startswith("test_oracle_") or t == "test_workloads.py")
        cmd = [sys.executable, "-u", "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + tests
        if LOGDIR:
            # the run's own output goes to a file as it is produced (a long GPU run stays visibly alive)
            log = os.path.join(LOGDIR, f"mutant_{idx}.log")
            with open(log, "w") as fh:
                r = subprocess.run(cmd + ["-v"], cwd=tree, stdout=fh, stderr=subprocess.STDOUT, text=True)
            out = open(log).read()
        else:
            r = subprocess.run(cmd, cwd=tree, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
            out = r.stdout
        where = [l for l in out.splitlines() if "Error" in l or "FAILED" in l][:1]
        return idx, "killed" if r.returncode != 0 else "SURVIVED", label, where[0][:100] if where else ""
    finally:
        shutil.rmtree(tree, ignore_errors=True)


def main():
    args = sys.argv[1:]
    jobs = 8
    global GPU, LOGDIR
    if args[:1] == ["-j"]:
        jobs, args = int(args[1]), args[2:]
    if args[:1] == ["--gpu"]:
        GPU, args = True, args[1:]
    if args[:1] == ["--logdir"]:
        LOGDIR, args = os.path.abspath(args[1]), args[2:]
        os.makedirs(LOGDIR, exist_ok=True)
    todo = [int(x) for x in args] or list(range(len(M)))
    survivors = []
    from concurrent.futures import as_completed

    with ThreadPoolExecutor(jobs) as pool:
        for fut in as_completed([pool.submit(check, i) for i in todo]):
            idx, outcome, label, where = fut.result()
            print(idx, outcome, "|", label, "|", where, flush=True)
            if outcome != "killed":
                survivors.append(idx)
    survivors.sort()
    print(f"{len(todo) - len(survivors)} of {len(todo)} mutants killed; survivors: {survivors}")
    return 1 if survivors else 0


if __name__ == "__main__":
    sys.exit(main())
