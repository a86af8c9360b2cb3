"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer: the pins of the threshold,
update, statistics, curvature, power-iteration and cast routines (the sampled cast test, not the
2^32 sweeps) are run once more, in a child process, against an instrumented build of the same
source.  Any out-of-bounds access, misaligned or overflowing arithmetic aborts the child."""
import os
import subprocess
import sys

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ["test_oracle_threshold.py", "test_oracle_update.py", "test_oracle_power.py", "test_oracle_stats.py",
        "test_oracle_curvature.py", "test_oracle_fisher.py", "test_oracle_elementwise.py", "test_oracle_decisions.py",
        "test_oracle_step.py", "test_oracle_casts.py"]


def _runtime(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True, check=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_oracle_pins_pass_under_asan_and_ubsan():
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    so = oracle.build(force=True, sanitize=True)
    env = dict(os.environ)
    # the instrumented library needs its runtime in the process before anything else is loaded; what
    # the environment already preloads stays in the list
    env["LD_PRELOAD"] = ":".join(x for x in (asan, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=66"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["TRIACCEL_ORACLE_SO"] = so
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-k", "not exhaustive"]
    cmd += [os.path.join(ROOT, "tests", f) for f in PINS]
    run = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    tail = run.stdout[-3000:] + run.stderr[-3000:]
    assert run.returncode == 0, tail
    assert "AddressSanitizer" not in tail and "runtime error" not in tail, tail
    assert " passed" in run.stdout
