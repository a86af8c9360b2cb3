"""Host-side checks that need no GPU: the library loads, exports every symbol the header declares,
the ctypes structures have the C layout, and the pure host entry points behave."""
import ctypes as C
import os
import re
import subprocess

import pytest

import paper_2508_16905_amd as ta
from paper_2508_16905_amd import binding as B
from paper_2508_16905_amd.build import build_library

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "triaccel.h")


@pytest.fixture(scope="module")
def lib():
    build_library(force=False)
    return ta.load_library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(triaccel_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert "triaccel_init" in names and "triaccel_step" in names and len(names) >= 10
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(B.EXPORTS) == names


def test_ctypes_layout_matches_the_header(tmp_path):
    src = tmp_path / "sizes.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "triaccel.h"\n'
        "int main(void){printf(\"%zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu %zu\\n\", sizeof(triaccel_config),"
        " sizeof(triaccel_tensor), sizeof(triaccel_step_args), sizeof(triaccel_step_result),"
        " sizeof(triaccel_layer_info), sizeof(triaccel_stage_times), offsetof(triaccel_config, rho_low),"
        " offsetof(triaccel_tensor, numel), offsetof(triaccel_layer_info, code), sizeof(triaccel_power_tensor),"
        " sizeof(triaccel_power_info), offsetof(triaccel_power_info, deficient),"
        " offsetof(triaccel_config, lambda_source)); return 0;}\n")
    exe = tmp_path / "sizes"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    want = [C.sizeof(B.Config), C.sizeof(B.Tensor), C.sizeof(B.StepArgs), C.sizeof(B.StepResult),
            C.sizeof(B.LayerInfo), C.sizeof(B.StageTimes), B.Config.rho_low.offset, B.Tensor.numel.offset,
            B.LayerInfo.code.offset, C.sizeof(B.PowerTensor), C.sizeof(B.PowerInfo), B.PowerInfo.deficient.offset,
            B.Config.lambda_source.offset]
    assert [int(x) for x in out] == want


def test_strerror_and_batch_rule(lib):
    assert ta.triaccel_strerror(0) == "success"
    assert "aligned" in ta.triaccel_strerror(-5)
    from workloads import get_workload

    cfg = ta.Config.from_hyper(get_workload("tiny_mlp").hyper)
    # Sec. 3.3 with rho_low = 0.70, rho_high = 0.90, delta = 16, clamp [16, 4096]
    assert ta.triaccel_batch_next(cfg, 96, 699, 1000) == 112
    assert ta.triaccel_batch_next(cfg, 96, 700, 1000) == 96
    assert ta.triaccel_batch_next(cfg, 96, 900, 1000) == 96
    assert ta.triaccel_batch_next(cfg, 96, 901, 1000) == 80
    assert ta.triaccel_batch_next(cfg, 16, 999, 1000) == 16
    assert ta.triaccel_batch_next(cfg, 4090, 0, 1000) == 4096


def test_argument_errors_without_a_device(lib):
    handle = C.c_void_p()
    assert lib.triaccel_init(C.byref(handle), None, None, 1, None) == -4
    cfg = B.Config()
    assert lib.triaccel_init(C.byref(handle), C.byref(cfg), None, 1, None) == -1  # struct_size not set
    assert lib.triaccel_step(None, None, 0, None) == -7
    assert lib.triaccel_result(None, None) == -7
    lib.triaccel_destroy(None)


def test_missing_library_is_an_error(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libtriaccel.so")
    with pytest.raises(RuntimeError):
        B.load_library()
