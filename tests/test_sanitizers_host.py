"""Host-side AddressSanitizer + UndefinedBehaviorSanitizer runs (no GPU): the CPU oracle's C code and
the runtime's host logic (workspace layout, prefill GEMM plan and slice map, argument validation) are
compiled with the sanitizers into small stand-alone drivers and executed; any out-of-bounds access,
signed overflow or misaligned access aborts the driver."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]


def _run(cmd, exe, tmp_path):
    res = subprocess.run(cmd, cwd=ROOT, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    assert res.returncode == 0, "build failed:\n" + out
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], cwd=str(tmp_path), stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env)
    assert run.returncode == 0 and "sanitizer run ok" in run.stdout, run.stdout[-4000:]
    return run.stdout


@pytest.mark.parametrize("precision", ["f32", "f64"])
def test_oracle_under_asan_ubsan(tmp_path, precision):
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    exe = str(tmp_path / ("oracle_san_" + precision))
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp"] + SAN + (["-DORACLE_F64"] if precision == "f64" else []) + \
          [os.path.join("tests", "sanitize", "oracle_san_main.c"), "-lm", "-o", exe]
    _run(cmd, exe, tmp_path)


def test_runtime_host_logic_under_asan_ubsan(tmp_path):
    if not os.path.exists(HIPCC):
        pytest.skip("no hipcc")
    exe = str(tmp_path / "plan_san")
    host = []
    for f in SAN:
        host += ["-Xarch_host", f]
    cmd = [HIPCC, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"] + host + \
          [os.path.join("paper_2604_23467_amd", "csrc", "ll_runtime.hip"),
           os.path.join("tests", "sanitize", "plan_san_main.cpp"), "-o", exe]
    out = _run(cmd, exe, tmp_path)
    assert "GEMM plans" in out
