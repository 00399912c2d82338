"""AddressSanitizer + UndefinedBehaviorSanitizer runs on the CPU: the oracle (plain C) and the
library's host-only layer (descriptor validation, geometry, the sizing walk).  GPU code is not
sanitised (not available for device code here): -Xarch_host keeps the flags on the host pass."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1",
           OMP_NUM_THREADS="2")


def _run(exe):
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=ENV, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr, res.stderr
    return res.stdout


def test_oracle_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.check_call(["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined",
                           "-fno-omit-frame-pointer", "-fno-sanitize-recover=undefined",
                           os.path.join(ROOT, "oracle", "litevar_oracle.c"), os.path.join(HERE, "oracle_main.c"),
                           "-lm", "-o", exe])
    out = _run(exe)
    assert "pairs mode 0: 395" in out and "pairs mode 1: 128" in out      # the two worked examples' totals
    assert "probs sum mode 0: 1.000000000000" in out and "probs sum mode 1: 1.000000000000" in out


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="no hipcc")
def test_library_host_layer_under_asan_and_ubsan(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    csrc = os.path.join(ROOT, "paper_2411_17178_amd", "csrc")
    from paper_2411_17178_amd.build import SOURCES
    exe = str(tmp_path / "host_san")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fno-honor-nans",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
           "-I", os.path.join(ROOT, "include"), "-o", exe, os.path.join(HERE, "host_layer_main.cpp")] + \
          [os.path.join(csrc, s) for s in SOURCES]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-3000:]
    out = _run(exe)
    assert "tiny mode 0 waves 16: 395" in out and "tiny mode 1 waves 4: 128" in out and out.strip().endswith("ok")
