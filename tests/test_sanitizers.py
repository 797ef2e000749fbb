"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the host-side code (no GPU): the C oracle on small seeded
inputs, and the library's argument validation / workspace sizing / segment choice over a grid of parameter values
(csrc/sla_api.hip with the host pass instrumented and the kernel launchers stubbed out)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, **kw)
    assert res.returncode == 0, f"{' '.join(cmd)}\n{res.stdout}\n{res.stderr}"
    return res.stdout


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    _run(["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fopenmp"] + SAN +
         [os.path.join(ROOT, "oracle", "sla_oracle.c"), os.path.join(ROOT, "tests", "sanitize", "oracle_main.c"), "-lm",
          "-o", exe])
    assert "ok" in _run([exe], env=ENV)


def test_host_validation_under_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not available")
    exe = str(tmp_path / "abi_san")
    host = [x for f in SAN for x in ("-Xarch_host", f)]
    _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17"] + host +
         ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
          "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "paper_2602_01744_amd", "csrc", "sla_api.hip"),
          os.path.join(ROOT, "tests", "sanitize", "abi_main.cpp"), "-o", exe])
    assert "0 failures" in _run([exe], env=ENV)
