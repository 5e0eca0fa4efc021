"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only): the library's
planner / tile-table builder is fuzzed by a C++ driver, the oracle is run by a C driver on
exactly-sized heap buffers.  GPU code is not involved."""
from __future__ import annotations

import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
# the sanitizer runtime is linked statically so that it does not depend on being the first
# library loaded into the process
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0")


def _run(cmd, **kw):
    try:
        return subprocess.run(cmd, check=True, capture_output=True, text=True, **kw)
    except subprocess.CalledProcessError as e:
        if "does not come first" in (e.stderr or ""):   # a preloaded library keeps ASan from starting
            pytest.skip("AddressSanitizer cannot start in this environment")
        raise AssertionError("%s\n%s\n%s" % (" ".join(cmd), e.stdout, e.stderr))


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_planner_and_tiles_under_sanitizers(tmp_path):
    exe = str(tmp_path / "plan_fuzz")
    _run(["g++", "-std=c++17", *SAN, "-I", os.path.join(ROOT, "include"),
          "-I", os.path.join(ROOT, "paper_2302_12445_amd", "csrc"),
          os.path.join(ROOT, "tests", "native", "plan_fuzz.cpp"),
          os.path.join(ROOT, "paper_2302_12445_amd", "csrc", "plan.cpp"), "-o", exe])
    out = _run([exe, "300"], env=ENV)
    assert "cases ok" in out.stdout


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    _run(["gcc", "-ffp-contract=off", *SAN, os.path.join(ROOT, "tests", "native", "oracle_sanitize.c"),
          os.path.join(ROOT, "oracle", "dear_oracle.c"), "-o", exe])
    out = _run([exe], env=ENV)
    assert "ok" in out.stdout
