"""Builds libdear.so (host planner + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libdear.so")
SOURCES = [os.path.join(CSRC, "plan.cpp"), os.path.join(CSRC, "dear_hip.hip")]
HEADERS = [os.path.join(CSRC, "dear_internal.h"), os.path.join(ROOT, "include", "dear.h")]
# measurement aid, a library of its own: bare HBM traffic patterns (include/dear_probe.h)
PROBE_LIB = os.path.join(PKG, "libdear_probe.so")
PROBE_SOURCES = [os.path.join(CSRC, "hbm_probe.hip")]
PROBE_HEADERS = [os.path.join(ROOT, "include", "dear_probe.h")]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # bit-exact fp32: one rounding per operation on host and device
    "-ffp-contract=off",
    # packed-fp32 instructions are kept out of the generated code on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _stale(lib, deps) -> bool:
    if not os.path.exists(lib):
        return True
    t = os.path.getmtime(lib)
    return any(os.path.getmtime(f) > t for f in deps)


def is_stale() -> bool:
    return _stale(LIB, SOURCES + HEADERS)


def _compile(lib, sources, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = lib + ".tmp.%d" % os.getpid()
    subprocess.run([hipcc, *HIPCC_FLAGS, *extra_flags, "-o", tmp, *sources], check=True)
    os.replace(tmp, lib)
    return lib


def build(force: bool = True, extra_flags=()) -> str:
    """Compile libdear.so.  With force=False an up-to-date library is kept."""
    if not force and not is_stale():
        return LIB
    return _compile(LIB, SOURCES, extra_flags)


def build_probe(force: bool = True) -> str:
    """Compile libdear_probe.so (the HBM stream-pattern probe)."""
    if not force and not _stale(PROBE_LIB, PROBE_SOURCES + PROBE_HEADERS):
        return PROBE_LIB
    return _compile(PROBE_LIB, PROBE_SOURCES)


if __name__ == "__main__":
    print(build())
    print(build_probe())
