"""HBM stream-pattern probe: what the MI355X sustains for the bare memory traffic of each
aggregation kernel (k streams read and summed; one stream written to k places, at once
or one after another in chunks; three streams read and two written back).  ctypes
binding of libdear_probe.so (include/dear_probe.h) plus a table printer.

    python -m paper_2302_12445_amd.hbm_probe            # one JSON line per pattern
"""
from __future__ import annotations

import ctypes as C
import json
import os
from typing import Dict, List

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdear_probe.so")

READ_K_WRITE_1, READ_1_WRITE_K, READ_1_WRITE_K_CHUNKED, READ_3_WRITE_2 = 0, 1, 2, 3
PATTERN_NAMES = {READ_K_WRITE_1: "read_k_write_1", READ_1_WRITE_K: "read_1_write_k",
                 READ_1_WRITE_K_CHUNKED: "read_1_write_k_chunked", READ_3_WRITE_2: "read_3_write_2"}
EXPORTS = ["dear_probe_streams"]

_lib = None


def load_library() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libdear_probe.so is not built: run `python -m paper_2302_12445_amd.build`")
        import torch  # noqa: F401  (one HIP runtime per process: torch's copy is loaded first)
        lib = C.CDLL(LIB_PATH)
        lib.dear_probe_streams.argtypes = [C.c_int32, C.c_int32, C.c_int64, C.c_int64, C.c_int32, C.c_int64,
                                           C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        lib.dear_probe_streams.restype = C.c_int
        _lib = lib
    return _lib


def dear_probe_streams(pattern: int, k: int, bytes_per_stream: int, chunk_bytes: int = 0,
                       elem_bytes_in: int = 4, reps: int = 10, skew_bytes: int = 0) -> Dict[str, float]:
    gbps, ms = C.c_double(), C.c_double()
    rc = load_library().dear_probe_streams(pattern, k, bytes_per_stream, chunk_bytes, elem_bytes_in, skew_bytes,
                                           reps, C.byref(gbps), C.byref(ms))
    if rc != 0:
        raise RuntimeError("dear_probe_streams: status %d" % rc)
    return {"GBps": gbps.value, "ms": ms.value}


def sweep(bytes_per_stream: int = 1 << 30, reps: int = 10) -> List[dict]:
    """The patterns of the three kernels at the worker counts of the benchmark workloads."""
    rows = []

    def run(pattern, k, elem=4, chunk=0, per_stream=bytes_per_stream, skew=0):
        r = dear_probe_streams(pattern, k, per_stream, chunk, elem, reps, skew)
        rows.append({"pattern": PATTERN_NAMES[pattern], "k": k, "elem_bytes_in": elem,
                     "chunk_MiB": chunk >> 20, "skew_bytes": skew, "bytes_per_stream_MiB": per_stream >> 20,
                     "GBps": round(r["GBps"], 1), "ms": round(r["ms"], 4), "frac_of_8TBps": round(r["GBps"] / 8000, 4)})

    for k in (1, 2, 4, 8, 16):
        run(READ_K_WRITE_1, k)
    for k in (1, 8, 16):
        run(READ_K_WRITE_1, k, elem=2, per_stream=bytes_per_stream // 2)
    for k in (1, 8, 16):
        run(READ_1_WRITE_K, k)
    for chunk in (4 << 20, 8 << 20, 16 << 20):
        run(READ_1_WRITE_K_CHUNKED, 8, chunk=chunk)
    run(READ_1_WRITE_K_CHUNKED, 16, chunk=8 << 20)
    run(READ_3_WRITE_2, 3)
    for skew in (256, 4096, 65536 + 4096, (1 << 20) + 8192):   # does shifting the streams against each other help?
        run(READ_K_WRITE_1, 8, skew=skew)
        run(READ_1_WRITE_K, 8, skew=skew)
    return rows


def main() -> None:
    import torch
    if not torch.cuda.is_available():
        raise SystemExit("hbm_probe needs a GPU")
    torch.cuda.init()
    for row in sweep():
        print(json.dumps(row), flush=True)


if __name__ == "__main__":
    main()
