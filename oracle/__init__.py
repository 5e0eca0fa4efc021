"""Python face of the CPU oracle (dear_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  It never imports the HIP package and the HIP package never imports it.

Arrays are numpy: gradients as float32, or uint16 holding bfloat16 bit patterns;
shard buffers as float32 of shape (P, total_shard_len).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dear_oracle.c")
_LIB = os.path.join(_HERE, "libdear_oracle.so")
CFLAGS = ["-O2", "-ffp-contract=off", "-Wall", "-Wextra", "-shared", "-fPIC"]

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict binary32: no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(["gcc", *CFLAGS, "-o", tmp, _SRC], check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_plan.restype = C.c_int32
        _lib.oracle_plan_fixed_layers.restype = C.c_int32
        for name in ("oracle_reduce_scatter", "oracle_shard_update", "oracle_all_gather",
                     "oracle_scatter_params"):
            getattr(_lib, name).restype = None
    return _lib


def _p(a: np.ndarray, ty):
    return a.ctypes.data_as(C.POINTER(ty))


@dataclass
class OraclePlan:
    sizes: np.ndarray              # int64 [L], forward order
    P: int
    threshold_bytes: int
    grad_elem_bytes: int
    n_buckets: int
    layer_bucket: np.ndarray       # int32 [L]
    layer_offset: np.ndarray       # int64 [L]
    bucket_first_layer: np.ndarray  # int32 [B]
    bucket_n_layers: np.ndarray    # int32 [B]
    bucket_len: np.ndarray         # int64 [B]  d_b
    bucket_shard_len: np.ndarray   # int64 [B]  S_b
    bucket_shard_base: np.ndarray  # int64 [B]

    @property
    def L(self) -> int:
        return int(self.sizes.shape[0])

    @property
    def total_shard_len(self) -> int:
        return int(self.bucket_shard_len.sum())

    @property
    def total_elems(self) -> int:
        return int(self.sizes.sum())


def plan(sizes: Sequence[int], P: int, threshold_bytes: int, grad_elem_bytes: int = 4) -> OraclePlan:
    lib = _load()
    n = np.ascontiguousarray(sizes, dtype=np.int64)
    L = int(n.shape[0])
    cap = max(L, 1)
    lb = np.zeros(cap, np.int32)
    lo = np.zeros(cap, np.int64)
    bf = np.zeros(cap, np.int32)
    bn = np.zeros(cap, np.int32)
    bl = np.zeros(cap, np.int64)
    bs = np.zeros(cap, np.int64)
    bb = np.zeros(cap, np.int64)
    B = lib.oracle_plan(_p(n, C.c_int64), C.c_int32(L), C.c_int32(P), C.c_int64(threshold_bytes),
                        C.c_int32(grad_elem_bytes), _p(lb, C.c_int32), _p(lo, C.c_int64),
                        _p(bf, C.c_int32), _p(bn, C.c_int32), _p(bl, C.c_int64),
                        _p(bs, C.c_int64), _p(bb, C.c_int64))
    if B < 0:
        raise ValueError("oracle_plan: invalid arguments")
    return OraclePlan(n, P, threshold_bytes, grad_elem_bytes, B, lb[:L], lo[:L],
                      bf[:B].copy(), bn[:B].copy(), bl[:B].copy(), bs[:B].copy(), bb[:B].copy())


def plan_fixed_layers(sizes: Sequence[int], P: int, layers_per_group: int,
                      grad_elem_bytes: int = 4) -> OraclePlan:
    """The fixed-number-of-layers grouping of the tensor-fusion study (Sec. VI-G).  The
    returned plan has threshold_bytes = -1 (no buffer size is involved)."""
    lib = _load()
    n = np.ascontiguousarray(sizes, dtype=np.int64)
    L = int(n.shape[0])
    cap = max(L, 1)
    lb = np.zeros(cap, np.int32)
    lo = np.zeros(cap, np.int64)
    bf = np.zeros(cap, np.int32)
    bn = np.zeros(cap, np.int32)
    bl = np.zeros(cap, np.int64)
    bs = np.zeros(cap, np.int64)
    bb = np.zeros(cap, np.int64)
    B = lib.oracle_plan_fixed_layers(_p(n, C.c_int64), C.c_int32(L), C.c_int32(P),
                                     C.c_int32(layers_per_group), C.c_int32(grad_elem_bytes),
                                     _p(lb, C.c_int32), _p(lo, C.c_int64), _p(bf, C.c_int32),
                                     _p(bn, C.c_int32), _p(bl, C.c_int64), _p(bs, C.c_int64),
                                     _p(bb, C.c_int64))
    if B < 0:
        raise ValueError("oracle_plan_fixed_layers: invalid arguments")
    return OraclePlan(n, P, -1, grad_elem_bytes, B, lb[:L], lo[:L],
                      bf[:B].copy(), bn[:B].copy(), bl[:B].copy(), bs[:B].copy(), bb[:B].copy())


def _bucket_layers(pl: OraclePlan, buckets: Sequence[int]) -> List[int]:
    out: List[int] = []
    for b in buckets:
        first = int(pl.bucket_first_layer[b])
        out.extend(range(first, first + int(pl.bucket_n_layers[b])))
    return out


def _layers_of_shards(pl: OraclePlan, b: int, s0: int, s1: int) -> List[int]:
    """Layers of bucket b that hold a position of shards s0 .. s1-1."""
    S = int(pl.bucket_shard_len[b])
    lo, hi = s0 * S, min(s1 * S, int(pl.bucket_len[b]))
    first = int(pl.bucket_first_layer[b])
    return [l for l in range(first, first + int(pl.bucket_n_layers[b]))
            if int(pl.layer_offset[l]) < hi and int(pl.layer_offset[l]) + int(pl.sizes[l]) > lo]


def _ptr_table(pl: OraclePlan, arrays: Sequence[Sequence[Optional[np.ndarray]]], layers: Sequence[int],
               dtype, workers: Optional[range] = None):
    """Host pointer table [p*L + l].  Only the listed layers (and workers) are needed by the
    call; arrays of other layers may be None and get a null entry."""
    P, L = pl.P, pl.L
    tab = (C.c_void_p * (P * L))()
    for p in (range(P) if workers is None else workers):
        assert len(arrays[p]) == L
        for l in layers:
            a = arrays[p][l]
            assert a is not None and a.dtype == dtype and a.size == pl.sizes[l] and a.flags["C_CONTIGUOUS"]
            tab[p * L + l] = a.ctypes.data
    return tab


def _check_rows(pl: OraclePlan, *bufs: np.ndarray) -> int:
    stride = None
    for a in bufs:
        assert a.dtype == np.float32 and a.ndim == 2 and a.shape[0] == pl.P
        assert a.flags["C_CONTIGUOUS"] and a.shape[1] >= pl.total_shard_len
        assert stride is None or stride == a.shape[1]
        stride = a.shape[1]
    return int(stride)


def _buckets(pl: OraclePlan, bucket: int, forward: bool) -> List[int]:
    if bucket >= 0:
        return [bucket]
    order = list(range(pl.n_buckets))
    return order[::-1] if forward else order


def reduce_scatter(pl: OraclePlan, bucket: int, grads: Sequence[Sequence[np.ndarray]],
                   shard_grad: np.ndarray, shards: Optional[range] = None) -> None:
    """grads[p][l]: worker p's gradient of layer l (float32, or uint16 = bf16 bits).
    bucket = -1: every bucket.  `shards` limits the shards computed."""
    lib = _load()
    stride = _check_rows(pl, shard_grad)
    want = np.float32 if pl.grad_elem_bytes == 4 else np.uint16
    todo = _buckets(pl, bucket, forward=False)
    s0, s1 = (0, pl.P) if shards is None else (shards.start, shards.stop)
    needed = [l for b in todo for l in _layers_of_shards(pl, b, s0, s1)]
    tab = _ptr_table(pl, grads, needed, want)
    for b in todo:
        lib.oracle_reduce_scatter(
            _p(pl.sizes, C.c_int64), C.c_int32(pl.L), C.c_int32(pl.P), C.c_int32(pl.grad_elem_bytes),
            _p(pl.layer_offset, C.c_int64),
            C.c_int32(int(pl.bucket_first_layer[b])), C.c_int32(int(pl.bucket_n_layers[b])),
            C.c_int64(int(pl.bucket_len[b])), C.c_int64(int(pl.bucket_shard_len[b])),
            C.c_int64(int(pl.bucket_shard_base[b])),
            tab, _p(shard_grad, C.c_float), C.c_int64(stride), C.c_int32(s0), C.c_int32(s1))


def shard_update(pl: OraclePlan, bucket: int, shard_grad: np.ndarray, shard_param: np.ndarray,
                 shard_mom: np.ndarray, lr: float, momentum: float,
                 shards: Optional[range] = None) -> None:
    lib = _load()
    stride = _check_rows(pl, shard_grad, shard_param, shard_mom)
    s0, s1 = (0, pl.P) if shards is None else (shards.start, shards.stop)
    for b in _buckets(pl, bucket, forward=False):
        lib.oracle_shard_update(
            C.c_int32(pl.P), C.c_int64(int(pl.bucket_shard_len[b])),
            C.c_int64(int(pl.bucket_shard_base[b])), C.c_int64(stride),
            _p(shard_grad, C.c_float), _p(shard_param, C.c_float), _p(shard_mom, C.c_float),
            C.c_float(lr), C.c_float(momentum), C.c_int32(s0), C.c_int32(s1))


def all_gather(pl: OraclePlan, bucket: int, shard_param: np.ndarray,
               params: Sequence[Sequence[np.ndarray]], workers: Optional[range] = None) -> None:
    """params[p][l]: worker p's parameter tensor of layer l (float32), overwritten."""
    lib = _load()
    stride = _check_rows(pl, shard_param)
    todo = _buckets(pl, bucket, forward=True)
    p0, p1 = (0, pl.P) if workers is None else (workers.start, workers.stop)
    tab = _ptr_table(pl, params, _bucket_layers(pl, todo), np.float32, range(p0, p1))
    for b in todo:
        lib.oracle_all_gather(
            _p(pl.sizes, C.c_int64), C.c_int32(pl.L), C.c_int32(pl.P), _p(pl.layer_offset, C.c_int64),
            C.c_int32(int(pl.bucket_first_layer[b])), C.c_int32(int(pl.bucket_n_layers[b])),
            C.c_int64(int(pl.bucket_shard_len[b])), C.c_int64(int(pl.bucket_shard_base[b])),
            _p(shard_param, C.c_float), C.c_int64(stride), tab, C.c_int32(p0), C.c_int32(p1))


def scatter_params(pl: OraclePlan, params: Sequence[Sequence[np.ndarray]], worker: int,
                   shard_param: np.ndarray, bucket: int = -1) -> None:
    """Seed the parameter shards (every bucket, or one) from worker `worker`'s full tensors."""
    lib = _load()
    stride = _check_rows(pl, shard_param)
    todo = _buckets(pl, bucket, forward=False)
    tab = _ptr_table(pl, params, _bucket_layers(pl, todo), np.float32, range(worker, worker + 1))
    for b in todo:
        lib.oracle_scatter_params(
            _p(pl.sizes, C.c_int64), C.c_int32(pl.L), C.c_int32(pl.P), _p(pl.layer_offset, C.c_int64),
            C.c_int32(int(pl.bucket_first_layer[b])), C.c_int32(int(pl.bucket_n_layers[b])),
            C.c_int64(int(pl.bucket_len[b])), C.c_int64(int(pl.bucket_shard_len[b])),
            C.c_int64(int(pl.bucket_shard_base[b])),
            tab, C.c_int32(worker), _p(shard_param, C.c_float), C.c_int64(stride))
