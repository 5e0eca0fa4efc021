"""ctypes binding of libdear.so: argument marshalling only.

Function names and argument order follow include/dear.h.  Device buffers are passed as
integer addresses (e.g. torch.Tensor.data_ptr()); streams as the integer hipStream_t
(e.g. torch.cuda.current_stream().cuda_stream).  Any non-zero status raises DearError.
There is no CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdear.so")

DEAR_OK, DEAR_EINVAL, DEAR_ENOMEM, DEAR_EHIP, DEAR_ERANGE, DEAR_EALIGN, DEAR_ETOOBIG = 0, -1, -2, -3, -4, -5, -6
DEAR_STATIC_MAX_POINTERS, DEAR_STATIC_MAX_TILES = 131072, 98304
DEAR_F32, DEAR_BF16 = 0, 1
DEAR_NO_LIMIT = (1 << 63) - 1
DEAR_SHARD_ALIGN = 32

EXPORTS = [
    "dear_plan", "dear_plan_fixed_layers", "dear_plan_free", "dear_plan_view", "dear_plan_tiles",
    "dear_ctx_create", "dear_ctx_destroy", "dear_ctx_set_max_workgroups", "dear_ctx_set_wave_priority",
    "dear_reduce_scatter", "dear_reduce_scatter_static", "dear_reduce_scatter_update", "dear_shard_update", "dear_all_gather",
    "dear_all_gather_workers", "dear_update_all_gather", "dear_scatter_params", "dear_strerror", "dear_version",
]


class DearError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, strerror(status), status))


class _PlanView(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("n_buckets", C.c_int32), ("P", C.c_int32),
        ("grad_elem_bytes", C.c_int32), ("shard_align", C.c_int32), ("reserved", C.c_int32),
        ("threshold_bytes", C.c_int64), ("total_elems", C.c_int64), ("total_shard_len", C.c_int64),
        ("layer_sizes", C.POINTER(C.c_int64)), ("layer_bucket", C.POINTER(C.c_int32)),
        ("layer_offset", C.POINTER(C.c_int64)), ("bucket_first_layer", C.POINTER(C.c_int32)),
        ("bucket_n_layers", C.POINTER(C.c_int32)), ("bucket_len", C.POINTER(C.c_int64)),
        ("bucket_shard_len", C.POINTER(C.c_int64)), ("bucket_shard_base", C.POINTER(C.c_int64)),
    ]


class Tile(C.Structure):
    _fields_ = [("src_begin", C.c_int64), ("dst_begin", C.c_int64), ("count", C.c_int32),
                ("layer", C.c_int32), ("shard", C.c_int32), ("bucket", C.c_int32)]


DEAR_TILE_ELEMS = 4096

_lib = None


def load_library() -> C.CDLL:
    """Load libdear.so from the package directory; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libdear.so is not built: run `python -m paper_2302_12445_amd.build` "
                          "(there is no CPU fallback)")
    # The device memory and streams handed to the library come from torch, so both must
    # use ONE HIP runtime.  torch ships its own copy; loading it first makes libdear's
    # dependency on libamdhip64.so.7 resolve to that copy instead of a second runtime.
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    lib.dear_plan.argtypes = [C.POINTER(i64), i32, i32, i64, i32, C.POINTER(vp)]
    lib.dear_plan_fixed_layers.argtypes = [C.POINTER(i64), i32, i32, i32, i32, C.POINTER(vp)]
    lib.dear_plan_free.argtypes = [vp]
    lib.dear_plan_free.restype = None
    lib.dear_plan_view.argtypes = [vp, C.POINTER(_PlanView)]
    lib.dear_plan_tiles.argtypes = [vp, C.POINTER(Tile), i64, C.POINTER(i64), C.POINTER(i64)]
    lib.dear_ctx_create.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp)]
    lib.dear_ctx_set_max_workgroups.argtypes = [vp, i32]
    lib.dear_ctx_set_max_workgroups.restype = C.c_int
    lib.dear_ctx_set_wave_priority.argtypes = [vp, i32]
    lib.dear_ctx_set_wave_priority.restype = C.c_int
    lib.dear_ctx_destroy.argtypes = [vp]
    lib.dear_ctx_destroy.restype = None
    lib.dear_reduce_scatter.argtypes = [vp, i32, vp, vp]
    lib.dear_reduce_scatter_static.argtypes = [vp, i32, C.POINTER(vp), i32, vp, vp]
    lib.dear_shard_update.argtypes = [vp, i32, vp, vp, vp, f32, f32, vp]
    lib.dear_reduce_scatter_update.argtypes = [vp, i32, vp, vp, f32, f32, vp]
    lib.dear_all_gather.argtypes = [vp, i32, vp, vp]
    lib.dear_update_all_gather.argtypes = [vp, i32, vp, vp, vp, f32, f32, vp]
    lib.dear_all_gather_workers.argtypes = [vp, i32, vp, i32, i32, vp]
    lib.dear_scatter_params.argtypes = [vp, i32, vp, vp]
    lib.dear_strerror.argtypes = [C.c_int]
    lib.dear_strerror.restype = C.c_char_p
    lib.dear_version.restype = C.c_int
    for name in ("dear_plan", "dear_plan_fixed_layers", "dear_plan_view", "dear_plan_tiles", "dear_ctx_create",
                 "dear_reduce_scatter", "dear_reduce_scatter_static", "dear_reduce_scatter_update", "dear_shard_update", "dear_all_gather",
                 "dear_all_gather_workers", "dear_update_all_gather", "dear_scatter_params"):
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load_library().dear_strerror(status).decode()


def _check(status: int, where: str) -> None:
    if status != DEAR_OK:
        raise DearError(status, where)


class Plan:
    """Owner of a dear_plan_t; attributes mirror dear_plan_view_t as Python lists."""

    def __init__(self, handle: int):
        self._h = C.c_void_p(handle)
        v = _PlanView()
        _check(load_library().dear_plan_view(self._h, C.byref(v)), "dear_plan_view")
        L, B = v.n_layers, v.n_buckets
        self.n_layers, self.n_buckets, self.P = L, B, v.P
        self.grad_elem_bytes, self.shard_align = v.grad_elem_bytes, v.shard_align
        self.threshold_bytes, self.total_elems = v.threshold_bytes, v.total_elems
        self.total_shard_len = v.total_shard_len
        self.layer_sizes = [v.layer_sizes[i] for i in range(L)]
        self.layer_bucket = [v.layer_bucket[i] for i in range(L)]
        self.layer_offset = [v.layer_offset[i] for i in range(L)]
        self.bucket_first_layer = [v.bucket_first_layer[i] for i in range(B)]
        self.bucket_n_layers = [v.bucket_n_layers[i] for i in range(B)]
        self.bucket_len = [v.bucket_len[i] for i in range(B)]
        self.bucket_shard_len = [v.bucket_shard_len[i] for i in range(B)]
        self.bucket_shard_base = [v.bucket_shard_base[i] for i in range(B)]

    @property
    def handle(self) -> C.c_void_p:
        if self._h is None:
            raise ValueError("plan already freed")
        return self._h

    def free(self) -> None:
        if self._h is not None:
            load_library().dear_plan_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def dear_plan(layer_sizes: Sequence[int], P: int, fusion_threshold_bytes: int,
              grad_elem_bytes: int = 4) -> Plan:
    lib = load_library()
    n = len(layer_sizes)
    arr = (C.c_int64 * max(n, 1))(*layer_sizes)
    out = C.c_void_p()
    _check(lib.dear_plan(arr, n, P, fusion_threshold_bytes, grad_elem_bytes, C.byref(out)), "dear_plan")
    return Plan(out.value)


def dear_plan_fixed_layers(layer_sizes: Sequence[int], P: int, layers_per_bucket: int,
                           grad_elem_bytes: int = 4) -> Plan:
    lib = load_library()
    n = len(layer_sizes)
    arr = (C.c_int64 * max(n, 1))(*layer_sizes)
    out = C.c_void_p()
    _check(lib.dear_plan_fixed_layers(arr, n, P, layers_per_bucket, grad_elem_bytes, C.byref(out)),
           "dear_plan_fixed_layers")
    return Plan(out.value)


def dear_plan_tiles(plan: Plan):
    """Returns (tiles, bucket_tile_begin): the plan's tile table as a ctypes array of Tile
    and the list of n_buckets+1 range starts."""
    lib = load_library()
    n = C.c_int64()
    _check(lib.dear_plan_tiles(plan.handle, None, 0, C.byref(n), None), "dear_plan_tiles")
    tiles = (Tile * max(n.value, 1))()
    begin = (C.c_int64 * (plan.n_buckets + 1))()
    _check(lib.dear_plan_tiles(plan.handle, tiles, n.value, C.byref(n), begin), "dear_plan_tiles")
    return tiles, list(begin)


class Context:
    """Owner of a dear_ctx_t."""

    def __init__(self, handle: int, plan: Plan):
        self._h = C.c_void_p(handle)
        self.plan = plan

    @property
    def handle(self) -> C.c_void_p:
        if self._h is None:
            raise ValueError("context already destroyed")
        return self._h

    def destroy(self) -> None:
        if self._h is not None:
            load_library().dear_ctx_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def dear_ctx_create(plan: Plan, grad_dtype: int, grad_ptrs: Sequence[int],
                    param_ptrs: Sequence[int]) -> Context:
    """grad_ptrs / param_ptrs: flat sequences of P*L device addresses, index p*L + l."""
    lib = load_library()
    n = plan.P * plan.n_layers
    if len(grad_ptrs) != n or len(param_ptrs) != n:
        raise ValueError("expected %d pointers, got %d / %d" % (n, len(grad_ptrs), len(param_ptrs)))
    g = (C.c_void_p * n)(*grad_ptrs)
    w = (C.c_void_p * n)(*param_ptrs)
    out = C.c_void_p()
    _check(lib.dear_ctx_create(plan.handle, grad_dtype, g, w, C.byref(out)), "dear_ctx_create")
    return Context(out.value, plan)


def dear_ctx_set_max_workgroups(ctx: Context, max_workgroups: int) -> None:
    _check(load_library().dear_ctx_set_max_workgroups(ctx.handle, max_workgroups), "dear_ctx_set_max_workgroups")


def dear_ctx_set_wave_priority(ctx: Context, priority: int) -> None:
    _check(load_library().dear_ctx_set_wave_priority(ctx.handle, priority), "dear_ctx_set_wave_priority")


def _stream(s: Optional[int]) -> C.c_void_p:
    return C.c_void_p(s or 0)


def dear_reduce_scatter(ctx: Context, bucket: int, shard_grad: int, stream: Optional[int] = None) -> None:
    _check(load_library().dear_reduce_scatter(ctx.handle, bucket, C.c_void_p(shard_grad), _stream(stream)),
           "dear_reduce_scatter")


def dear_reduce_scatter_static(plan: Plan, grad_dtype: int, grad_ptrs: Sequence[int], bucket: int,
                               shard_grad: int, stream: Optional[int] = None) -> None:
    """dear_reduce_scatter without a context and without any allocation (see dear.h)."""
    n = plan.P * plan.n_layers
    if len(grad_ptrs) != n:
        raise ValueError("expected %d pointers, got %d" % (n, len(grad_ptrs)))
    g = (C.c_void_p * n)(*grad_ptrs)
    _check(load_library().dear_reduce_scatter_static(plan.handle, grad_dtype, g, bucket, C.c_void_p(shard_grad),
                                                     _stream(stream)), "dear_reduce_scatter_static")


def dear_shard_update(ctx: Context, bucket: int, shard_grad: int, shard_param: int, shard_mom: int,
                      lr: float, momentum: float, stream: Optional[int] = None) -> None:
    _check(load_library().dear_shard_update(ctx.handle, bucket, C.c_void_p(shard_grad),
                                            C.c_void_p(shard_param), C.c_void_p(shard_mom),
                                            lr, momentum, _stream(stream)), "dear_shard_update")


def dear_reduce_scatter_update(ctx: Context, bucket: int, shard_param: int, shard_mom: int,
                               lr: float, momentum: float, stream: Optional[int] = None) -> None:
    _check(load_library().dear_reduce_scatter_update(ctx.handle, bucket, C.c_void_p(shard_param),
                                                     C.c_void_p(shard_mom), lr, momentum, _stream(stream)),
           "dear_reduce_scatter_update")


def dear_all_gather(ctx: Context, bucket: int, shard_param: int, stream: Optional[int] = None) -> None:
    _check(load_library().dear_all_gather(ctx.handle, bucket, C.c_void_p(shard_param), _stream(stream)),
           "dear_all_gather")


def dear_update_all_gather(ctx: Context, bucket: int, shard_grad: int, shard_param: int, shard_mom: int,
                           lr: float, momentum: float, stream: Optional[int] = None) -> None:
    _check(load_library().dear_update_all_gather(ctx.handle, bucket, C.c_void_p(shard_grad),
                                                 C.c_void_p(shard_param), C.c_void_p(shard_mom),
                                                 lr, momentum, _stream(stream)), "dear_update_all_gather")


def dear_all_gather_workers(ctx: Context, bucket: int, shard_param: int, first_worker: int, n_workers: int,
                            stream: Optional[int] = None) -> None:
    _check(load_library().dear_all_gather_workers(ctx.handle, bucket, C.c_void_p(shard_param), first_worker,
                                                  n_workers, _stream(stream)), "dear_all_gather_workers")


def dear_scatter_params(ctx: Context, worker: int, shard_param: int, stream: Optional[int] = None) -> None:
    _check(load_library().dear_scatter_params(ctx.handle, worker, C.c_void_p(shard_param), _stream(stream)),
           "dear_scatter_params")


def dear_version() -> int:
    return load_library().dear_version()
