"""MI355X-native gradient-aggregation path of DeAR (decoupled all-reduce with tensor fusion).

The product is libdear.so (C ABI in include/dear.h, HIP kernels for gfx950); this package
is its thin ctypes binding.  Importing the package does not load the library; the first
call does, and raises if the library has not been built.
"""
from .binding import (  # noqa: F401
    DEAR_BF16, DEAR_F32, DEAR_NO_LIMIT, DEAR_SHARD_ALIGN, Context, DearError, Plan,
    dear_all_gather, dear_all_gather_workers, dear_ctx_create, dear_ctx_set_max_workgroups, dear_ctx_set_wave_priority,
    dear_plan, dear_plan_fixed_layers, dear_plan_tiles,
    dear_reduce_scatter, dear_reduce_scatter_static, dear_reduce_scatter_update,
    dear_scatter_params, dear_shard_update, dear_update_all_gather, dear_version, load_library, strerror,
)
