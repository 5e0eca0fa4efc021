"""Device-memory plumbing for the one-GPU emulation of P data-parallel workers.

Allocates, with torch, what a caller of libdear owns: P replicas of per-layer gradient
and parameter tensors and the three shard buffers, and binds them to a context.  Every
step of the path itself runs in the library's kernels; nothing here computes.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import torch

from . import binding as B


def _stream_handle(stream: Optional["torch.cuda.Stream"]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


class EmulatedWorkers:
    """P workers' tensors on one GPU plus a libdear context over them.

    layout "flat": each replica is one allocation, layers start on 256-byte boundaries.
    layout "separate": every layer tensor of every replica is its own allocation.
    """

    LAYER_ALIGN_BYTES = 256

    def __init__(self, sizes: Sequence[int], P: int, grad_dtype: str, threshold_bytes: int,
                 device: str = "cuda:0", layout: str = "flat", plan: Optional[B.Plan] = None):
        if not torch.cuda.is_available():
            raise RuntimeError("EmulatedWorkers needs a GPU; there is no CPU path")
        B.load_library()
        self.sizes = list(sizes)
        self.P = P
        self.grad_dtype = grad_dtype
        self.device = torch.device(device)
        tg = torch.float32 if grad_dtype == "f32" else torch.bfloat16
        g = 4 if grad_dtype == "f32" else 2
        self.plan = plan if plan is not None else B.dear_plan(self.sizes, P, threshold_bytes, g)
        if self.plan.grad_elem_bytes != g or self.plan.P != P or self.plan.layer_sizes != self.sizes:
            raise ValueError("plan does not match the workers")

        self.grads: List[List[torch.Tensor]] = []
        self.params: List[List[torch.Tensor]] = []
        self._keep = []
        for _ in range(P):
            self.grads.append(self._alloc_layers(tg, g, layout))
            self.params.append(self._alloc_layers(torch.float32, 4, layout))

        row = self.plan.total_shard_len
        self.shard_grad = torch.zeros(P, row, dtype=torch.float32, device=self.device)
        self.shard_param = torch.zeros(P, row, dtype=torch.float32, device=self.device)
        self.shard_mom = torch.zeros(P, row, dtype=torch.float32, device=self.device)

        gp = [t.data_ptr() for rep in self.grads for t in rep]
        wp = [t.data_ptr() for rep in self.params for t in rep]
        with torch.cuda.device(self.device):
            self.ctx = B.dear_ctx_create(self.plan, B.DEAR_F32 if g == 4 else B.DEAR_BF16, gp, wp)

    def _alloc_layers(self, dtype, elem_bytes: int, layout: str) -> List[torch.Tensor]:
        if layout == "separate":
            return [torch.zeros(n, dtype=dtype, device=self.device) for n in self.sizes]
        if layout != "flat":
            raise ValueError(layout)
        a = self.LAYER_ALIGN_BYTES // elem_bytes
        starts, pos = [], 0
        for n in self.sizes:
            starts.append(pos)
            pos = (pos + n + a - 1) // a * a
        buf = torch.zeros(max(pos, 1), dtype=dtype, device=self.device)
        self._keep.append(buf)
        return [buf[s:s + n] for s, n in zip(starts, self.sizes)]

    # ------------------------------------------------------------------ data movement (plumbing)
    def load_dense(self, dst_layers: List[torch.Tensor], dense: torch.Tensor) -> None:
        """Copy a dense concatenation of all layers into one replica's layer tensors."""
        pos = 0
        for t in dst_layers:
            t.copy_(dense[pos:pos + t.numel()])
            pos += t.numel()

    def dense(self, layers: List[torch.Tensor]) -> torch.Tensor:
        return torch.cat([t.reshape(-1) for t in layers])

    # ------------------------------------------------------------------ the path
    def scatter_params(self, worker: int = 0, stream=None) -> None:
        B.dear_scatter_params(self.ctx, worker, self.shard_param.data_ptr(), _stream_handle(stream))

    def reduce_scatter(self, bucket: int = -1, stream=None) -> None:
        B.dear_reduce_scatter(self.ctx, bucket, self.shard_grad.data_ptr(), _stream_handle(stream))

    def reduce_scatter_update(self, bucket: int, lr: float, momentum: float, stream=None) -> None:
        B.dear_reduce_scatter_update(self.ctx, bucket, self.shard_param.data_ptr(), self.shard_mom.data_ptr(),
                                     lr, momentum, _stream_handle(stream))

    def shard_update(self, bucket: int, lr: float, momentum: float, stream=None) -> None:
        B.dear_shard_update(self.ctx, bucket, self.shard_grad.data_ptr(), self.shard_param.data_ptr(),
                            self.shard_mom.data_ptr(), lr, momentum, _stream_handle(stream))

    def all_gather(self, bucket: int = -1, stream=None) -> None:
        B.dear_all_gather(self.ctx, bucket, self.shard_param.data_ptr(), _stream_handle(stream))

    def update_all_gather(self, bucket: int, lr: float, momentum: float, stream=None) -> None:
        B.dear_update_all_gather(self.ctx, bucket, self.shard_grad.data_ptr(), self.shard_param.data_ptr(),
                                 self.shard_mom.data_ptr(), lr, momentum, _stream_handle(stream))

    def iteration(self, lr: float, momentum: float, per_bucket: bool = True, stream=None,
                  fused_update: bool = False, fused_gather: bool = False) -> None:
        """One pass of the whole path on one stream: reduce-scatter the buckets in the order
        their gradients become ready, update the owned shards, all-gather in forward order.
        fused_update: reduce-scatter and update of a bucket in one kernel.
        fused_gather: update and all-gather of a bucket in one kernel."""
        buckets = list(range(self.plan.n_buckets)) if per_bucket else [-1]
        if fused_gather:
            for b in buckets:
                self.reduce_scatter(b, stream)
            for b in reversed(buckets):
                self.update_all_gather(b, lr, momentum, stream)
            return
        if fused_update:
            for b in buckets:
                self.reduce_scatter_update(b, lr, momentum, stream)
        else:
            for b in buckets:
                self.reduce_scatter(b, stream)
            for b in buckets:
                self.shard_update(b, lr, momentum, stream)
        for b in reversed(buckets):
            self.all_gather(b, stream)

    def replan(self, threshold_bytes: Optional[int] = None, plan: Optional[B.Plan] = None, stream=None) -> None:
        """Switch to another bucket plan over the same tensors, carrying the optimizer state
        over: parameters and momentum are re-sharded for the new plan with library calls only.
        Expects the state after an all-gather (every replica holds the current parameters)."""
        g = self.plan.grad_elem_bytes
        new_plan = plan if plan is not None else B.dear_plan(self.sizes, self.P, threshold_bytes, g)
        gp = [t.data_ptr() for rep in self.grads for t in rep]
        wp = [t.data_ptr() for rep in self.params for t in rep]
        with torch.cuda.device(self.device):
            new_ctx = B.dear_ctx_create(new_plan, B.DEAR_F32 if g == 4 else B.DEAR_BF16, gp, wp)
        row = new_plan.total_shard_len
        new_param = torch.zeros(self.P, row, dtype=torch.float32, device=self.device)
        new_mom = torch.zeros(self.P, row, dtype=torch.float32, device=self.device)
        new_grad = torch.zeros(self.P, row, dtype=torch.float32, device=self.device)
        h = _stream_handle(stream)
        # w: worker 0's tensors -> new shards
        B.dear_scatter_params(new_ctx, 0, new_param.data_ptr(), h)
        # v: old shards -> worker 0's tensors (borrowed) -> new shards
        B.dear_all_gather_workers(self.ctx, -1, self.shard_mom.data_ptr(), 0, 1, h)
        B.dear_scatter_params(new_ctx, 0, new_mom.data_ptr(), h)
        # give worker 0 its parameters back
        B.dear_all_gather_workers(new_ctx, -1, new_param.data_ptr(), 0, 1, h)
        s = stream if stream is not None else torch.cuda.current_stream()
        s.synchronize()  # the old context and buffers are released below
        self.ctx.destroy()
        self.ctx, self.plan = new_ctx, new_plan
        B.dear_ctx_set_max_workgroups(self.ctx, getattr(self, "max_workgroups", 0))
        B.dear_ctx_set_wave_priority(self.ctx, getattr(self, "wave_priority", 0))
        self.shard_grad, self.shard_param, self.shard_mom = new_grad, new_param, new_mom

    def capture_iteration(self, lr: float, momentum: float, per_bucket: bool = True,
                          fused_update: bool = False) -> "torch.cuda.CUDAGraph":
        """Record one iteration (all its launches) into a HIP graph and return it; replay()
        then runs the iteration with one submission, which matters when the step is
        launch-bound (many small buckets).  Nothing is executed by the capture itself.  The
        library's launches contain no memset nodes and allocate nothing, so they are safe to
        capture; the graph is bound to this context's tensors and launch width."""
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream(device=self.device)
        side.wait_stream(torch.cuda.current_stream(self.device))
        with torch.cuda.graph(graph, stream=side):
            self.iteration(lr, momentum, per_bucket=per_bucket, fused_update=fused_update)
        return graph

    def set_max_workgroups(self, n: int) -> None:
        """0: one workgroup per work item (default); n > 0: bounded grid for running beside compute."""
        self.max_workgroups = n
        B.dear_ctx_set_max_workgroups(self.ctx, n)

    def set_wave_priority(self, priority: int) -> None:
        """Wave priority (0..3) of bounded-grid launches."""
        self.wave_priority = priority
        B.dear_ctx_set_wave_priority(self.ctx, priority)

    def close(self) -> None:
        self.ctx.destroy()
