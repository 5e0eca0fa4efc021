"""DistOptim: the paper's distributed optimizer (Section V) over libdear, for P model
replicas that live on one GPU.

The paper wraps a torch optimizer and drives communication from autograd hooks
(Section V-A): a gradient that becomes ready is pushed to the tensor-fusion controller;
when a whole group is ready its reduce-scatter is issued (BackPipe, Section III-B); the
all-gathers are issued in forward order and a layer's forward computation waits for the
all-gather of its group (FeedPipe).  Users call synchronize() before reading parameters
(Section V-B).

Here the P "workers" are P copies of a torch module in one process.  Their .grad and
.data tensors are handed to libdear as they are (no staging copy): hooks only count
arrivals, record events and launch the library's kernels on a communication stream.

    models = [copy.deepcopy(model).cuda() for _ in range(P)]
    optim = DistOptim(models, lr=0.1, momentum=0.9, fusion_threshold_bytes=25 << 20)
    for batch in loader:                       # batch split into P equal shards
        for p, m in enumerate(models):
            loss_fn(m(x[p]), y[p]).backward()  # reduce-scatter + update start inside backward
        optim.step()                           # queues the all-gathers; next forward waits per layer
    optim.synchronize()
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import torch

from . import binding as B


class DistOptim:
    def __init__(self, models: Sequence[torch.nn.Module], lr: float, momentum: float,
                 fusion_threshold_bytes: int = 25 << 20, fused_update: bool = True):
        if not models:
            raise ValueError("need at least one replica")
        self.models = list(models)
        self.P = len(self.models)
        self.lr, self.momentum, self.fused_update = lr, momentum, fused_update
        per_model = [[p for p in m.parameters() if p.requires_grad] for m in self.models]
        self.params = per_model
        sizes = [p.numel() for p in per_model[0]]
        for plist in per_model:
            if [p.numel() for p in plist] != sizes:
                raise ValueError("replicas differ in their parameter lists")
            for p in plist:
                if p.dtype != torch.float32 or not p.is_cuda or not p.is_contiguous():
                    raise ValueError("parameters must be contiguous fp32 CUDA tensors")
                p.grad = torch.zeros_like(p)          # fixed gradient storage for the library
        self.device = per_model[0][0].device
        self.plan = B.dear_plan(sizes, self.P, fusion_threshold_bytes, 4)
        self._grad_ptrs = [p.grad.data_ptr() for plist in per_model for p in plist]
        param_ptrs = [p.data_ptr() for plist in per_model for p in plist]
        with torch.cuda.device(self.device):
            self.ctx = B.dear_ctx_create(self.plan, B.DEAR_F32, self._grad_ptrs, param_ptrs)
        row = self.plan.total_shard_len
        self.shard_grad = torch.zeros(self.P, row, dtype=torch.float32, device=self.device)
        self.shard_param = torch.zeros(self.P, row, dtype=torch.float32, device=self.device)
        self.shard_mom = torch.zeros(self.P, row, dtype=torch.float32, device=self.device)
        self.comm = torch.cuda.Stream(device=self.device)
        B.dear_scatter_params(self.ctx, 0, self.shard_param.data_ptr(), torch.cuda.current_stream().cuda_stream)
        self.comm.wait_stream(torch.cuda.current_stream())

        nb = self.plan.n_buckets
        self._arrived = [0] * nb
        self._need = [self.plan.bucket_n_layers[b] * self.P for b in range(nb)]
        self._launched = [False] * nb
        self._ag_done: List[torch.cuda.Event] = [torch.cuda.Event() for _ in range(nb)]
        self._have_ag = False
        self._hooks = []
        for plist in per_model:
            for l, p in enumerate(plist):
                b = self.plan.layer_bucket[l]
                self._hooks.append(p.register_post_accumulate_grad_hook(self._make_grad_hook(b)))
        # FeedPipe: a module's forward waits for the all-gather of the groups its parameters are in
        index_of: Dict[int, int] = {}
        for plist in per_model:
            for l, p in enumerate(plist):
                index_of[id(p)] = l
        for m in self.models:
            for sub in m.modules():
                own = [index_of[id(p)] for p in sub.parameters(recurse=False) if id(p) in index_of]
                if own:
                    buckets = sorted({self.plan.layer_bucket[l] for l in own})
                    self._hooks.append(sub.register_forward_pre_hook(self._make_forward_hook(buckets)))

    # ------------------------------------------------------------------ hooks
    def _make_grad_hook(self, b: int):
        def hook(_param):
            self._arrived[b] += 1
            if self._arrived[b] == self._need[b]:
                self._reduce_scatter(b)
        return hook

    def _make_forward_hook(self, buckets: List[int]):
        def hook(_module, _inputs):
            if self._have_ag:
                cur = torch.cuda.current_stream()
                for b in buckets:
                    cur.wait_event(self._ag_done[b])
        return hook

    def _reduce_scatter(self, b: int) -> None:
        """BackPipe: the group's gradients of all workers are ready on the current stream."""
        ready = torch.cuda.Event()
        ready.record(torch.cuda.current_stream())
        self.comm.wait_event(ready)
        h = self.comm.cuda_stream
        if self.fused_update:
            B.dear_reduce_scatter_update(self.ctx, b, self.shard_param.data_ptr(), self.shard_mom.data_ptr(),
                                         self.lr, self.momentum, h)
        else:
            B.dear_reduce_scatter(self.ctx, b, self.shard_grad.data_ptr(), h)
            B.dear_shard_update(self.ctx, b, self.shard_grad.data_ptr(), self.shard_param.data_ptr(),
                                self.shard_mom.data_ptr(), self.lr, self.momentum, h)
        self._launched[b] = True

    # ------------------------------------------------------------------ user calls
    def step(self) -> None:
        """End of the backward passes of all replicas: every group must have been reduced;
        queue the all-gathers in forward order and clear the gradients for the next iteration."""
        nb = self.plan.n_buckets
        missing = [b for b in range(nb) if not self._launched[b]]
        if missing:
            raise RuntimeError("gradients of groups %s did not arrive on all %d replicas" % (missing, self.P))
        got = [p.grad.data_ptr() for plist in self.params for p in plist]
        if got != self._grad_ptrs:
            raise RuntimeError("a .grad tensor was replaced; keep gradients in place (set_to_none=False)")
        h = self.comm.cuda_stream
        rs_done = torch.cuda.Event()       # all reduce-scatters are queued: they precede every all-gather
        rs_done.record(self.comm)
        for b in reversed(range(nb)):
            B.dear_all_gather(self.ctx, b, self.shard_param.data_ptr(), h)
            self._ag_done[b].record(self.comm)
        self._have_ag = True
        # gradients may be cleared only after the reduce-scatters that read them
        torch.cuda.current_stream().wait_event(rs_done)
        for plist in self.params:
            for p in plist:
                p.grad.zero_()
        self._arrived = [0] * nb
        self._launched = [False] * nb

    def synchronize(self) -> None:
        """Wait for outstanding all-gathers (before evaluation or checkpointing)."""
        self.comm.synchronize()

    def close(self) -> None:
        for h in self._hooks:
            h.remove()
        self._hooks = []
        self.ctx.destroy()
