"""The DeAR schedule on one GPU: BackPipe and FeedPipe over two HIP streams.

Paper Section III-B: the first half of every group's all-reduce (reduce-scatter, OP1)
starts as soon as the group's gradients are ready in the backward pass (BackPipe); all
OP1 are complete before any second half starts; the second half (all-gather, OP2) of a
group must complete before that group's feed-forward computation in the next iteration,
and OP2 are issued in forward order (FeedPipe).  Communication is issued in the same
order on every worker, last layer first in the backward pass and the reverse in the
forward pass, so no negotiation is needed.

Here the "network" is libdear's kernels on a communication stream and the model's
computation is a stream of synthetic GEMMs on a compute stream (forward: ff_gemms per
bucket, backward: bp_gemms per bucket; back-propagation costs about twice the forward
pass, Section VI-F).  Ordering between the two streams is by HIP events only.  The shard
update runs on the communication stream directly after the bucket's reduce-scatter.

This module is stream/event plumbing: every aggregation step runs in the library.
"""
from __future__ import annotations

import time
from typing import Callable, Dict, List, Optional, Sequence, Union

import torch

from .emulation import EmulatedWorkers


def spread_gemms(total: int, plan) -> List[int]:
    """Split `total` GEMMs of synthetic compute over the plan's buckets in proportion to the
    number of layers each bucket holds, with the remainders carried along, so that the sum is
    `total` for every plan: the model's compute does not change when its gradients are
    grouped differently (a bucket with few layers may get none)."""
    out, seen = [], 0
    L = plan.n_layers
    for b in range(plan.n_buckets):
        lo = total * seen // L
        seen += plan.bucket_n_layers[b]
        out.append(total * seen // L - lo)
    return out


def streams_run_concurrently(busy: torch.cuda.Stream, other: torch.cuda.Stream, work: Callable[[], None],
                             probe: torch.Tensor) -> bool:
    """True if a kernel queued on `other` completes while `busy` is still working.  HIP maps
    its streams onto a few hardware queues; two streams that land on the same queue run
    strictly one after the other, and a schedule built on them cannot overlap anything."""
    torch.cuda.synchronize()
    with torch.cuda.stream(busy):
        for _ in range(4):
            work()
        busy_done = torch.cuda.Event()
        busy_done.record(busy)
    with torch.cuda.stream(other):
        probe.zero_()
        other_done = torch.cuda.Event()
        other_done.record(other)
    other_done.synchronize()
    concurrent = not busy_done.query()
    busy.synchronize()
    return concurrent


class DearSchedule:
    MODES = ("dear", "wfbp", "serial", "compute_only", "comm_only")

    def __init__(self, em: EmulatedWorkers, lr: float, momentum: float, gemm_dim: int = 4096,
                 ff_gemms: Union[int, Sequence[int]] = 1, bp_gemms: Union[int, Sequence[int]] = 2,
                 on_backward: Optional[Callable[[int, int], None]] = None,
                 overlap_workgroups: int = 256, overlap_workgroups_ag: Optional[int] = 256,
                 fused_update: bool = True, gemm_dtype: torch.dtype = torch.float32,
                 full_width_when_alone: bool = True,
                 wave_priority: int = 3, wave_priority_ag: Optional[int] = 0,
                 compute_stream: Optional[torch.cuda.Stream] = None,
                 comm_stream: Optional[torch.cuda.Stream] = None):
        """on_backward(iteration, bucket) runs on the compute stream behind the bucket's
        backward GEMMs; tests use it to write that bucket's fresh gradients.
        overlap_workgroups bounds the grid of the aggregation kernels in the overlapping
        modes (dear, wfbp); 0 leaves them unbounded.  overlap_workgroups_ag, if given, is
        the bound for the all-gather (the forward pass it hides under is half as long as
        the backward pass).  The defaults are what hid most on an MI355X beside fp32 4096^3
        GEMMs: 256 workgroups for both, reduce-scatter at wave priority 3 (it has many
        instructions per byte and little slack under two GEMMs), all-gather at priority 0 (it
        has few and the whole forward pass to finish in).
        fused_update: reduce-scatter and update of a bucket in one kernel (fewer bytes).
        wave_priority / wave_priority_ag: wave priority (0..3) of the bounded reduce-scatter /
        update and of the bounded all-gather.
        full_width_when_alone: in mode dear, the kernels that can have no compute beside
        them (the last bucket's reduce-scatter/update after the backward pass has ended,
        and the first all-gather the forward pass waits for) run with an unbounded grid."""
        self.em, self.lr, self.momentum = em, lr, momentum
        self.fused_update = fused_update
        self.full_width_when_alone = full_width_when_alone
        self.wave_priority = wave_priority
        self.wave_priority_ag = wave_priority if wave_priority_ag is None else wave_priority_ag
        self.overlap_workgroups = overlap_workgroups
        self.overlap_workgroups_ag = overlap_workgroups if overlap_workgroups_ag is None else overlap_workgroups_ag
        if overlap_workgroups == 0:
            self.overlap_workgroups_ag = 0
        self.nb = em.plan.n_buckets
        # GEMMs per bucket: one number for every bucket, or one per bucket (backward order)
        self.ff_gemms = [ff_gemms] * self.nb if isinstance(ff_gemms, int) else list(ff_gemms)
        self.bp_gemms = [bp_gemms] * self.nb if isinstance(bp_gemms, int) else list(bp_gemms)
        if len(self.ff_gemms) != self.nb or len(self.bp_gemms) != self.nb:
            raise ValueError("one GEMM count per bucket expected")
        self.on_backward = on_backward
        dev = em.device
        self.a = torch.randn(gemm_dim, gemm_dim, device=dev, dtype=torch.float32).to(gemm_dtype)
        self.b = torch.randn(gemm_dim, gemm_dim, device=dev, dtype=torch.float32).to(gemm_dtype)
        self.c = torch.empty(gemm_dim, gemm_dim, device=dev, dtype=gemm_dtype)
        self.compute = compute_stream if compute_stream is not None else torch.cuda.Stream(device=dev)
        self.comm = comm_stream
        self.streams_concurrent = True
        if self.comm is None:
            # take the first stream that really runs beside the compute stream (different hardware queue)
            probe = torch.zeros(64, device=dev)
            m = torch.zeros(4096, 4096, device=dev)       # about a millisecond of work per product
            tried = []
            for _ in range(8):
                cand = torch.cuda.Stream(device=dev)
                tried.append(cand)
                if streams_run_concurrently(self.compute, cand, lambda: torch.matmul(m, m), probe):
                    self.comm = cand
                    break
            del m
            if self.comm is None:
                self.comm, self.streams_concurrent = tried[0], False
        self.grad_ready = [torch.cuda.Event() for _ in range(self.nb)]
        self.rs_done = [torch.cuda.Event() for _ in range(self.nb)]
        self.ag_done = [torch.cuda.Event() for _ in range(self.nb)]
        self.iteration_index = 0
        self._have_ag = False

    # -------------------------------------------------------------- pieces
    def _gemms(self, n: int) -> None:
        for _ in range(n):
            torch.matmul(self.a, self.b, out=self.c)

    def _forward(self, wait_for_ag: bool) -> None:
        """Feed-forward compute, first layer (highest bucket index) to last."""
        with torch.cuda.stream(self.compute):
            for b in reversed(range(self.nb)):
                if wait_for_ag and self._have_ag:
                    self.compute.wait_event(self.ag_done[b])      # FeedPipe: OP2 of b before FF of b
                self._gemms(self.ff_gemms[b])

    def _backward(self, signal: bool) -> None:
        """Back-propagation compute, last layer (bucket 0) to first."""
        with torch.cuda.stream(self.compute):
            for b in range(self.nb):
                if signal and self._have_ag:
                    # the tensors of bucket b are still read by the previous iteration's OP1
                    # until rs_done[b]; in order on the communication stream this is long past
                    self.compute.wait_event(self.rs_done[b])
                self._gemms(self.bp_gemms[b])
                if self.on_backward is not None:
                    self.on_backward(self.iteration_index, b)
                if signal:
                    self.grad_ready[b].record(self.compute)

    def _reduce_scatter_and_update(self, b: int, stream) -> None:
        if self.fused_update:
            self.em.reduce_scatter_update(b, self.lr, self.momentum, stream)
        else:
            self.em.reduce_scatter(b, stream)
            self.em.shard_update(b, self.lr, self.momentum, stream)

    # -------------------------------------------------------------- one iteration
    def iteration(self, mode: str = "dear") -> None:
        em, nb = self.em, self.nb
        overlapping = mode in ("dear", "wfbp")
        w_rs = self.overlap_workgroups if overlapping else 0
        w_ag = self.overlap_workgroups_ag if overlapping else 0
        em.set_max_workgroups(w_rs)
        em.set_wave_priority(self.wave_priority)
        if mode == "compute_only":
            self._forward(False)
            self._backward(False)
        elif mode == "comm_only":
            for b in range(nb):
                self._reduce_scatter_and_update(b, self.comm)
            for b in reversed(range(nb)):
                em.all_gather(b, self.comm)
        elif mode == "serial":
            # no overlap: compute, then the whole aggregation, on one stream
            self._forward(False)
            self._backward(False)
            for b in range(nb):
                self._reduce_scatter_and_update(b, self.compute)
            for b in reversed(range(nb)):
                em.all_gather(b, self.compute)
        elif mode == "wfbp":
            # all-reduce (= RS + AG back to back) of a bucket as soon as it is ready; the next
            # forward pass waits for all of them
            if self._have_ag:
                self.compute.wait_event(self.ag_done[nb - 1])
            self._forward(False)
            self._backward(True)
            for b in range(nb):
                self.comm.wait_event(self.grad_ready[b])
                em.set_max_workgroups(w_rs)
                em.set_wave_priority(self.wave_priority)
                self._reduce_scatter_and_update(b, self.comm)
                self.rs_done[b].record(self.comm)
                em.set_max_workgroups(w_ag)
                em.set_wave_priority(self.wave_priority_ag)
                em.all_gather(b, self.comm)
            self.ag_done[nb - 1].record(self.comm)
            for b in range(nb - 1):
                self.ag_done[b].record(self.comm)
            self._have_ag = True
        elif mode == "dear":
            # FeedPipe: the OP2 queued at the end of the previous iteration run under this
            # forward pass; each bucket's FF waits for its own OP2
            self._forward(True)
            # BackPipe: OP1 of a bucket as soon as its gradients are ready
            self._backward(True)
            alone = self.full_width_when_alone
            for b in range(nb):
                self.comm.wait_event(self.grad_ready[b])
                if alone and b == nb - 1:   # the backward pass has ended: nothing runs beside it
                    em.set_max_workgroups(0)
                self._reduce_scatter_and_update(b, self.comm)
                self.rs_done[b].record(self.comm)
            # all OP1 precede every OP2: in order on the one communication stream.
            # OP2 in forward order, to be hidden under the next forward pass
            em.set_wave_priority(self.wave_priority_ag)
            for b in reversed(range(nb)):
                em.set_max_workgroups(0 if (alone and b == nb - 1) else w_ag)   # the forward pass waits for the first
                em.all_gather(b, self.comm)
                self.ag_done[b].record(self.comm)
            self._have_ag = True
        else:
            raise ValueError(mode)
        self.iteration_index += 1

    def synchronize(self) -> None:
        """The paper's optim.synchronize(): wait for outstanding OP2 before reading parameters."""
        self.compute.synchronize()
        self.comm.synchronize()

    # -------------------------------------------------------------- measurement
    def time_mode(self, mode: str, iterations: int = 10, warmup: int = 3) -> float:
        """Steady-state milliseconds per iteration."""
        self._have_ag = False
        for _ in range(warmup):
            self.iteration(mode)
        self.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(iterations):
            self.iteration(mode)
        self.synchronize()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / iterations

    def time_phases(self, iterations: int = 10) -> Dict[str, float]:
        """Milliseconds of each part alone: FF, BP, RS(+update), AG."""
        out: Dict[str, float] = {}

        def timed(fn: Callable[[], None]) -> float:
            fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(iterations):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / iterations

        self.em.set_max_workgroups(0)   # every part alone, at full width
        out["ff"] = timed(lambda: self._forward(False))
        out["bp"] = timed(lambda: self._backward(False))
        out["rs"] = timed(lambda: [self._reduce_scatter_and_update(b, self.comm) for b in range(self.nb)])
        out["ag"] = timed(lambda: [self.em.all_gather(b, self.comm) for b in reversed(range(self.nb))])
        return out


def overlap_report(sched: DearSchedule, iterations: int = 10) -> Dict[str, object]:
    ph = sched.time_phases(iterations)
    t = {m: sched.time_mode(m, iterations) for m in ("compute_only", "comm_only", "serial", "wfbp", "dear")}
    t_comp, t_comm = t["compute_only"], t["comm_only"]
    hidden = (t_comp + t_comm - t["dear"]) / min(t_comp, t_comm)
    hidden_wfbp = (t_comp + t_comm - t["wfbp"]) / min(t_comp, t_comm)
    ideal_dear = max(ph["ff"], ph["ag"]) + max(ph["bp"], ph["rs"])      # paper Sec. VI-I
    ideal_base = ph["ff"] + max(ph["bp"], ph["rs"] + ph["ag"])
    return {
        "streams_concurrent": sched.streams_concurrent,
        "phases_ms": {k: round(v, 4) for k, v in ph.items()},
        "iteration_ms": {k: round(v, 4) for k, v in t.items()},
        "hidden_fraction_dear": round(hidden, 4), "hidden_fraction_wfbp": round(hidden_wfbp, 4),
        "ideal_ms": {"dear": round(ideal_dear, 4), "baseline": round(ideal_base, 4)},
    }
