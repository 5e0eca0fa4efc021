"""GPU: the DeAR two-stream schedule (BackPipe / FeedPipe) must give exactly the oracle's
parameters when every bucket's gradients are written on the compute stream just before
its reduce-scatter is released -- i.e. the event wiring preserves the data dependencies."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
import workloads as W
from helpers import small_workload, split_np, to_numpy

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("mode", ["dear", "wfbp", "serial"])
def test_schedule_matches_oracle(mode, fused):
    from paper_2302_12445_amd.emulation import EmulatedWorkers
    from paper_2302_12445_amd.schedule import DearSchedule
    print("case: schedule parity, mode", mode, "fused update" if fused else "separate update", flush=True)
    sizes = [4097, 3, 8191, 4096, 1, 12289, 7, 30001, 64, 513, 70000, 9]
    w = small_workload(sizes, 4, 30000 * 4, "f32", index=81)
    em = EmulatedWorkers(w.sizes, w.P, w.grad_dtype, w.threshold_bytes, DEV)
    op = oracle.plan(w.sizes, w.P, w.threshold_bytes, 4)
    nb = em.plan.n_buckets
    assert nb >= 4
    iters = 4
    flats = [[W.make_flat_grad(w, p, it) for p in range(w.P)] for it in range(iters)]
    dev_flats = [[f.to(DEV) for f in row] for row in flats]
    starts = np.concatenate([[0], np.cumsum(w.sizes)])

    def on_backward(it, b):
        # "back-propagation" of bucket b: its layers' gradients appear now, on the compute stream
        first, cnt = em.plan.bucket_first_layer[b], em.plan.bucket_n_layers[b]
        for p in range(w.P):
            for l in range(first, first + cnt):
                em.grads[p][l].copy_(dev_flats[it][p][starts[l]:starts[l + 1]], non_blocking=True)

    param = W.make_flat_param(w)
    for p in range(w.P):
        em.load_dense(em.params[p], param.to(DEV))
        for t in em.grads[p]:
            t.fill_(float("nan"))
    em.scatter_params(0)
    torch.cuda.synchronize()

    sched = DearSchedule(em, w.lr, w.momentum, gemm_dim=512, ff_gemms=1, bp_gemms=2, on_backward=on_backward,
                         overlap_workgroups=8, overlap_workgroups_ag=5, fused_update=fused)
    for it in range(iters):
        sched.iteration(mode)
    sched.synchronize()
    torch.cuda.synchronize()

    params = [split_np(to_numpy(param).copy(), w.sizes) for _ in range(w.P)]
    sg = np.zeros((w.P, op.total_shard_len), np.float32)
    sp, sm = np.zeros_like(sg), np.zeros_like(sg)
    oracle.scatter_params(op, params, 0, sp)
    for it in range(iters):
        grads = [split_np(to_numpy(f), w.sizes) for f in flats[it]]
        oracle.reduce_scatter(op, -1, grads, sg)
        oracle.shard_update(op, -1, sg, sp, sm, w.lr, w.momentum)
        oracle.all_gather(op, -1, sp, params)
    assert np.array_equal(em.shard_param.cpu().numpy().view(np.uint32), sp.view(np.uint32))
    assert np.array_equal(em.shard_mom.cpu().numpy().view(np.uint32), sm.view(np.uint32))
    for p in range(w.P):
        got = em.dense(em.params[p]).cpu().numpy()
        assert np.array_equal(got.view(np.uint32), np.concatenate(params[p]).view(np.uint32))
    em.close()


def test_replan_carries_optimizer_state():
    """Changing the buffer size mid-training (what the tuner does) re-shards parameters and
    momentum with library calls; the run must equal the oracle's, which gathers its momentum
    shards to full tensors and scatters them under the new plan."""
    from paper_2302_12445_amd.emulation import EmulatedWorkers
    print("case: replan with state carry-over", flush=True)
    sizes = [4097, 3, 8191, 4096, 1, 12289, 7, 30001, 64, 513]
    w = small_workload(sizes, 4, 21000 * 4, "f32", index=91)
    thresholds = [21000 * 4, 9000 * 4, W.NO_LIMIT, 0]
    em = EmulatedWorkers(w.sizes, w.P, w.grad_dtype, thresholds[0], DEV)
    param = W.make_flat_param(w)
    for p in range(w.P):
        em.load_dense(em.params[p], param.to(DEV))
    em.scatter_params(0)

    op = oracle.plan(w.sizes, w.P, thresholds[0], 4)
    params = [split_np(to_numpy(param).copy(), w.sizes) for _ in range(w.P)]
    sg = np.zeros((w.P, op.total_shard_len), np.float32)
    sp, sm = np.zeros_like(sg), np.zeros_like(sg)
    oracle.scatter_params(op, params, 0, sp)
    it = 0
    for phase, thr in enumerate(thresholds):
        if phase:
            em.replan(thr)
            mom_full = [[np.zeros(n, np.float32) for n in w.sizes] for _ in range(w.P)]
            oracle.all_gather(op, -1, sm, mom_full)
            op = oracle.plan(w.sizes, w.P, thr, 4)
            sg = np.zeros((w.P, op.total_shard_len), np.float32)
            sp, sm = np.zeros_like(sg), np.zeros_like(sg)
            oracle.scatter_params(op, params, 0, sp)
            oracle.scatter_params(op, mom_full, 0, sm)
            assert em.plan.n_buckets == op.n_buckets
        for _ in range(2):
            flats = [W.make_flat_grad(w, p, it) for p in range(w.P)]
            for p in range(w.P):
                em.load_dense(em.grads[p], flats[p].to(DEV))
            em.iteration(w.lr, w.momentum, fused_update=bool(it % 2))
            grads = [split_np(to_numpy(f), w.sizes) for f in flats]
            oracle.reduce_scatter(op, -1, grads, sg)
            oracle.shard_update(op, -1, sg, sp, sm, w.lr, w.momentum)
            oracle.all_gather(op, -1, sp, params)
            it += 1
        torch.cuda.synchronize()
        assert np.array_equal(em.shard_param.cpu().numpy().view(np.uint32), sp.view(np.uint32)), phase
        assert np.array_equal(em.shard_mom.cpu().numpy().view(np.uint32), sm.view(np.uint32)), phase
        for p in range(w.P):
            got = em.dense(em.params[p]).cpu().numpy()
            assert np.array_equal(got.view(np.uint32), np.concatenate(params[p]).view(np.uint32)), (phase, p)
    em.close()


def test_all_gather_workers_range_errors_and_subset():
    import ctypes as C
    import paper_2302_12445_amd as dear
    from paper_2302_12445_amd import binding
    from paper_2302_12445_amd.emulation import EmulatedWorkers
    w = small_workload([5000, 77, 4096], 4, 5000 * 4, "f32", index=92)
    em = EmulatedWorkers(w.sizes, w.P, "f32", w.threshold_bytes, DEV)
    for p in range(4):
        em.load_dense(em.params[p], torch.full((w.N,), float(p + 1), device=DEV))
    em.shard_param.fill_(7.0)
    dear.dear_all_gather_workers(em.ctx, -1, em.shard_param.data_ptr(), 1, 2)
    torch.cuda.synchronize()
    vals = [float(em.params[p][0][0]) for p in range(4)]
    assert vals == [1.0, 7.0, 7.0, 4.0]
    assert all(bool((t == 7.0).all()) for t in em.params[1]) and all(bool((t == 4.0).all()) for t in em.params[3])
    lib = dear.load_library()
    sp = C.c_void_p(em.shard_param.data_ptr())
    for first, n in ((-1, 1), (0, 0), (0, 5), (3, 2), (4, 1)):
        assert lib.dear_all_gather_workers(em.ctx.handle, -1, sp, first, n, None) == binding.DEAR_ERANGE
    for bad in (-1, 4):
        assert lib.dear_ctx_set_wave_priority(em.ctx.handle, bad) == binding.DEAR_EINVAL
    assert lib.dear_ctx_set_max_workgroups(em.ctx.handle, -1) == binding.DEAR_EINVAL
    # a bound below the tile count but above nothing else: the bounded all-gather must still cover everything
    em.set_max_workgroups(1)
    em.shard_param.fill_(9.0)
    dear.dear_all_gather(em.ctx, -1, em.shard_param.data_ptr())
    torch.cuda.synchronize()
    assert all(bool((t == 9.0).all()) for p in range(4) for t in em.params[p])
    em.close()


@pytest.mark.parametrize("fused", [False, True])
def test_graph_replays_match_eager_oracle(fused):
    """One iteration captured into a HIP graph: every replay, with eager work (fresh
    gradients, a synchronisation) between replays, must equal the oracle's iteration."""
    from paper_2302_12445_amd.emulation import EmulatedWorkers
    print("case: graph capture, fused =", fused, flush=True)
    w = W.get_workload("tiny")
    em = EmulatedWorkers(w.sizes, w.P, w.grad_dtype, w.threshold_bytes, DEV)
    op = oracle.plan(w.sizes, w.P, w.threshold_bytes, 4)
    param = W.make_flat_param(w)
    params = [split_np(to_numpy(param).copy(), w.sizes) for _ in range(w.P)]
    for p in range(w.P):
        em.load_dense(em.params[p], param.to(DEV))
    em.scatter_params(0)
    sg = np.zeros((w.P, op.total_shard_len), np.float32)
    sp, sm = np.zeros_like(sg), np.zeros_like(sg)
    oracle.scatter_params(op, params, 0, sp)
    torch.cuda.synchronize()
    graph = em.capture_iteration(w.lr, w.momentum, fused_update=fused)
    # the capture must not have executed anything
    assert np.array_equal(em.shard_param.cpu().numpy().view(np.uint32), sp.view(np.uint32))
    for it in range(4):
        flats = [W.make_flat_grad(w, p, it) for p in range(w.P)]
        for p in range(w.P):
            em.load_dense(em.grads[p], flats[p].to(DEV))       # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        grads = [split_np(to_numpy(f), w.sizes) for f in flats]
        oracle.reduce_scatter(op, -1, grads, sg)
        oracle.shard_update(op, -1, sg, sp, sm, w.lr, w.momentum)
        oracle.all_gather(op, -1, sp, params)
        assert np.array_equal(em.shard_param.cpu().numpy().view(np.uint32), sp.view(np.uint32)), it
        assert np.array_equal(em.shard_mom.cpu().numpy().view(np.uint32), sm.view(np.uint32)), it
        for p in range(w.P):
            got = em.dense(em.params[p]).cpu().numpy()
            assert np.array_equal(got.view(np.uint32), np.concatenate(params[p]).view(np.uint32)), (it, p)
    del graph
    em.close()
