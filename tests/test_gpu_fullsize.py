"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(one launch per bucket and phase): whole sampled buckets / shards are recomputed by the
oracle and compared bit for bit, and properties that hold at any size are checked over
everything (all replicas identical after the all-gather, padding slots +0)."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _host(t: torch.Tensor) -> np.ndarray:
    t = t.cpu().contiguous()
    return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()


def _fill(em, w):
    param = W.make_flat_param(w, DEV)
    for p in range(w.P):
        em.load_dense(em.params[p], param)
        em.load_dense(em.grads[p], W.make_flat_grad(w, p, 0, DEV))
    del param
    em.scatter_params(0)
    torch.cuda.synchronize()


def _bucket_layers(op, b):
    first = int(op.bucket_first_layer[b])
    return list(range(first, first + int(op.bucket_n_layers[b])))


def _check_replicas_and_pads(em, op, w):
    for l in range(w.n_layers):
        for p in range(1, w.P):
            assert torch.equal(em.params[p][l], em.params[0][l]), (p, l)
    for b in range(op.n_buckets):
        S, base, d = int(op.bucket_shard_len[b]), int(op.bucket_shard_base[b]), int(op.bucket_len[b])
        flat = em.shard_grad[:, base:base + S].reshape(-1)[d:]
        assert flat.numel() == w.P * S - d
        assert bool((flat.view(torch.int32) == 0).all())


def test_bert_large_full_size_sampled_buckets():
    from paper_2302_12445_amd.emulation import EmulatedWorkers
    print("case: bert_large full size, buckets 0 / 5 / 10 recomputed by the oracle", flush=True)
    w = W.get_workload("bert_large")
    em = EmulatedWorkers(w.sizes, w.P, w.grad_dtype, w.threshold_bytes, DEV)
    op = oracle.plan(w.sizes, w.P, w.threshold_bytes, w.grad_elem_bytes)
    assert op.n_buckets == 11
    _fill(em, w)
    row = op.total_shard_len
    sample = [0, 5, 10]
    grads = [[None] * w.n_layers for _ in range(w.P)]
    params = [[None] * w.n_layers for _ in range(w.P)]
    for b in sample:
        for l in _bucket_layers(op, b):
            for p in range(w.P):
                grads[p][l] = _host(em.grads[p][l])
            for p in (0, w.P - 1):
                params[p][l] = _host(em.params[p][l]).copy()
    sg = np.zeros((w.P, row), np.float32)
    sp, sm = np.zeros_like(sg), np.zeros_like(sg)
    for b in sample:
        oracle.scatter_params(op, params, 0, sp, bucket=b)

    em.shard_grad.fill_(float("nan"))
    em.iteration(w.lr, w.momentum, per_bucket=True)
    torch.cuda.synchronize()

    for b in sample:
        oracle.reduce_scatter(op, b, grads, sg)
        oracle.shard_update(op, b, sg, sp, sm, w.lr, w.momentum)
        oracle.all_gather(op, b, sp, params, workers=range(0, 1))
        oracle.all_gather(op, b, sp, params, workers=range(w.P - 1, w.P))
        lo, S = int(op.bucket_shard_base[b]), int(op.bucket_shard_len[b])
        for name, dev, ref in (("grad", em.shard_grad, sg), ("param", em.shard_param, sp), ("mom", em.shard_mom, sm)):
            got = dev[:, lo:lo + S].cpu().numpy()
            assert np.array_equal(got.view(np.uint32), ref[:, lo:lo + S].view(np.uint32)), (b, name)
        for p in (0, w.P - 1):
            for l in _bucket_layers(op, b):
                assert np.array_equal(_host(em.params[p][l]).view(np.uint32), params[p][l].view(np.uint32)), (b, p, l)
    _check_replicas_and_pads(em, op, w)
    em.close()


@pytest.mark.parametrize("name,buckets", [("stress_16mb", [0, 24, 25]), ("stress_single", [0])])
def test_scale_stress_sampled_shards(name, buckets):
    """P = 64 replicas at BERT-Base shape (28 GB of gradients resident).  The oracle recomputes
    single shards (first, a middle one, last) of the sampled buckets."""
    from paper_2302_12445_amd.emulation import EmulatedWorkers
    print("case:", name, "sampled shards", flush=True)
    w = W.get_workload(name)
    em = EmulatedWorkers(w.sizes, w.P, w.grad_dtype, w.threshold_bytes, DEV)
    op = oracle.plan(w.sizes, w.P, w.threshold_bytes, w.grad_elem_bytes)
    _fill(em, w)
    row = op.total_shard_len

    # sampled (bucket, shard) pairs, the layers they touch, and their initial parameters
    samples = []
    sp = np.zeros((w.P, row), np.float32)
    for b in buckets:
        S, base, d = int(op.bucket_shard_len[b]), int(op.bucket_shard_base[b]), int(op.bucket_len[b])
        last_real = (d - 1) // S
        for s in sorted({0, 37 if 37 <= last_real else last_real // 2, last_real}):
            lo, hi = s * S, min((s + 1) * S, d)
            need = [l for l in _bucket_layers(op, b)
                    if int(op.layer_offset[l]) < hi and int(op.layer_offset[l]) + w.sizes[l] > lo]
            for l in need:  # slot = position in the bucket; filled from replica 0's tensors
                off = int(op.layer_offset[l])
                a, c = max(lo, off), min(hi, off + w.sizes[l])
                sp[s, base + a - lo:base + c - lo] = _host(em.params[0][l][a - off:c - off])
            samples.append((b, s, lo, hi, need))

    em.shard_grad.fill_(float("nan"))
    em.iteration(w.lr, w.momentum, per_bucket=True)
    torch.cuda.synchronize()

    sg = np.zeros((w.P, row), np.float32)
    sm = np.zeros_like(sg)
    for b, s, lo, hi, need in samples:
        S, base = int(op.bucket_shard_len[b]), int(op.bucket_shard_base[b])
        grads = [[None] * w.n_layers for _ in range(w.P)]
        for l in need:
            for p in range(w.P):
                grads[p][l] = _host(em.grads[p][l])
        oracle.reduce_scatter(op, b, grads, sg, shards=range(s, s + 1))
        oracle.shard_update(op, b, sg, sp, sm, w.lr, w.momentum, shards=range(s, s + 1))
        for nm, dev, ref in (("grad", em.shard_grad, sg), ("param", em.shard_param, sp), ("mom", em.shard_mom, sm)):
            got = dev[s, base:base + S].cpu().numpy()
            assert np.array_equal(got.view(np.uint32), ref[s, base:base + S].view(np.uint32)), (b, s, nm)
        for l in need:  # the gathered parameters are the updated slots, for every worker
            off = int(op.layer_offset[l])
            a, c = max(lo, off), min(hi, off + w.sizes[l])
            for p in (0, 31, 63):
                got = _host(em.params[p][l][a - off:c - off])
                assert np.array_equal(got.view(np.uint32), sp[s, base + a - lo:base + c - lo].view(np.uint32)), (b, s, l, p)
    _check_replicas_and_pads(em, op, w)
    em.close()
