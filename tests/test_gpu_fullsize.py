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


@pytest.mark.parametrize("name,n_buckets,sample,per_bucket", [
    ("bert_large", 11, [0, 5, 10], True),   # P = 8, bf16 gradients, 64 MB; bucket 10 = word embedding alone
    ("bert_base", 7, [0, 3, 6], True),      # P = 16, fp32 gradients, 64 MB; bucket 6 = the oversized embedding
    ("bert_large", 11, [1, 9], False),      # one launch per phase over all buckets (bench.py --launch all_buckets)
])
def test_full_size_sampled_buckets(name, n_buckets, sample, per_bucket):
    from paper_2302_12445_amd.emulation import EmulatedWorkers
    print("case: %s full size, buckets %s recomputed by the oracle, %s" % (
        name, sample, "one launch per bucket" if per_bucket else "one launch per phase"), flush=True)
    w = W.get_workload(name)
    em = EmulatedWorkers(w.sizes, w.P, w.grad_dtype, w.threshold_bytes, DEV)
    op = oracle.plan(w.sizes, w.P, w.threshold_bytes, w.grad_elem_bytes)
    assert op.n_buckets == n_buckets
    if name == "bert_base":   # the embedding tensor alone exceeds the buffer size and is never split
        assert int(op.bucket_n_layers[6]) == 1 and int(op.bucket_len[6]) * 4 > w.threshold_bytes
    _fill(em, w)
    row = op.total_shard_len
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
    em.iteration(w.lr, w.momentum, per_bucket=per_bucket)
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


def test_scale_stress_one_bucket_every_shard_and_full_replicas():
    """P = 64, 16 MB buckets: for one whole bucket the oracle is run over all 64 shards and the
    GPU's three shard buffers are compared slot by slot; every parameter tensor of the bucket is
    compared in full on replica 0 (and on the last replica)."""
    from paper_2302_12445_amd.emulation import EmulatedWorkers
    print("case: stress_16mb, bucket 12, all 64 shards, replica 0 in full", flush=True)
    w = W.get_workload("stress_16mb")
    em = EmulatedWorkers(w.sizes, w.P, w.grad_dtype, w.threshold_bytes, DEV)
    op = oracle.plan(w.sizes, w.P, w.threshold_bytes, w.grad_elem_bytes)
    assert op.n_buckets == 26
    _fill(em, w)
    b = 12
    layers = _bucket_layers(op, b)
    assert len(layers) > 1
    grads = [[None] * w.n_layers for _ in range(w.P)]
    params = [[None] * w.n_layers for _ in range(w.P)]
    for l in layers:
        for p in range(w.P):
            grads[p][l] = _host(em.grads[p][l])
        for p in (0, w.P - 1):
            params[p][l] = _host(em.params[p][l]).copy()
    row = op.total_shard_len
    sg = np.zeros((w.P, row), np.float32)
    sp, sm = np.zeros_like(sg), np.zeros_like(sg)
    oracle.scatter_params(op, params, 0, sp, bucket=b)

    em.shard_grad.fill_(float("nan"))
    for p in (0, w.P - 1):
        for l in layers:
            em.params[p][l].fill_(float("nan"))
    em.iteration(w.lr, w.momentum, per_bucket=True)
    torch.cuda.synchronize()

    oracle.reduce_scatter(op, b, grads, sg)
    oracle.shard_update(op, b, sg, sp, sm, w.lr, w.momentum)
    oracle.all_gather(op, b, sp, params, workers=range(0, 1))
    oracle.all_gather(op, b, sp, params, workers=range(w.P - 1, w.P))
    lo, S = int(op.bucket_shard_base[b]), int(op.bucket_shard_len[b])
    for nm, dev, ref in (("grad", em.shard_grad, sg), ("param", em.shard_param, sp), ("mom", em.shard_mom, sm)):
        got = dev[:, lo:lo + S].cpu().numpy()
        assert np.array_equal(got.view(np.uint32), ref[:, lo:lo + S].view(np.uint32)), nm
    for p in (0, w.P - 1):
        for l in layers:
            assert np.array_equal(_host(em.params[p][l]).view(np.uint32), params[p][l].view(np.uint32)), (p, l)
    _check_replicas_and_pads(em, op, w)
    em.close()
