"""dear_reduce_scatter_static (no context, no allocation: tables in a static device array)
against dear_reduce_scatter through a context, and against the oracle, bit for bit -- two
calls in a row on the same GPU, the second with a smaller input, so the array still holds the
first call's longer tables when the second call's kernel runs."""
from __future__ import annotations

import ctypes as C

import numpy as np
import pytest
import torch

import oracle
import workloads as W
from helpers import small_workload, split_np, to_numpy

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _bits(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)


def _case(sizes, P, threshold, dtype, index, bucket):
    """Returns nothing; asserts static == context == oracle for one call."""
    from paper_2302_12445_amd import binding as B
    from paper_2302_12445_amd.emulation import EmulatedWorkers
    print("case: static reduce-scatter, %d layers, P=%d, %s, bucket %d" % (len(sizes), P, dtype, bucket), flush=True)
    lib = B.load_library()
    w = small_workload(sizes, P, threshold, dtype, index=index, std=1e-2)
    em = EmulatedWorkers(w.sizes, w.P, w.grad_dtype, w.threshold_bytes, DEV)
    flats = [W.make_flat_grad(w, p, 0) for p in range(P)]
    for p in range(P):
        em.load_dense(em.grads[p], flats[p].to(DEV))
    row = em.plan.total_shard_len

    # the existing entry point, through its context
    em.shard_grad.fill_(float("nan"))
    rc = lib.dear_reduce_scatter(em.ctx.handle, bucket, C.c_void_p(em.shard_grad.data_ptr()), None)
    assert rc == 0
    torch.cuda.synchronize()
    want = em.shard_grad.clone()

    # the new entry point: raw C ABI, plan + host pointer array, its own output buffer
    out = torch.full((P, row), float("nan"), dtype=torch.float32, device=DEV)
    n = P * len(sizes)
    ptrs = (C.c_void_p * n)(*[t.data_ptr() for rep in em.grads for t in rep])
    s = torch.cuda.Stream(device=DEV)
    s.wait_stream(torch.cuda.current_stream())
    rc = lib.dear_reduce_scatter_static(em.plan.handle, B.DEAR_F32 if dtype == "f32" else B.DEAR_BF16, ptrs,
                                        bucket, C.c_void_p(out.data_ptr()), C.c_void_p(s.cuda_stream))
    assert rc == 0, B.strerror(rc)
    s.synchronize()
    assert np.array_equal(_bits(out), _bits(want))      # NaN fill compares equal bit for bit where untouched

    # and both against the oracle on the slots the call covers
    op = oracle.plan(w.sizes, P, threshold, w.grad_elem_bytes)
    sg = np.zeros((P, row), np.float32)
    oracle.reduce_scatter(op, bucket, [split_np(to_numpy(f), w.sizes) for f in flats], sg)
    buckets = range(op.n_buckets) if bucket < 0 else [bucket]
    got = out.cpu().numpy()
    for b in buckets:
        lo, S = int(op.bucket_shard_base[b]), int(op.bucket_shard_len[b])
        assert np.array_equal(got[:, lo:lo + S].view(np.uint32), sg[:, lo:lo + S].view(np.uint32)), b
    em.close()


def test_static_reduce_scatter_two_calls_second_smaller():
    big = [300_001, 4097, 3, 8191, 4096, 1, 12289, 7, 30001, 64, 513, 1_000_003]
    _case(big, 8, 1_100_000 * 2, "bf16", 71, -1)          # many tiles, several buckets, all in one launch
    _case(big[:5], 3, W.NO_LIMIT, "f32", 72, 0)            # fewer pointers, fewer tiles, other dtype and P
    _case([37], 2, 0, "f32", 73, 0)                       # a single ragged tile plus padding


def test_static_reduce_scatter_rejects_what_does_not_fit():
    from paper_2302_12445_amd import binding as B
    lib = B.load_library()
    buf = torch.zeros(1 << 16, dtype=torch.float32, device=DEV)
    good = buf.data_ptr()
    # more pointers than the static table holds
    L = B.DEAR_STATIC_MAX_POINTERS // 64 + 1
    pl = B.dear_plan([1] * L, 64, B.DEAR_NO_LIMIT, 4)
    ptrs = (C.c_void_p * (64 * L))(*([good] * (64 * L)))
    assert lib.dear_reduce_scatter_static(pl.handle, B.DEAR_F32, ptrs, -1, C.c_void_p(good), None) == B.DEAR_ETOOBIG
    # more tiles than the static table holds (nothing is dereferenced: rejected before any launch)
    pl = B.dear_plan([B.DEAR_STATIC_MAX_TILES * 4096 + 1], 1, B.DEAR_NO_LIMIT, 4)
    ptrs = (C.c_void_p * 1)(good)
    assert lib.dear_reduce_scatter_static(pl.handle, B.DEAR_F32, ptrs, 0, C.c_void_p(good), None) == B.DEAR_ETOOBIG
    # ordinary argument errors
    pl = B.dear_plan([8, 8], 2, 0, 4)
    ptrs = (C.c_void_p * 4)(good, good, good, good)
    assert lib.dear_reduce_scatter_static(pl.handle, B.DEAR_BF16, ptrs, 0, C.c_void_p(good), None) == B.DEAR_EINVAL
    assert lib.dear_reduce_scatter_static(pl.handle, B.DEAR_F32, ptrs, 2, C.c_void_p(good), None) == B.DEAR_ERANGE
    assert lib.dear_reduce_scatter_static(pl.handle, B.DEAR_F32, ptrs, 0, C.c_void_p(good + 4), None) == B.DEAR_EALIGN
    assert lib.dear_reduce_scatter_static(None, B.DEAR_F32, ptrs, 0, C.c_void_p(good), None) == B.DEAR_EINVAL
    assert "scratch" in B.strerror(B.DEAR_ETOOBIG)
