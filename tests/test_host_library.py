"""CPU-only checks of libdear: exports, argument errors, and the host planner / tile
table against the oracle's plan (bit-exact integer parity).  No kernel is launched."""
from __future__ import annotations

import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_2302_12445_amd as dear
import workloads as W
from paper_2302_12445_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "dear.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(dear_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    lib = dear.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert dear.dear_version() >= 100
    assert dear.strerror(0) == "ok" and "align" in dear.strerror(-5)


def test_probe_library_exports_every_declared_symbol():
    from paper_2302_12445_amd import hbm_probe
    header = open(os.path.join(ROOT, "include", "dear_probe.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(dear_[a-z_]+)\s*\(", header))
    assert declared == set(hbm_probe.EXPORTS)
    lib = hbm_probe.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    out = C.c_double()
    # argument errors are rejected before any HIP call
    assert lib.dear_probe_streams(0, 0, 1 << 20, 0, 4, 0, 1, C.byref(out), None) == -1
    assert lib.dear_probe_streams(0, 8, 1000, 0, 4, 0, 1, C.byref(out), None) == -1
    assert lib.dear_probe_streams(9, 8, 1 << 20, 0, 4, 0, 1, C.byref(out), None) == -1
    assert lib.dear_probe_streams(1, 8, 1 << 20, 0, 2, 0, 1, C.byref(out), None) == -1
    assert lib.dear_probe_streams(0, 8, 1 << 20, 0, 4, 100, 1, C.byref(out), None) == -1
    assert lib.dear_probe_streams(0, 8, 1 << 20, 0, 4, 0, 1, None, None) == -1


def assert_plans_equal(lp, op):
    assert lp.n_buckets == op.n_buckets and lp.P == op.P and lp.n_layers == op.L
    assert lp.total_shard_len == op.total_shard_len and lp.total_elems == op.total_elems
    assert lp.layer_bucket == [int(v) for v in op.layer_bucket]
    assert lp.layer_offset == [int(v) for v in op.layer_offset]
    assert lp.bucket_first_layer == [int(v) for v in op.bucket_first_layer]
    assert lp.bucket_n_layers == [int(v) for v in op.bucket_n_layers]
    assert lp.bucket_len == [int(v) for v in op.bucket_len]
    assert lp.bucket_shard_len == [int(v) for v in op.bucket_shard_len]
    assert lp.bucket_shard_base == [int(v) for v in op.bucket_shard_base]


@pytest.mark.parametrize("name", W.WORKLOAD_NAMES)
def test_plan_matches_oracle_on_configs(name):
    w = W.get_workload(name)
    lp = dear.dear_plan(w.sizes, w.P, w.threshold_bytes, w.grad_elem_bytes)
    op = oracle.plan(w.sizes, w.P, w.threshold_bytes, w.grad_elem_bytes)
    assert_plans_equal(lp, op)


def test_plan_matches_oracle_random():
    rng = np.random.default_rng(4321)
    for _ in range(400):
        L = int(rng.integers(1, 50))
        sizes = [int(v) for v in rng.integers(1, 9000, size=L)]
        P = int(rng.integers(1, 70))
        g = int(rng.choice([2, 4]))
        x = int(rng.choice([0, 1, 3, 100, 4000, 36000, 10 ** 6, W.NO_LIMIT - 1, W.NO_LIMIT]))
        assert_plans_equal(dear.dear_plan(sizes, P, x, g), oracle.plan(sizes, P, x, g))


def test_plan_large_sizes_do_not_overflow():
    sizes = [2 ** 40, 2 ** 41 + 5, 7]
    for x in (0, 2 ** 43, W.NO_LIMIT):
        assert_plans_equal(dear.dear_plan(sizes, 64, x, 4), oracle.plan(sizes, 64, x, 4))


def test_plan_fixed_layers():
    sizes = [5, 9, 1, 300, 2, 8, 8]
    lp = dear.dear_plan_fixed_layers(sizes, 3, 4, 4)
    assert lp.bucket_first_layer == [3, 0] and lp.bucket_n_layers == [4, 3]
    assert lp.bucket_len == [318, 15]
    assert lp.layer_offset == [10, 1, 0, 18, 16, 8, 0]
    # same chunking rule as the threshold plan: with every layer in one bucket both agree
    one = dear.dear_plan_fixed_layers(sizes, 3, len(sizes), 4)
    assert_plans_equal(one, oracle.plan(sizes, 3, W.NO_LIMIT, 4))
    assert dear.dear_plan_fixed_layers(sizes, 3, 1, 4).n_buckets == len(sizes)


def test_plan_fixed_layers_matches_oracle():
    """Integer parity of dear_plan_fixed_layers with the oracle's fixed-layers rule (Sec. VI-G)."""
    rng = np.random.default_rng(777)
    for _ in range(300):
        L = int(rng.integers(1, 50))
        sizes = [int(v) for v in rng.integers(1, 9000, size=L)]
        P = int(rng.integers(1, 70))
        g = int(rng.choice([2, 4]))
        K = int(rng.integers(1, 60))
        assert_plans_equal(dear.dear_plan_fixed_layers(sizes, P, K, g), oracle.plan_fixed_layers(sizes, P, K, g))
    for name in ("resnet50", "densenet201", "bert_base", "bert_large"):
        w = W.get_workload(name)
        assert_plans_equal(dear.dear_plan_fixed_layers(w.sizes, w.P, 4, w.grad_elem_bytes),
                           oracle.plan_fixed_layers(w.sizes, w.P, 4, w.grad_elem_bytes))
    big = [2 ** 40, 2 ** 41 + 5, 7]
    assert_plans_equal(dear.dear_plan_fixed_layers(big, 64, 2, 4), oracle.plan_fixed_layers(big, 64, 2, 4))


def test_plan_argument_errors():
    for args in (([], 2, 10, 4), ([1, 0], 2, 10, 4), ([1], 0, 10, 4), ([1], 2, -1, 4), ([1], 2, 10, 3)):
        with pytest.raises(dear.DearError) as e:
            dear.dear_plan(*args)
        assert e.value.status == binding.DEAR_EINVAL
    with pytest.raises(dear.DearError):
        dear.dear_plan_fixed_layers([1, 2], 2, 0, 4)
    lib = dear.load_library()
    arr = (C.c_int64 * 1)(5)
    assert lib.dear_plan(arr, 1, 1, 0, 4, None) == binding.DEAR_EINVAL
    assert lib.dear_plan(None, 1, 1, 0, 4, C.byref(C.c_void_p())) == binding.DEAR_EINVAL
    assert lib.dear_plan_view(None, None) == binding.DEAR_EINVAL
    lib.dear_plan_free(None)
    lib.dear_ctx_destroy(None)


def test_calls_reject_bad_arguments_before_touching_the_gpu():
    lib = dear.load_library()
    assert lib.dear_reduce_scatter(None, 0, None, None) == binding.DEAR_EINVAL
    assert lib.dear_shard_update(None, 0, None, None, None, 0.1, 0.9, None) == binding.DEAR_EINVAL
    assert lib.dear_all_gather(None, 0, None, None) == binding.DEAR_EINVAL
    assert lib.dear_scatter_params(None, 0, None, None) == binding.DEAR_EINVAL
    assert lib.dear_ctx_set_max_workgroups(None, 4) == binding.DEAR_EINVAL
    assert lib.dear_ctx_set_wave_priority(None, 1) == binding.DEAR_EINVAL
    pl = dear.dear_plan([8, 8], 2, 0, 4)
    out = C.c_void_p()
    good = (C.c_void_p * 4)(0x1000, 0x2000, 0x3000, 0x4000)
    odd = (C.c_void_p * 4)(0x1000, 0x2004, 0x3000, 0x4000)
    null = (C.c_void_p * 4)(0x1000, 0, 0x3000, 0x4000)
    assert lib.dear_ctx_create(pl.handle, binding.DEAR_F32, odd, good, C.byref(out)) == binding.DEAR_EALIGN
    assert lib.dear_ctx_create(pl.handle, binding.DEAR_F32, good, odd, C.byref(out)) == binding.DEAR_EALIGN
    assert lib.dear_ctx_create(pl.handle, binding.DEAR_F32, null, good, C.byref(out)) == binding.DEAR_EINVAL
    assert lib.dear_ctx_create(pl.handle, binding.DEAR_BF16, good, good, C.byref(out)) == binding.DEAR_EINVAL
    assert lib.dear_ctx_create(pl.handle, 7, good, good, C.byref(out)) == binding.DEAR_EINVAL
    assert lib.dear_ctx_create(None, binding.DEAR_F32, good, good, C.byref(out)) == binding.DEAR_EINVAL
    assert out.value is None


# ----------------------------------------------------------------- tile table
def check_tiles(sizes, P, x, g):
    """The tile table must cover every (layer, element) exactly once at the slot the
    oracle's plan assigns, cover every padding slot exactly once, and keep the shape the
    kernels rely on (one layer, one shard, bounded count, aligned interior cuts)."""
    lp = dear.dear_plan(sizes, P, x, g)
    op = oracle.plan(sizes, P, x, g)
    tiles, begin = dear.dear_plan_tiles(lp)
    assert begin[0] == 0 and begin[-1] == len(tiles)
    row = op.total_shard_len
    covered = np.zeros(P * row, np.int32)
    elem_seen = [np.zeros(n, np.int32) for n in sizes]
    T = binding.DEAR_TILE_ELEMS
    for b in range(lp.n_buckets):
        S, base = int(op.bucket_shard_len[b]), int(op.bucket_shard_base[b])
        for ti in range(begin[b], begin[b + 1]):
            t = tiles[ti]
            assert t.bucket == b and 1 <= t.count <= T and 0 <= t.shard < P
            lo = t.shard * row + base
            assert lo <= t.dst_begin and t.dst_begin + t.count <= lo + S        # inside one shard
            covered[t.dst_begin:t.dst_begin + t.count] += 1
            if t.layer < 0:
                e = t.shard * S + (t.dst_begin - lo)
                assert e >= op.bucket_len[b]                                    # really padding
                continue
            l = t.layer
            assert op.layer_bucket[l] == b
            assert 0 <= t.src_begin and t.src_begin + t.count <= sizes[l]
            elem_seen[l][t.src_begin:t.src_begin + t.count] += 1
            # slot of the tile's first element, from the oracle's tables
            e = int(op.layer_offset[l]) + t.src_begin
            assert e // S == t.shard and (e + t.count - 1) // S == t.shard
            assert t.dst_begin == t.shard * row + base + e % S
            # a tile never crosses a multiple of T of the layer's own index
            assert t.src_begin // T == (t.src_begin + t.count - 1) // T
    assert np.all(covered == 1)
    for seen in elem_seen:
        assert np.all(seen == 1)


def test_tiles_tiny_and_ragged():
    w = W.get_workload("tiny")
    check_tiles(w.sizes, w.P, w.threshold_bytes, 4)
    check_tiles([10], 4, W.NO_LIMIT, 4)              # trailing shards are pure padding
    check_tiles([1], 1, 0, 2)
    check_tiles([4097, 3, 8191, 4096, 1, 12289], 3, 9000 * 4, 4)
    check_tiles([4097, 3, 8191, 4096, 1, 12289], 5, W.NO_LIMIT, 2)


def test_tiles_random():
    rng = np.random.default_rng(77)
    for _ in range(60):
        L = int(rng.integers(1, 12))
        sizes = [int(v) for v in rng.choice([1, 2, 3, 5, 31, 32, 33, 100, 4095, 4096, 4097, 10000, 30001], size=L)]
        P = int(rng.integers(1, 9))
        g = int(rng.choice([2, 4]))
        x = int(rng.choice([0, 4000, 40000, W.NO_LIMIT]))
        check_tiles(sizes, P, x, g)


def test_tiles_resnet50():
    w = W.get_workload("resnet50")
    check_tiles(w.sizes, w.P, w.threshold_bytes, 4)


def test_recorded_counter_traffic_belongs_to_the_kernel_sources_in_the_tree():
    """bench.py reports roofline.traffic from profiles/hbm_traffic.json only while that record
    was taken with the kernel sources in the tree; a change to them must be followed by new
    counter runs (this test then fails until the record is renewed)."""
    import json
    import bench
    rec = json.load(open(bench.TRAFFIC_FILE))
    assert rec["kernel_source_sha256"] == bench.kernel_source_hash()
    for wl in ("bert_large", "resnet50", "bert_base"):
        w = W.get_workload(wl)
        nb = oracle.plan(w.sizes, w.P, w.threshold_bytes, w.grad_elem_bytes).n_buckets
        alg = w.algorithmic_bytes()
        for phase in ("rs", "update", "ag"):
            got = bench.recorded_traffic(wl, phase)
            assert got is not None
            assert 0.95 < got / (alg[phase] / nb) < 1.10, (wl, phase)   # HBM traffic ~ algorithmic bytes
