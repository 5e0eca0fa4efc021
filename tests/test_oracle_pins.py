"""Pins that tie the CPU oracle to the paper and to mathematics, not to itself.

Each pin is chosen so that a plausible slip in the oracle (wrong grouping rule, wrong
ring start, dropped 1/P, swapped lr/momentum, wrong slot index) fails at least one.
"""
from __future__ import annotations

import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
import workloads as W
from helpers import as_f32, bf16_bits_to_f32, grads_np, params_np, small_workload, split_np, to_numpy

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(path):
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                yield line.split()


# ----------------------------------------------------------------- workloads vs Table I
def test_shapes_match_table1():
    gens = {"resnet50": W.resnet50_sizes, "densenet201": W.densenet201_sizes,
            "inception_v4": W.inception_v4_sizes, "bert_base": W.bert_base_sizes,
            "bert_large": W.bert_large_sizes}
    seen = 0
    for name, tensors, params_m in _rows(os.path.join(GOLDEN, "table1_models.txt")):
        sizes = gens[name]()
        assert len(sizes) == int(tensors)
        assert round(sum(sizes) / 1e6, 1) == float(params_m)
        seen += 1
    assert seen == 5


# ----------------------------------------------------------------- plan: worked example
def test_plan_worked_example_tiny():
    w = W.get_workload("tiny")
    pl = oracle.plan(w.sizes, w.P, w.threshold_bytes, 4)
    buckets = [r for r in _rows(os.path.join(GOLDEN, "tiny_plan.txt")) if r[0] != "L"]
    layers = [r[1:] for r in _rows(os.path.join(GOLDEN, "tiny_plan.txt")) if r[0] == "L"]
    assert pl.n_buckets == len(buckets) == 5
    for b, first, cnt, d, S, base in buckets:
        b = int(b)
        assert pl.bucket_first_layer[b] == int(first)
        assert pl.bucket_n_layers[b] == int(cnt)
        assert pl.bucket_len[b] == int(d)
        assert pl.bucket_shard_len[b] == int(S)
        assert pl.bucket_shard_base[b] == int(base)
    for l, b, off in layers:
        assert pl.layer_bucket[int(l)] == int(b)
        assert pl.layer_offset[int(l)] == int(off)
    assert pl.total_shard_len == 87200


def test_plan_config_bucket_lengths():
    for name, P, x, g, *ds in _rows(os.path.join(GOLDEN, "config_buckets.txt")):
        w = W.get_workload(name)
        assert (w.P, w.threshold_bytes, w.grad_elem_bytes) == (int(P), int(x), int(g))
        pl = oracle.plan(w.sizes, w.P, w.threshold_bytes, w.grad_elem_bytes)
        assert list(pl.bucket_len) == [int(d) for d in ds]


# ----------------------------------------------------------------- plan: invariants
def check_plan_invariants(sizes, P, x_bytes, g, pl):
    """Properties that single out the plan: groups are runs of consecutive layers taken
    last-to-first; a group exceeds X only if it is one tensor; no group could have taken
    the next layer as well; chunking covers the group with P chunks of equal length."""
    L = len(sizes)
    X = x_bytes // g
    B = pl.n_buckets
    nxt = L  # one past the highest layer not yet assigned
    for b in range(B):
        first, cnt, d = int(pl.bucket_first_layer[b]), int(pl.bucket_n_layers[b]), int(pl.bucket_len[b])
        assert cnt >= 1 and first + cnt == nxt          # contiguous, descending, no gap
        nxt = first
        assert d == sum(sizes[first:first + cnt])
        assert d <= X or cnt == 1
        if first > 0:                                   # greedy maximality
            assert d + sizes[first - 1] > X
        off = 0
        for l in range(first + cnt - 1, first - 1, -1):  # arrival order, densely packed
            assert pl.layer_bucket[l] == b and pl.layer_offset[l] == off
            off += sizes[l]
        S = int(pl.bucket_shard_len[b])
        assert S % 32 == 0 and P * S >= d
        assert S == 32 or (S - 32) * P < d              # smallest such multiple of 32
        assert pl.bucket_shard_base[b] == sum(int(s) for s in pl.bucket_shard_len[:b])
    assert nxt == 0


@pytest.mark.parametrize("name", W.WORKLOAD_NAMES)
def test_plan_invariants_configs(name):
    w = W.get_workload(name)
    pl = oracle.plan(w.sizes, w.P, w.threshold_bytes, w.grad_elem_bytes)
    check_plan_invariants(w.sizes, w.P, w.threshold_bytes, w.grad_elem_bytes, pl)


def test_plan_invariants_random():
    rng = np.random.default_rng(1234)
    for _ in range(300):
        L = int(rng.integers(1, 40))
        sizes = [int(v) for v in rng.integers(1, 5000, size=L)]
        P = int(rng.integers(1, 12))
        g = int(rng.choice([2, 4]))
        x = int(rng.choice([0, 1, 7, 100, 4000, 20000, 10 ** 6, W.NO_LIMIT]))
        pl = oracle.plan(sizes, P, x, g)
        check_plan_invariants(sizes, P, x, g, pl)


def test_plan_threshold_extremes():
    sizes = [5, 9, 1, 300, 2]
    assert oracle.plan(sizes, 3, 0, 4).n_buckets == len(sizes)       # no fusion
    assert oracle.plan(sizes, 3, W.NO_LIMIT, 4).n_buckets == 1        # one bucket
    # equality with x stays in the group; one more element does not
    assert oracle.plan([4, 6], 2, 10 * 4, 4).n_buckets == 1
    assert oracle.plan([4, 6], 2, 10 * 4 - 1, 4).n_buckets == 2
    # x counts bytes of the gradient type
    assert oracle.plan([4, 6], 2, 20, 2).n_buckets == 1
    assert oracle.plan([4, 6], 2, 20, 4).n_buckets == 2


def test_plan_rejects_bad_arguments():
    for args in (([], 2, 10, 4), ([1, 0], 2, 10, 4), ([1], 0, 10, 4), ([1], 2, -1, 4), ([1], 2, 10, 3)):
        with pytest.raises(ValueError):
            oracle.plan(*args)


# ----------------------------------------------------------------- plan: fixed number of layers
def test_fixed_layers_worked_example_tiny():
    """Section VI-G's naive grouping (a fixed number of nearby layers), hand-worked for the
    Tiny layer list with four layers per group (the paper's number) and with three."""
    w = W.get_workload("tiny")
    rows = list(_rows(os.path.join(GOLDEN, "tiny_fixed_layers_plan.txt")))
    for K in (4, 3):
        pl = oracle.plan_fixed_layers(w.sizes, w.P, K, 4)
        buckets = [r[1:] for r in rows if r[0] == str(K)]
        layers = [r[2:] for r in rows if r[0] == "L" and r[1] == str(K)]
        assert pl.n_buckets == len(buckets) == (2 if K == 4 else 3)
        assert len(layers) == 8
        for b, first, cnt, d, S, base in buckets:
            b = int(b)
            assert pl.bucket_first_layer[b] == int(first)
            assert pl.bucket_n_layers[b] == int(cnt)
            assert pl.bucket_len[b] == int(d)
            assert pl.bucket_shard_len[b] == int(S)
            assert pl.bucket_shard_base[b] == int(base)
        for l, b, off in layers:
            assert pl.layer_bucket[int(l)] == int(b)
            assert pl.layer_offset[int(l)] == int(off)


def check_fixed_layers_invariants(sizes, P, K, pl):
    """What singles out the fixed-layers plan: groups are runs of exactly K consecutive
    layers taken last-to-first, only the final group (the model's first layers) may be
    shorter, layers are packed densely in arrival order, chunking as for any group."""
    L = len(sizes)
    B = pl.n_buckets
    assert B == -(-L // K)
    nxt = L
    for b in range(B):
        first, cnt, d = int(pl.bucket_first_layer[b]), int(pl.bucket_n_layers[b]), int(pl.bucket_len[b])
        assert first + cnt == nxt
        assert cnt == (K if b < B - 1 else L - K * (B - 1))
        nxt = first
        assert d == sum(sizes[first:first + cnt])
        off = 0
        for l in range(first + cnt - 1, first - 1, -1):
            assert pl.layer_bucket[l] == b and pl.layer_offset[l] == off
            off += sizes[l]
        S = int(pl.bucket_shard_len[b])
        assert S % 32 == 0 and P * S >= d and (S == 32 or (S - 32) * P < d)
        assert pl.bucket_shard_base[b] == sum(int(s) for s in pl.bucket_shard_len[:b])
    assert nxt == 0


def test_fixed_layers_invariants_random():
    rng = np.random.default_rng(4321)
    for _ in range(300):
        L = int(rng.integers(1, 40))
        sizes = [int(v) for v in rng.integers(1, 5000, size=L)]
        P = int(rng.integers(1, 12))
        K = int(rng.integers(1, 45))
        check_fixed_layers_invariants(sizes, P, K, oracle.plan_fixed_layers(sizes, P, K, int(rng.choice([2, 4]))))
    for name in ("resnet50", "bert_base"):   # the models of the paper's study, four layers per group
        w = W.get_workload(name)
        check_fixed_layers_invariants(w.sizes, w.P, 4, oracle.plan_fixed_layers(w.sizes, w.P, 4, 4))


def test_fixed_layers_special_cases_reduce_to_the_threshold_rule():
    """One layer per group is the no-fusion plan (x = 0); at least L layers per group is the
    single-group plan (no limit): there the two grouping rules must agree table by table."""
    rng = np.random.default_rng(99)
    for _ in range(50):
        L = int(rng.integers(1, 30))
        sizes = [int(v) for v in rng.integers(1, 3000, size=L)]
        P = int(rng.integers(1, 9))
        for K, x in ((1, 0), (L, W.NO_LIMIT), (L + 3, W.NO_LIMIT)):
            a, b = oracle.plan_fixed_layers(sizes, P, K, 4), oracle.plan(sizes, P, x, 4)
            assert a.n_buckets == b.n_buckets
            for f in ("layer_bucket", "layer_offset", "bucket_first_layer", "bucket_n_layers", "bucket_len",
                      "bucket_shard_len", "bucket_shard_base"):
                assert np.array_equal(getattr(a, f), getattr(b, f)), f
    for args in (([], 2, 1, 4), ([1, 0], 2, 1, 4), ([1], 0, 1, 4), ([1], 2, 0, 4), ([1], 2, 1, 3)):
        with pytest.raises(ValueError):
            oracle.plan_fixed_layers(*args)


def test_slot_map_is_a_bijection():
    """Every (layer, element) lands on exactly one non-pad slot; pads stay untouched."""
    sizes = [13, 1, 70, 33, 5, 64, 2]
    for P in (1, 2, 3, 5):
        pl = oracle.plan(sizes, P, 80 * 4, 4)
        params = [[np.arange(n, dtype=np.float32) + 1000.0 * (l + 1) for l, n in enumerate(sizes)]
                  for _ in range(P)]
        shard = np.full((P, pl.total_shard_len), np.nan, np.float32)
        oracle.scatter_params(pl, params, 0, shard)
        real = shard[shard != 0.0]
        want = np.concatenate(params[0])
        assert np.array_equal(np.sort(real), np.sort(want))           # each element exactly once
        assert shard.size - real.size == P * pl.total_shard_len - sum(sizes)
        # positions computed independently from the plan tables
        for l, n in enumerate(sizes):
            b = pl.layer_bucket[l]
            S, base = int(pl.bucket_shard_len[b]), int(pl.bucket_shard_base[b])
            for i in range(n):
                e = int(pl.layer_offset[l]) + i
                assert shard[e // S, base + e % S] == params[0][l][i]


# ----------------------------------------------------------------- ring order: simulator
def ring_reduce_scatter_sim(copies, P, S):
    """Message-passing ring reduce-scatter (Sec. III-A): every worker holds a full copy
    of the group cut into P chunks of S; in round k worker r sends its running chunk
    (r-k-1) mod P to worker r+1, which adds it to its own copy.  After P-1 rounds
    worker r holds the finished chunk r."""
    buf = [c.copy() for c in copies]
    for k in range(P - 1):
        msgs = []
        for r in range(P):
            c = (r - k - 1) % P
            msgs.append(((r + 1) % P, c, buf[r][c * S:(c + 1) * S].copy()))
        for dst, c, payload in msgs:
            buf[dst][c * S:(c + 1) * S] = payload + buf[dst][c * S:(c + 1) * S]
    return [buf[r][r * S:(r + 1) * S] for r in range(P)]


@pytest.mark.parametrize("P", [1, 2, 3, 4, 5, 8])
def test_ring_order_matches_message_passing(P):
    rng = np.random.default_rng(99 + P)
    magnitudes = np.array([1e8, 1.0, -1e8, 1e-3, 3.0, -7e5, 1e-7, 12345.678], np.float32)
    for d in list(range(1, 71, 3)) + [70]:
        # values whose fp32 sum depends on the association order
        grads = [[(rng.choice(magnitudes, size=d) * rng.uniform(0.5, 1.5, size=d)).astype(np.float32)]
                 for _ in range(P)]
        pl = oracle.plan([d], P, W.NO_LIMIT, 4)
        S = int(pl.bucket_shard_len[0])
        out = np.full((P, pl.total_shard_len), np.nan, np.float32)
        oracle.reduce_scatter(pl, 0, grads, out)
        copies = []
        for p in range(P):
            c = np.zeros(P * S, np.float32)
            c[:d] = grads[p][0]
            copies.append(c)
        owned = ring_reduce_scatter_sim(copies, P, S)
        inv = np.float32(1.0) / np.float32(P)
        for r in range(P):
            want = owned[r] * inv
            assert np.array_equal(out[r].view(np.uint32), want.view(np.uint32)), (P, d, r)


def test_ring_order_is_observable():
    """The pin above is only meaningful if a different start would change bits."""
    P, d = 4, 1
    vals = [np.float32(1e8), np.float32(1.0), np.float32(-1e8), np.float32(1e-3)]
    pl = oracle.plan([d], P, W.NO_LIMIT, 4)
    out = np.zeros((P, pl.total_shard_len), np.float32)
    oracle.reduce_scatter(pl, 0, [[np.array([v], np.float32)] for v in vals], out)
    # element 0 is in chunk 0: order is workers 1, 2, 3, 0
    want = ((vals[1] + vals[2]) + vals[3]) + vals[0]
    assert out[0, 0] == want * np.float32(0.25)
    natural = ((vals[0] + vals[1]) + vals[2]) + vals[3]
    assert natural != want


# ----------------------------------------------------------------- exact arithmetic, end to end
def _frac(a):
    return Fraction(float(a))


@pytest.mark.parametrize("dtype,P", [("f32", 1), ("f32", 2), ("f32", 8), ("f32", 64), ("bf16", 4), ("bf16", 16)])
def test_exact_rational_three_iterations(dtype, P):
    """Integer gradients, power-of-two P, lr = 1/8, momentum = 1/2, parameters on a 2^-10
    grid: every intermediate is exactly representable in binary32, so the result is
    independent of summation order and must equal exact rational S-SGD with momentum
    (Eq. 2 plus the momentum buffer)."""
    rng = np.random.default_rng(7 * P + (dtype == "bf16"))
    sizes = [5, 1, 37, 64, 3, 20]
    lim = 1024 if dtype == "f32" else 256
    g = 4 if dtype == "f32" else 2
    pl = oracle.plan(sizes, P, 45 * g, g)
    assert pl.n_buckets >= 3
    lr, mu = 0.125, 0.5
    w0 = [(rng.integers(-100, 100, size=n) / 1024.0).astype(np.float32) for n in sizes]
    params = [[a.copy() for a in w0] for _ in range(P)]
    sg = np.zeros((P, pl.total_shard_len), np.float32)
    sp = np.zeros_like(sg)
    sm = np.zeros_like(sg)
    oracle.scatter_params(pl, params, 0, sp)
    exact_w = [[_frac(v) for v in a] for a in w0]
    exact_v = [[Fraction(0)] * n for n in sizes]
    for it in range(3):
        ints = [[rng.integers(-lim, lim + 1, size=n) for n in sizes] for _ in range(P)]
        if dtype == "f32":
            grads = [[a.astype(np.float32) for a in row] for row in ints]
        else:
            grads = [[to_numpy(torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16)) for a in row]
                     for row in ints]
        oracle.reduce_scatter(pl, -1, grads, sg)
        oracle.shard_update(pl, -1, sg, sp, sm, lr, mu)
        oracle.all_gather(pl, -1, sp, params)
        for l, n in enumerate(sizes):
            for i in range(n):
                gbar = Fraction(int(sum(int(ints[p][l][i]) for p in range(P))), P)
                exact_v[l][i] = Fraction(1, 2) * exact_v[l][i] + gbar
                exact_w[l][i] = exact_w[l][i] - Fraction(1, 8) * exact_v[l][i]
        for p in range(P):
            for l, n in enumerate(sizes):
                got = [_frac(v) for v in params[p][l]]
                assert got == exact_w[l], (it, p, l)


# ----------------------------------------------------------------- invariants from the paper
def _run_oracle_iteration(w, pl, grads, sg, sp, sm):
    oracle.reduce_scatter(pl, -1, grads, sg)
    oracle.shard_update(pl, -1, sg, sp, sm, w.lr, w.momentum)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_rs_then_ag_is_an_allreduce_average(dtype):
    """Reduce-scatter followed by all-gather is an all-reduce (Sec. III-A): gathering the
    averaged gradient gives every worker (1/P) sum_p g_p, within the fp32 summation bound."""
    w = small_workload([300, 17, 2048, 5, 64, 999], 6, 1100 * 4, dtype, std=1.0)
    pl = oracle.plan(w.sizes, w.P, w.threshold_bytes, w.grad_elem_bytes)
    grads = grads_np(w, 0)
    sg = np.full((w.P, pl.total_shard_len), np.nan, np.float32)
    oracle.reduce_scatter(pl, -1, grads, sg)
    out = [[np.full(n, np.nan, np.float32) for n in w.sizes] for _ in range(w.P)]
    oracle.all_gather(pl, -1, sg, out)
    for l, n in enumerate(w.sizes):
        stack = np.stack([as_f32(grads[p][l]).astype(np.float64) for p in range(w.P)])
        mean = stack.sum(0) / w.P
        bound = (w.P) * 2.0 ** -24 * np.abs(stack).sum(0) / w.P + 1e-45
        for p in range(w.P):
            assert np.all(np.abs(out[p][l].astype(np.float64) - mean) <= bound)
            assert np.array_equal(out[p][l], out[0][l])               # consistent replicas
    # pads reduce to +0
    for b in range(pl.n_buckets):
        S, base, d = int(pl.bucket_shard_len[b]), int(pl.bucket_shard_base[b]), int(pl.bucket_len[b])
        flat = sg[:, base:base + S].reshape(-1)
        assert np.all(flat[d:].view(np.uint32) == 0)


def test_shard_update_then_gather_equals_gather_then_full_update():
    """The paper gathers gradients and lets every worker update the whole model; this path
    updates the owned chunk and gathers parameters.  The update is element-wise, so both
    must give the same bits.  The full update below is written with numpy float32 ops."""
    w = small_workload([513, 40, 7, 1024, 129], 4, 600 * 4, "f32", std=0.05)
    pl = oracle.plan(w.sizes, w.P, w.threshold_bytes, 4)
    params = params_np(w)
    full_w = [a.copy() for a in params[0]]
    full_v = [np.zeros_like(a) for a in full_w]
    sg = np.zeros((w.P, pl.total_shard_len), np.float32)
    sp, sm = np.zeros_like(sg), np.zeros_like(sg)
    oracle.scatter_params(pl, params, 0, sp)
    lr, mu = np.float32(w.lr), np.float32(w.momentum)
    for it in range(3):
        grads = grads_np(w, it)
        _run_oracle_iteration(w, pl, grads, sg, sp, sm)
        oracle.all_gather(pl, -1, sp, params)
        gbar = [[np.zeros(n, np.float32) for n in w.sizes] for _ in range(w.P)]
        oracle.all_gather(pl, -1, sg, gbar)
        for l in range(w.n_layers):
            full_v[l] = (mu * full_v[l]) + gbar[0][l]
            full_w[l] = full_w[l] - (lr * full_v[l])
        for p in range(w.P):
            for l in range(w.n_layers):
                assert np.array_equal(params[p][l].view(np.uint32), full_w[l].view(np.uint32))


def test_constant_gradient_averages_to_itself():
    """Identical gradients on all workers average to themselves: for any value when P = 2
    (c + c is exact), and for P = 8 when the value has few significand bits so that
    every partial sum k*c is exact."""
    sizes = [100, 3, 257]
    for P, c in ((2, np.float32(0.3)), (8, np.float32(0.3125)), (8, np.float32(5 * 2.0 ** -20))):
        pl = oracle.plan(sizes, P, 200 * 4, 4)
        grads = [[np.full(n, c, np.float32) for n in sizes] for _ in range(P)]
        sg = np.zeros((P, pl.total_shard_len), np.float32)
        oracle.reduce_scatter(pl, -1, grads, sg)
        out = [[np.zeros(n, np.float32) for n in sizes] for _ in range(P)]
        oracle.all_gather(pl, -1, sg, out)
        for l in range(len(sizes)):
            assert np.all(out[P - 1][l] == c)


def test_signed_zero():
    """A sum of negative zeros is -0 and stays -0 after the 1/P; padding is +0."""
    P, sizes = 4, [5]
    pl = oracle.plan(sizes, P, W.NO_LIMIT, 4)
    grads = [[np.full(5, -0.0, np.float32)] for _ in range(P)]
    sg = np.full((P, pl.total_shard_len), np.nan, np.float32)
    oracle.reduce_scatter(pl, 0, grads, sg)
    assert np.all(sg[0, :5].view(np.uint32) == 0x80000000)
    assert np.all(sg[0, 5:].view(np.uint32) == 0) and np.all(sg[1:].view(np.uint32) == 0)


# ----------------------------------------------------------------- library special case
def test_single_worker_is_plain_sgd_momentum():
    """P = 1, one bucket: reduce-scatter multiplies by 1, all-gather copies, so three
    iterations must agree with torch.optim.SGD(momentum).  The library may fuse the
    multiply-add, which moves a result by up to one ULP of the larger operand per step
    (|w| <= 0.11, lr*|v| <= 0.01 here); exact bits are pinned by the rational test."""
    w = small_workload([700, 33, 1500], 1, W.NO_LIMIT, "f32", std=0.02)
    pl = oracle.plan(w.sizes, 1, w.threshold_bytes, 4)
    assert pl.n_buckets == 1
    params = params_np(w)
    tparams = [torch.nn.Parameter(torch.from_numpy(a.copy())) for a in params[0]]
    opt = torch.optim.SGD(tparams, lr=w.lr, momentum=w.momentum)
    sg = np.zeros((1, pl.total_shard_len), np.float32)
    sp, sm = np.zeros_like(sg), np.zeros_like(sg)
    oracle.scatter_params(pl, params, 0, sp)
    for it in range(3):
        grads = grads_np(w, it)
        for tp, g in zip(tparams, grads[0]):
            tp.grad = torch.from_numpy(g.copy())
        opt.step()
        _run_oracle_iteration(w, pl, grads, sg, sp, sm)
        oracle.all_gather(pl, -1, sp, params)
        for tp, mine in zip(tparams, params[0]):
            ref = tp.detach().numpy()
            tol = (it + 1) * 2.0 ** -23 * np.maximum(np.abs(ref), 0.01)
            assert np.all(np.abs(mine - ref) <= tol)
            assert np.mean(mine == ref) > 0.5


def test_update_distinguishes_lr_and_momentum():
    """Hand-computed two steps of v <- mu v + g, w <- w - lr v on one element."""
    pl = oracle.plan([1], 1, W.NO_LIMIT, 4)
    sg = np.zeros((1, pl.total_shard_len), np.float32)
    sp, sm = np.zeros_like(sg), np.zeros_like(sg)
    sp[0, 0] = 1.0
    sg[0, 0] = 2.0
    oracle.shard_update(pl, 0, sg, sp, sm, 0.25, 0.5)
    assert (sm[0, 0], sp[0, 0]) == (2.0, 0.5)            # v = 2, w = 1 - 0.25*2
    sg[0, 0] = 4.0
    oracle.shard_update(pl, 0, sg, sp, sm, 0.25, 0.5)
    assert (sm[0, 0], sp[0, 0]) == (5.0, -0.75)          # v = 0.5*2 + 4, w = 0.5 - 0.25*5


# ----------------------------------------------------------------- bf16 gradients
def test_bf16_widening_and_accuracy():
    w = small_workload([1000, 24, 333], 8, 1100 * 2, "bf16", std=1e-3)
    pl = oracle.plan(w.sizes, w.P, w.threshold_bytes, 2)
    flat = [W.make_flat_grad(w, p, 0) for p in range(w.P)]
    grads = [split_np(to_numpy(t), w.sizes) for t in flat]
    # widening: uint16 << 16 equals torch's bfloat16 -> float32 conversion
    for p in range(w.P):
        assert np.array_equal(bf16_bits_to_f32(to_numpy(flat[p])), flat[p].float().numpy())
    sg = np.zeros((w.P, pl.total_shard_len), np.float32)
    oracle.reduce_scatter(pl, -1, grads, sg)
    out = [[np.zeros(n, np.float32) for n in w.sizes] for _ in range(w.P)]
    oracle.all_gather(pl, -1, sg, out)
    from helpers import bf16_ulp
    for l in range(w.n_layers):
        stack = np.stack([flat[p].float().numpy().astype(np.float64)[sum(w.sizes[:l]):sum(w.sizes[:l + 1])]
                          for p in range(w.P)])
        mean = stack.sum(0) / w.P
        err = np.abs(out[0][l].astype(np.float64) - mean)
        assert np.all(err <= w.P * 2.0 ** -24 * np.abs(stack).sum(0) / w.P + 1e-45)
        assert np.all(err <= 2 * bf16_ulp(mean))


# ----------------------------------------------------------------- sub-range calls
def test_shard_ranges_compose():
    """Splitting the work by shard (used to time the oracle on several cores) changes nothing."""
    w = small_workload([300, 17, 2048, 5], 4, 600 * 4, "f32")
    pl = oracle.plan(w.sizes, w.P, w.threshold_bytes, 4)
    grads = grads_np(w, 0)
    a = np.zeros((w.P, pl.total_shard_len), np.float32)
    b = np.zeros_like(a)
    oracle.reduce_scatter(pl, -1, grads, a)
    for s in range(w.P):
        oracle.reduce_scatter(pl, -1, grads, b, shards=range(s, s + 1))
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
