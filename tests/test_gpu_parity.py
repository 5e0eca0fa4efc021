"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element
on the same seeded inputs.  fp32 gradients: bit-exact.  bf16 gradients: the shard values
are fp32 on both sides and the ring order is fixed, so bits are compared too (the stated
acceptance floor of 2 bf16 ULP is asserted separately as the weaker bound).  Bucket and
shard indexing: bit-exact through the positions of the values."""
from __future__ import annotations

import ctypes as C
import sys

import numpy as np
import pytest
import torch

import oracle
import workloads as W
from helpers import bf16_ulp, small_workload, split_np, to_numpy

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _bits(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a).view(np.uint32)


class Pair:
    """The same problem on both sides: EmulatedWorkers on the GPU, numpy + oracle on the CPU."""

    def __init__(self, w: W.Workload, layout="flat", plan=None, oracle_plan=None):
        """plan / oracle_plan: the two sides' own plans when the grouping is not the
        workload's threshold rule (each side builds its plan with its own planner)."""
        from paper_2302_12445_amd.emulation import EmulatedWorkers
        self.w = w
        self.em = EmulatedWorkers(w.sizes, w.P, w.grad_dtype, w.threshold_bytes, DEV, layout, plan)
        self.op = oracle_plan if oracle_plan is not None else oracle.plan(
            w.sizes, w.P, w.threshold_bytes, w.grad_elem_bytes)
        row = self.op.total_shard_len
        assert row == self.em.plan.total_shard_len
        self.sg = np.zeros((w.P, row), np.float32)
        self.sp = np.zeros_like(self.sg)
        self.sm = np.zeros_like(self.sg)
        flat = W.make_flat_param(w)
        self.params = [split_np(to_numpy(flat).copy(), w.sizes) for _ in range(w.P)]
        for p in range(w.P):
            self.em.load_dense(self.em.params[p], flat.to(DEV))
        self.grads = None

    def seed_shards(self):
        oracle.scatter_params(self.op, self.params, 0, self.sp)
        self.em.shard_param.fill_(float("nan"))
        self.em.scatter_params(0)
        self.compare_buffer("scatter_params", self.em.shard_param, self.sp)

    def load_grads(self, it, flats=None):
        w = self.w
        if flats is None:
            flats = [W.make_flat_grad(w, p, it) for p in range(w.P)]
        self.grads = [split_np(to_numpy(f), w.sizes) for f in flats]
        for p in range(w.P):
            self.em.load_dense(self.em.grads[p], flats[p].to(DEV))

    def compare_buffer(self, what, dev: torch.Tensor, host: np.ndarray):
        got = dev.cpu().numpy()
        same = _bits(got) == _bits(host)
        if not same.all():
            idx = np.argwhere(~same)[:5]
            raise AssertionError("%s: %d of %d slots differ, first at %s: got %s want %s" % (
                what, (~same).sum(), same.size, idx.tolist(),
                [got[tuple(i)] for i in idx], [host[tuple(i)] for i in idx]))

    def compare_params(self, what):
        for p in range(self.w.P):
            for l in range(self.w.n_layers):
                got = self.em.params[p][l].cpu().numpy()
                want = self.params[p][l]
                if not np.array_equal(_bits(got), _bits(want)):
                    bad = np.argwhere(_bits(got) != _bits(want))[:5].ravel()
                    raise AssertionError("%s: worker %d layer %d differs at %s: got %s want %s" % (
                        what, p, l, bad.tolist(), got[bad], want[bad]))

    def oracle_iteration(self):
        w = self.w
        oracle.reduce_scatter(self.op, -1, self.grads, self.sg)
        oracle.shard_update(self.op, -1, self.sg, self.sp, self.sm, w.lr, w.momentum)
        oracle.all_gather(self.op, -1, self.sp, self.params)

    def run(self, iterations=3, per_bucket=True, poison=True, stream=None, fused=False, width=0, priority=0,
            fused_gather=False):
        w, em = self.w, self.em
        em.set_max_workgroups(width)
        em.set_wave_priority(priority)
        self.seed_shards()
        for it in range(iterations):
            self.load_grads(it)
            if poison:  # nothing may survive from before: every slot and element is rewritten
                em.shard_grad.fill_(float("nan"))
                for p in range(w.P):
                    for t in em.params[p]:
                        t.fill_(float("nan"))
            torch.cuda.synchronize()
            em.iteration(w.lr, w.momentum, per_bucket=per_bucket, stream=stream, fused_update=fused,
                         fused_gather=fused_gather)
            torch.cuda.synchronize()
            self.oracle_iteration()
            if not fused:  # the fused kernel never writes the averaged gradient
                self.compare_buffer("shard_grad it%d" % it, em.shard_grad, self.sg)
            self.compare_buffer("shard_mom it%d" % it, em.shard_mom, self.sm)
            self.compare_buffer("shard_param it%d" % it, em.shard_param, self.sp)
            self.compare_params("params it%d" % it)

    def close(self):
        self.em.close()


RAGGED = [4097, 3, 8191, 4096, 1, 12289, 7, 30001, 64, 513]


def test_tiny_config_three_iterations():
    say("case: tiny config, per-bucket launches")
    pr = Pair(W.get_workload("tiny"))
    assert pr.em.plan.n_buckets == 5
    pr.run(3, per_bucket=True)
    pr.close()


def test_tiny_config_all_buckets_in_one_launch():
    say("case: tiny config, bucket=-1 launches, separate allocations")
    pr = Pair(W.get_workload("tiny"), layout="separate")
    pr.run(3, per_bucket=False)
    pr.close()


@pytest.mark.parametrize("P", [1, 2, 3, 4, 5, 8, 9, 12, 16, 24, 64])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_ragged_layers_all_worker_counts(P, dtype):
    say("case: ragged layers P=%d %s" % (P, dtype))
    g = 4 if dtype == "f32" else 2
    w = small_workload(RAGGED, P, 21000 * g, dtype, index=10 + P)
    pr = Pair(w)
    assert pr.em.plan.n_buckets >= 3
    pr.run(2 if P > 16 else 3, per_bucket=(P % 2 == 0))
    pr.close()


@pytest.mark.parametrize("P", [1, 2, 3, 4, 8, 9, 12, 64])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fused_reduce_scatter_update(P, dtype):
    """dear_reduce_scatter_update must leave the same bits in the parameter and momentum
    shards as dear_reduce_scatter followed by dear_shard_update (both compared with the oracle)."""
    say("case: fused RS+update P=%d %s" % (P, dtype))
    g = 4 if dtype == "f32" else 2
    w = small_workload(RAGGED + [70001, 2], P, 36000 * g, dtype, index=110 + P)
    pr = Pair(w)
    pr.run(3, per_bucket=(P % 2 == 1), fused=True)
    pr.close()


@pytest.mark.parametrize("width", [1, 3, 64, 256])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_bounded_grid_gives_the_same_bits(width, dtype):
    """A bounded grid (workgroups striding over the work items) is only a launch shape."""
    say("case: bounded grid width=%d %s" % (width, dtype))
    g = 4 if dtype == "f32" else 2
    w = small_workload(RAGGED + [300_001], 4, 40000 * g, dtype, index=120 + width)
    pr = Pair(w)
    pr.run(2, per_bucket=(width != 3), fused=(width == 64), width=width, priority=width % 4)
    pr.close()


def test_fused_tiny_and_many_tiles():
    say("case: fused RS+update, tiny config and many tiles")
    pr = Pair(W.get_workload("tiny"))
    pr.run(3, fused=True)
    pr.close()
    w = small_workload([1_000_003, 5, 65_537, 250_001, 2], 8, 1_100_000 * 2, "bf16", index=42, std=1e-3)
    pr = Pair(w)
    pr.run(2, fused=True)
    pr.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_single_bucket_and_no_fusion(dtype):
    g = 4 if dtype == "f32" else 2
    for thr in (W.NO_LIMIT, 0):
        say("case: threshold %d %s" % (thr, dtype))
        w = small_workload(RAGGED, 4, thr, dtype, index=31)
        pr = Pair(w)
        assert pr.em.plan.n_buckets == (1 if thr else len(RAGGED))
        pr.run(2)
        pr.close()
    del g


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_many_tiles_per_shard(dtype):
    """Several hundred tiles per shard, layer starts that are odd in the bucket, a layer
    spanning several shards."""
    say("case: many tiles %s" % dtype)
    g = 4 if dtype == "f32" else 2
    w = small_workload([1_000_003, 5, 65_537, 250_001, 2], 8, 1_100_000 * g, dtype, index=41, std=1e-3)
    pr = Pair(w)
    pr.run(2)
    pr.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layers_per_bucket", [4, 3])
def test_fixed_layers_plan(dtype, layers_per_bucket):
    """The fixed-number-of-layers grouping of the tensor-fusion study (Section VI-G) drives the
    same kernels: the library's plan and the oracle's own fixed-layers plan, bit for bit over
    the shards of every worker and the parameters of every replica, three iterations."""
    import paper_2302_12445_amd as dear
    say("case: fixed-layers plan, %d layers per bucket, %s" % (layers_per_bucket, dtype))
    g = 4 if dtype == "f32" else 2
    w = small_workload(RAGGED, 4, W.NO_LIMIT, dtype, index=51)
    plan = dear.dear_plan_fixed_layers(w.sizes, w.P, layers_per_bucket, g)
    op = oracle.plan_fixed_layers(w.sizes, w.P, layers_per_bucket, g)
    assert plan.n_buckets == op.n_buckets == -(-len(RAGGED) // layers_per_bucket)
    pr = Pair(w, plan=plan, oracle_plan=op)
    pr.run(3)
    pr.run(1, fused=True)
    pr.close()


def test_fixed_layers_plan_resnet50_shape():
    """Four layers per bucket (the paper's number) on the ResNet-50 tensor list: 41 buckets of
    very uneven size, one launch per bucket."""
    import paper_2302_12445_amd as dear
    say("case: fixed-layers plan, resnet50 shape")
    w = W.get_workload("resnet50")
    plan = dear.dear_plan_fixed_layers(w.sizes, w.P, 4, 4)
    op = oracle.plan_fixed_layers(w.sizes, w.P, 4, 4)
    assert plan.n_buckets == op.n_buckets == 41
    pr = Pair(w, plan=plan, oracle_plan=op)
    pr.run(1)
    pr.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("P,width", [(1, 0), (4, 0), (8, 5), (13, 0)])
def test_fused_update_all_gather_gives_the_same_bits(P, width, dtype):
    """dear_update_all_gather: update and all-gather of a bucket in one kernel; shard buffers
    (padding slots included) and every replica's parameters as from the two separate calls."""
    say("case: fused update+all-gather P=%d width=%d %s" % (P, width, dtype))
    g = 4 if dtype == "f32" else 2
    w = small_workload(RAGGED + [100_003], P, 30000 * g, dtype, index=140 + P)
    pr = Pair(w)
    pr.run(3, fused_gather=True, width=width, priority=P % 4)
    pr.run(1, per_bucket=False, fused_gather=True)
    pr.close()


def test_signed_zero_nan_inf():
    say("case: signed zeros, NaN, Inf")
    w = small_workload([37, 4100], 4, W.NO_LIMIT, "f32", index=61)
    pr = Pair(w)
    pr.seed_shards()
    flats = [torch.full((w.N,), -0.0) for _ in range(4)]
    pr.load_grads(0, flats)
    pr.em.shard_grad.fill_(float("nan"))
    pr.em.reduce_scatter(-1)
    oracle.reduce_scatter(pr.op, -1, pr.grads, pr.sg)
    pr.compare_buffer("negative zeros", pr.em.shard_grad, pr.sg)
    assert (_bits(pr.sg[0, :37]) == 0x80000000).all()
    flats = [W.make_flat_grad(w, p, 0) for p in range(4)]
    flats[1][5] = float("inf")
    flats[2][6] = float("-inf")
    flats[3][7] = float("nan")
    flats[0][4000] = float("inf")
    flats[1][4000] = float("-inf")
    pr.load_grads(0, flats)
    pr.em.reduce_scatter(-1)
    oracle.reduce_scatter(pr.op, -1, pr.grads, pr.sg)
    got = pr.em.shard_grad.cpu().numpy()
    assert np.array_equal(np.isnan(got), np.isnan(pr.sg))
    ok = ~np.isnan(got)
    assert np.array_equal(_bits(got[ok]), _bits(pr.sg[ok]))
    pr.close()


def test_denormals_are_kept():
    say("case: denormal gradients")
    w = small_workload([4096 + 9], 2, W.NO_LIMIT, "f32", index=62)
    pr = Pair(w)
    pr.seed_shards()
    tiny = np.float32(1e-41)
    flats = [torch.full((w.N,), float(tiny)), torch.full((w.N,), float(tiny) * 3)]
    pr.load_grads(0, flats)
    pr.em.reduce_scatter(-1)
    oracle.reduce_scatter(pr.op, -1, pr.grads, pr.sg)
    assert pr.sg[0, 0] != 0.0
    pr.compare_buffer("denormals", pr.em.shard_grad, pr.sg)
    pr.close()


def test_bf16_within_two_ulp_of_exact_mean():
    """The acceptance floor stated for bf16 gradients, checked against the exact mean."""
    say("case: bf16 two-ULP floor")
    w = small_workload([5000, 123], 8, W.NO_LIMIT, "bf16", index=63, std=1e-3)
    pr = Pair(w)
    pr.seed_shards()
    flats = [W.make_flat_grad(w, p, 0) for p in range(8)]
    pr.load_grads(0, flats)
    pr.em.reduce_scatter(-1)
    pr.em.shard_param.copy_(pr.em.shard_grad)
    pr.em.all_gather(-1)
    torch.cuda.synchronize()
    mean = torch.stack([f.double() for f in flats]).sum(0).numpy() / 8
    got = pr.em.dense(pr.em.params[3]).cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - mean) <= 2 * bf16_ulp(mean))
    pr.close()


def test_side_stream_and_argument_errors():
    import paper_2302_12445_amd as dear
    from paper_2302_12445_amd import binding
    say("case: side stream, error codes")
    w = small_workload(RAGGED, 4, 21000 * 4, "f32", index=71)
    pr = Pair(w)
    side = torch.cuda.Stream()
    pr.run(2, stream=side)
    em = pr.em
    lib = dear.load_library()
    h = em.ctx.handle
    sg, sp, sm = em.shard_grad.data_ptr(), em.shard_param.data_ptr(), em.shard_mom.data_ptr()
    nb = em.plan.n_buckets
    assert lib.dear_reduce_scatter(h, nb, C.c_void_p(sg), None) == binding.DEAR_ERANGE
    assert lib.dear_reduce_scatter(h, -2, C.c_void_p(sg), None) == binding.DEAR_ERANGE
    assert lib.dear_reduce_scatter(h, 0, C.c_void_p(sg + 64), None) == binding.DEAR_EALIGN
    assert lib.dear_reduce_scatter(h, 0, None, None) == binding.DEAR_EINVAL
    assert lib.dear_all_gather(h, nb, C.c_void_p(sp), None) == binding.DEAR_ERANGE
    assert lib.dear_all_gather(h, 0, C.c_void_p(sp + 4), None) == binding.DEAR_EALIGN
    assert lib.dear_shard_update(h, 0, C.c_void_p(sg), C.c_void_p(sg), C.c_void_p(sm), 0.1, 0.9, None) == binding.DEAR_EINVAL
    assert lib.dear_shard_update(h, nb, C.c_void_p(sg), C.c_void_p(sp), C.c_void_p(sm), 0.1, 0.9, None) == binding.DEAR_ERANGE
    assert lib.dear_scatter_params(h, 4, C.c_void_p(sp), None) == binding.DEAR_ERANGE
    assert lib.dear_scatter_params(h, -1, C.c_void_p(sp), None) == binding.DEAR_ERANGE
    torch.cuda.synchronize()
    # nothing was launched by the failing calls: state still equals the oracle's
    pr.compare_buffer("after errors", em.shard_param, pr.sp)
    pr.close()


def test_resnet50_config_one_iteration():
    """Config 2 at full size: 161 tensors, 5 buckets of up to 76 small tensors, P = 8."""
    say("case: resnet50 full size")
    pr = Pair(W.get_workload("resnet50"))
    assert pr.em.plan.n_buckets == 5
    pr.run(1)
    pr.close()


@pytest.mark.parametrize("name", ["densenet201", "inception_v4"])
def test_many_small_tensors_full_size(name):
    """The paper's other two CNNs at full size: 604 / 449 tensors, hundreds of them a few
    hundred elements long, so most tiles are short runs and edge vectors."""
    say("case: %s full size" % name)
    pr = Pair(W.get_workload(name))
    pr.run(1, fused=(name == "inception_v4"))
    pr.close()


def test_random_configurations():
    """Seeded random layer lists, worker counts, thresholds, gradient types, launch widths,
    fused or not, flat or separate allocations: each compared bit for bit with the oracle."""
    rng = np.random.default_rng(20230212)
    picks = [1, 2, 3, 5, 7, 8, 31, 32, 33, 63, 64, 65, 100, 255, 256, 257, 1000, 1023, 1024, 1025,
             4095, 4096, 4097, 8191, 8192, 8193, 12289, 20000, 40001]
    for case in range(40):
        L = int(rng.integers(1, 14))
        sizes = [int(rng.choice(picks)) for _ in range(L)]
        if rng.random() < 0.3:
            sizes[int(rng.integers(0, L))] = int(rng.integers(50000, 300000))
        P = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 9, 12, 16, 17, 24, 33]))
        dtype = str(rng.choice(["f32", "bf16"]))
        g = 4 if dtype == "f32" else 2
        thr = int(rng.choice([0, 64 * g, 5000 * g, 30000 * g, 200000 * g, W.NO_LIMIT]))
        width = int(rng.choice([0, 0, 1, 2, 7, 64, 256]))
        fused = bool(rng.random() < 0.5)
        per_bucket = bool(rng.random() < 0.5)
        layout = str(rng.choice(["flat", "separate"]))
        say("case: random %d sizes=%s P=%d %s thr=%d width=%d fused=%d per_bucket=%d %s" % (
            case, sizes, P, dtype, thr, width, fused, per_bucket, layout))
        pr = Pair(small_workload(sizes, P, thr, dtype, index=1000 + case), layout=layout)
        pr.run(2, per_bucket=per_bucket, fused=fused, width=width, priority=case % 4)
        pr.close()
