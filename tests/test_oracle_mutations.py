"""Are the oracle's pins sharp?  Plausible mistakes are planted in a COPY of the oracle's
source (on the CPU, in a temporary directory), the copy is compiled, and the pins are run
against it: every planted mistake must make at least one pin fail.  The real oracle is
never modified and is restored afterwards."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "dear_oracle.c")

# (name, text in the oracle, replacement, pins expected to notice)
MUTATIONS = [
    ("group closes on equality", "if (cnt > 0 && n[l] > X - tot)", "if (cnt > 0 && n[l] >= X - tot)",
     [pins.test_plan_threshold_extremes, pins.test_plan_worked_example_tiny]),
    ("threshold counted in fp32 elements whatever the gradient type", "x_bytes / g;", "x_bytes / 4;",
     [pins.test_plan_threshold_extremes]),
    ("layers taken first-to-last", "for (int32_t l = L - 1; l >= 0; --l) {  /* gradient-ready order */",
     "for (int32_t l = 0; l < L; ++l) {", [pins.test_plan_worked_example_tiny]),
    ("shard length rounded to 16", "#define ORACLE_SHARD_ALIGN 32", "#define ORACLE_SHARD_ALIGN 16",
     [pins.test_plan_worked_example_tiny]),
    ("shard length not rounded up from d/P", "(bucket_len[b] + P - 1) / P", "bucket_len[b] / P",
     [pins.test_plan_invariants_random]),
    ("fixed-layers group takes one layer too many", "if (held == k) {", "if (held == k + 1) {",
     [pins.test_fixed_layers_worked_example_tiny, pins.test_fixed_layers_invariants_random]),
    ("fixed-layers groups counted from the first layer",
     "for (int32_t l = L - 1; l >= 0; --l) {  /* same arrival order as the threshold rule */",
     "for (int32_t l = 0; l < L; ++l) {", [pins.test_fixed_layers_worked_example_tiny]),
    ("fixed-layers offsets not reset at a new group", "            pos = 0;\n            held = 0;",
     "            held = 0;", [pins.test_fixed_layers_worked_example_tiny]),
    ("ring sum starts at the owner", "grad_at(grad, L, g, (s + 1) % P, l, i);", "grad_at(grad, L, g, (s + 0) % P, l, i);",
     [lambda: pins.test_ring_order_matches_message_passing(4), pins.test_ring_order_is_observable]),
    ("ring runs the other way", "(s + k) % P, l, i);", "(s + 2 * P - k + 2) % P, l, i);",
     [lambda: pins.test_ring_order_matches_message_passing(5)]),
    ("one worker left out of the sum", "for (int32_t k = 2; k <= P; ++k)", "for (int32_t k = 2; k < P; ++k)",
     [lambda: pins.test_exact_rational_three_iterations("f32", 8)]),
    ("average dropped", "out[j] = acc * inv_P;", "out[j] = acc;",
     [lambda: pins.test_exact_rational_three_iterations("f32", 2), pins.test_constant_gradient_averages_to_itself]),
    ("average over P+1", "1.0f / (float)P;", "1.0f / (float)(P + 1);",
     [lambda: pins.test_exact_rational_three_iterations("f32", 8)]),
    ("padding not zero", "out[j] = 0.0f;\n                continue;", "out[j] = 1.0f;\n                continue;",
     [pins.test_signed_zero]),
    ("bf16 widened by 15 bits", "(uint32_t)h << 16", "(uint32_t)h << 15",
     [pins.test_bf16_widening_and_accuracy, lambda: pins.test_exact_rational_three_iterations("bf16", 4)]),
    ("lr and momentum swapped", "float t1 = mu * shard_mom[r + j];", "float t1 = lr * shard_mom[r + j];",
     [pins.test_update_distinguishes_lr_and_momentum]),
    ("step applied with the wrong sign", "shard_param[r + j] - t2;", "shard_param[r + j] + t2;",
     [pins.test_update_distinguishes_lr_and_momentum, pins.test_single_worker_is_plain_sgd_momentum]),
    ("momentum buffer not stored", "shard_mom[r + j] = v;", "(void)v;",
     [pins.test_update_distinguishes_lr_and_momentum]),
    ("all-gather reads the neighbouring shard", "const int64_t s = e / S;\n                const int64_t slot",
     "const int64_t s = (e / S + 1) % P;\n                const int64_t slot",
     [lambda: pins.test_rs_then_ag_is_an_allreduce_average("f32")]),
    ("all-gather slot off by one", "shard_base + e % S;", "shard_base + (e + 1) % S;",
     [lambda: pins.test_rs_then_ag_is_an_allreduce_average("f32")]),
    ("scatter ignores the layer offset", "val = param[(size_t)p * L + l][e - layer_offset[l]];",
     "val = param[(size_t)p * L + l][(e - layer_offset[l]) % n[l] == 0 ? 0 : e - layer_offset[l] - 1];",
     [pins.test_slot_map_is_a_bijection]),
]


def _load(path):
    lib = C.CDLL(path)
    lib.oracle_plan.restype = C.c_int32
    lib.oracle_plan_fixed_layers.restype = C.c_int32
    for name in ("oracle_reduce_scatter", "oracle_shard_update", "oracle_all_gather", "oracle_scatter_params"):
        getattr(lib, name).restype = None
    return lib


@pytest.mark.parametrize("name,old,new,watchers", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, name, old, new, watchers):
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation site not found exactly once: %r" % old
    src = tmp_path / "mutant.c"
    src.write_text(text.replace(old, new))
    so = tmp_path / "libmutant.so"
    subprocess.run(["gcc", *oracle.CFLAGS, "-o", str(so), str(src)], check=True)
    oracle._load()
    real = oracle._lib
    oracle._lib = _load(str(so))
    try:
        caught = False
        for watch in watchers:
            try:
                watch()
            except (AssertionError, ValueError):
                caught = True
                break
        assert caught, "no pin noticed: " + name
    finally:
        oracle._lib = real
    # and the unmodified oracle still passes the same pins
    for watch in watchers:
        watch()
