"""One-GPU shape of the paper's tensor-fusion study (Section VI-G): how the grouping of the
gradients changes the cost of the aggregation and of the overlapped iteration.

Plans compared on one workload (every plan aggregates the same tensors):
    no fusion             one bucket per tensor (buffer size 0)                ["DeAR w/o TF"]
    4 layers per bucket   a fixed number of nearby layers, four as in the paper ["DeAR-NL"]
    5 MB / 25 MB / 64 MB  a fixed buffer size (5 MB is the paper's fixed buffer) ["DeAR-FB"]
    tuned                 the buffer size found by Bayesian optimisation         ["DeAR-BO"]
For each: the aggregation alone (reduce-scatter+update and all-gather of every bucket, one
launch per bucket, full width) and one iteration of the DeAR schedule beside a synthetic
compute stream whose total work is the same for every plan.  Then the cost of the search
itself: trials until Bayesian optimisation, random search and grid search first come within
1 % of the best throughput any of them saw.  One JSON line per row.

    python -m paper_2302_12445_amd.fusion_study --workload resnet50
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> None:
    import workloads as W
    from paper_2302_12445_amd import binding as B
    from paper_2302_12445_amd.emulation import EmulatedWorkers
    from paper_2302_12445_amd.schedule import DearSchedule, spread_gemms
    from paper_2302_12445_amd.tuner import MB, BufferSizeTuner, grid_search, random_search

    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="resnet50", choices=W.WORKLOAD_NAMES)
    ap.add_argument("--gemm-dim", type=int, default=2048)
    ap.add_argument("--forward-gemms", type=int, default=24,
                    help="GEMMs of the whole forward pass (twice as many backward), the same for every plan")
    ap.add_argument("--steps", type=int, default=10, help="iterations averaged per measurement")
    ap.add_argument("--trials", type=int, default=12, help="trials of each search method")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("fusion_study needs a GPU", file=sys.stderr)
        sys.exit(2)

    device = "cuda:0"
    w = W.get_workload(args.workload)
    g = w.grad_elem_bytes
    em = EmulatedWorkers(w.sizes, w.P, w.grad_dtype, 25 * MB, device)
    param = W.make_flat_param(w, device)
    for p in range(w.P):
        em.load_dense(em.params[p], param)
        em.load_dense(em.grads[p], W.make_flat_grad(w, p, 0, device))
    em.scatter_params(0)
    torch.cuda.synchronize()

    ALL_MODES = ("comm_only", "compute_only", "serial", "wfbp", "dear")

    def measure_plan(plan=None, x_bytes=None, modes=ALL_MODES):
        em.replan(threshold_bytes=x_bytes, plan=plan)
        sched = DearSchedule(em, w.lr, w.momentum, args.gemm_dim,
                             ff_gemms=spread_gemms(args.forward_gemms, em.plan),
                             bp_gemms=spread_gemms(2 * args.forward_gemms, em.plan))
        out = {"buckets": em.plan.n_buckets, "streams_concurrent": sched.streams_concurrent}
        for mode in modes:
            out[mode + "_ms"] = round(sched.time_mode(mode, iterations=args.steps, warmup=2), 4)
        return out

    print(json.dumps({"workload": w.name, "P": w.P, "N": w.N, "layers": w.n_layers, "gemm_dim": args.gemm_dim,
                      "forward_gemms": args.forward_gemms, "backward_gemms": 2 * args.forward_gemms,
                      "steps": args.steps}), flush=True)
    rows = [("no fusion", dict(x_bytes=0)),
            ("4 layers per bucket", dict(plan=B.dear_plan_fixed_layers(w.sizes, w.P, 4, g))),
            ("5 MB", dict(x_bytes=5 * MB)), ("25 MB", dict(x_bytes=25 * MB)), ("64 MB", dict(x_bytes=64 * MB))]
    for name, kw in rows:
        print(json.dumps({"plan": name, **measure_plan(**kw)}), flush=True)

    # the search: throughput of the DeAR schedule as a function of the buffer size
    def throughput(x_bytes: int) -> float:
        return 1e3 / measure_plan(x_bytes=int(x_bytes), modes=("dear",))["dear_ms"]

    t0 = time.perf_counter()
    tuner = BufferSizeTuner()
    bx, by = tuner.run(throughput, args.trials)
    bo_s = time.perf_counter() - t0
    bo_trace = list(tuner.ys)
    rx, ry, r_trace = random_search(throughput, args.trials)
    gx, gy, g_trace = grid_search(throughput, args.trials)
    print(json.dumps({"plan": "tuned (%.1f MB)" % (bx / MB), **measure_plan(x_bytes=bx)}), flush=True)

    best = max(by, ry, gy)

    def trials_to(trace):
        for i, v in enumerate(trace):
            if v >= 0.99 * best:
                return i + 1
        return None

    print(json.dumps({"search": {"trials_each": args.trials, "best_it_per_s": round(best, 3),
                                 "bo": {"best_mb": round(bx / MB, 2), "best_it_per_s": round(by, 3),
                                        "trials_to_within_1pct": trials_to(bo_trace),
                                        "seconds_per_trial": round(bo_s / args.trials, 3),
                                        "trace_it_per_s": [round(v, 2) for v in bo_trace]},
                                 "random": {"best_mb": round(rx / MB, 2), "best_it_per_s": round(ry, 3),
                                            "trials_to_within_1pct": trials_to(r_trace)},
                                 "grid": {"best_mb": round(gx / MB, 2), "best_it_per_s": round(gy, 3),
                                          "trials_to_within_1pct": trials_to(g_trace)}}}), flush=True)
    em.close()


if __name__ == "__main__":
    main()
