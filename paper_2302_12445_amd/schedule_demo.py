"""One-GPU demonstration of the DeAR schedule (paper Section III-B): reduce-scatter kernels
on a side stream under a synthetic back-propagation GEMM stream, all-gather kernels under
the next iteration's feed-forward GEMM stream.  Prints one JSON line with the time of each
part alone, of the serial / WFBP-like / DeAR schedules, the hidden fraction
(t_compute + t_comm - t_overlapped) / min(t_compute, t_comm) and the paper's ideal
iteration times max(t_ff, t_ag) + max(t_bp, t_rs) and t_ff + max(t_bp, t_ar)
(Section VI-I).

    python -m paper_2302_12445_amd.schedule_demo --workload resnet50
"""
from __future__ import annotations

import argparse
import json
import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> None:
    import workloads as W
    from paper_2302_12445_amd.emulation import EmulatedWorkers
    from paper_2302_12445_amd.schedule import DearSchedule, overlap_report

    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="resnet50", choices=W.WORKLOAD_NAMES)
    ap.add_argument("--gemm-dim", type=int, default=4096)
    ap.add_argument("--ff-gemms", type=int, default=1, help="forward GEMMs per bucket")
    ap.add_argument("--bp-gemms", type=int, default=2, help="backward GEMMs per bucket")
    ap.add_argument("--iterations", type=int, default=10)
    ap.add_argument("--overlap-workgroups", type=int, default=256,
                    help="grid bound of reduce-scatter/update while they overlap compute (0 = unbounded)")
    ap.add_argument("--overlap-workgroups-ag", type=int, default=256,
                    help="grid bound of the all-gather while it overlaps compute")
    ap.add_argument("--wave-priority", type=int, default=3, help="wave priority of bounded reduce-scatter/update")
    ap.add_argument("--wave-priority-ag", type=int, default=0, help="wave priority of the bounded all-gather")
    ap.add_argument("--unfused", action="store_true", help="reduce-scatter and update as two kernels")
    ap.add_argument("--gemm-dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--blas", default="default", choices=["default", "hipblaslt", "rocblas"],
                    help="library torch takes its GEMM kernels from")
    ap.add_argument("--trace-iterations", type=int, default=0,
                    help="after the report, run this many DeAR iterations only (for a kernel trace)")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("schedule_demo needs a GPU", file=sys.stderr)
        sys.exit(2)

    if args.blas != "default":
        torch.backends.cuda.preferred_blas_library("cublaslt" if args.blas == "hipblaslt" else "cublas")
    device = "cuda:0"
    w = W.get_workload(args.workload)
    em = EmulatedWorkers(w.sizes, w.P, w.grad_dtype, w.threshold_bytes, device)
    param = W.make_flat_param(w, device)
    for p in range(w.P):
        em.load_dense(em.params[p], param)
        em.load_dense(em.grads[p], W.make_flat_grad(w, p, 0, device))
    em.scatter_params(0)
    torch.cuda.synchronize()

    sched = DearSchedule(em, w.lr, w.momentum, args.gemm_dim, args.ff_gemms, args.bp_gemms,
                         overlap_workgroups=args.overlap_workgroups,
                         overlap_workgroups_ag=args.overlap_workgroups_ag,
                         fused_update=not args.unfused,
                         gemm_dtype=torch.float32 if args.gemm_dtype == "f32" else torch.bfloat16,
                         wave_priority=args.wave_priority, wave_priority_ag=args.wave_priority_ag)
    rep = overlap_report(sched, args.iterations)
    rep["config"] = {"workload": w.name, "P": w.P, "buckets": em.plan.n_buckets, "gemm_dim": args.gemm_dim,
                     "ff_gemms_per_bucket": args.ff_gemms, "bp_gemms_per_bucket": args.bp_gemms,
                     "gemm_dtype": args.gemm_dtype, "blas": args.blas, "fused_update": not args.unfused,
                     "overlap_workgroups": [args.overlap_workgroups, args.overlap_workgroups_ag],
                     "wave_priority": [args.wave_priority, args.wave_priority_ag]}
    print(json.dumps(rep), flush=True)
    for _ in range(args.trace_iterations):
        sched.iteration("dear")
    if args.trace_iterations:
        sched._forward(True)   # the forward pass the last iteration's all-gathers run under
    sched.synchronize()
    em.close()


if __name__ == "__main__":
    main()
