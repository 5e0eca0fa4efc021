#!/usr/bin/env python3
"""Benchmark of the DeAR gradient-aggregation path on one MI355X.

One step = one pass of the whole hot path over every bucket of the workload:
reduce-scatter (pack fused) of all buckets in gradient-ready order, SGD-momentum update of
the owned shards, all-gather (unpack fused) in forward order -- by default one launch per
bucket and phase, back to back on one stream, inputs resident in HBM.

Prints ONE JSON line.  `value` is effective GB/s = algorithmic bytes / wall time, with
algorithmic bytes per step N*(g*P + 4*P + 28): reduce-scatter reads g*P*N and writes 4N,
the update reads 12N and writes 8N, the all-gather reads 4N and writes 4*P*N.

Extra objects on the line:
  step_ms       mean / median / min of the per-step durations (HIP events on the launch stream)
  roofline      the phase that takes the most time, its algorithmic bytes per launch over
                its average launch duration (HIP events on the launch stream), against
                the 8 TB/s HBM peak; `traffic` = HBM bytes per launch from the rocprofv3
                counter runs recorded in profiles/hbm_traffic.json, or null when the kernel
                sources have changed since those runs
  fused_rs_update  the same steps with reduce-scatter and update of a bucket in one kernel
  fused_update_ag  the same steps with update and all-gather of a bucket in one kernel
  cpu_baseline  the CPU oracle as it stands, timed on this host on the same workload (one
                iteration, all buckets unless --sample-buckets says fewer; a baseline, not a
                target); its output is also compared bit for bit with the GPU's first iteration

--launch: per_bucket (default, the DeAR launch granularity), all_buckets (one launch per
phase), graph (the per-bucket launches recorded once into a HIP graph and replayed).
--hbm-probe: instead of the benchmark, print the bare-pattern HBM ceilings (one JSON line
per pattern, see include/dear_probe.h).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import torch

import workloads as W

HBM_PEAK_GBPS = 8000.0
ROOT = os.path.dirname(os.path.abspath(__file__))
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
KERNEL_SOURCES = ["paper_2302_12445_amd/csrc/dear_hip.hip", "paper_2302_12445_amd/csrc/plan.cpp",
                  "paper_2302_12445_amd/csrc/dear_internal.h", "include/dear.h"]


def kernel_source_hash() -> str:
    import hashlib
    h = hashlib.sha256()
    for rel in KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def recorded_traffic(workload: str, phase: str):
    """HBM bytes per launch (average over the buckets) from the rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE runs of this benchmark, each scaled by what the counter reads for a plain 1 GiB
    device copy; None if there is no record for this workload or it was taken with other
    kernel sources than the ones in the tree."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return None
    if rec.get("kernel_source_sha256") != kernel_source_hash():
        return None
    return rec.get("bytes_per_launch", {}).get(workload, {}).get(phase)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="bert_large", choices=W.WORKLOAD_NAMES)
    ap.add_argument("--launch", default="per_bucket", choices=["per_bucket", "all_buckets", "graph"],
                    help="one launch per bucket and phase (the DeAR schedule), one per phase, or the "
                         "per-bucket launches replayed from a HIP graph")
    ap.add_argument("--hbm-probe", action="store_true",
                    help="print the bare-pattern HBM ceilings instead of running the benchmark")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run three plain 1 GiB device copies (torch) so that a counter "
                         "profile of this command holds a dispatch of known traffic")
    ap.add_argument("--sample-buckets", type=int, default=11,
                    help="buckets (from bucket 0) the CPU oracle is timed on")
    return ap.parse_args()


def fill_inputs(em, w, device):
    param = W.make_flat_param(w, device)
    for p in range(w.P):
        em.load_dense(em.params[p], param)
        em.load_dense(em.grads[p], W.make_flat_grad(w, p, 0, device))
    del param
    em.scatter_params(0)
    torch.cuda.synchronize()


class CpuBaseline:
    """The oracle on a bounded sample of the workload (the first n_buckets buckets, all P
    replicas): snapshot() copies the sample's inputs to the host and runs the GPU's first
    iteration, keeping its results; run() times the oracle (single thread, as it stands, and
    split over host threads) after the GPU timing is done and compares the two."""

    def __init__(self, em, w, n_buckets):
        import numpy as np
        import oracle
        self.np, self.oracle, self.em, self.w = np, oracle, em, w
        self.op = oracle.plan(w.sizes, w.P, w.threshold_bytes, w.grad_elem_bytes)
        op = self.op
        self.buckets = list(range(min(n_buckets, op.n_buckets)))
        self.layers = [l for b in self.buckets
                       for l in range(int(op.bucket_first_layer[b]),
                                      int(op.bucket_first_layer[b]) + int(op.bucket_n_layers[b]))]

    def host(self, t):
        np = self.np
        t = t.cpu().contiguous()
        return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()

    def snapshot(self):
        em, w, op = self.em, self.w, self.op
        self.grads = [[None] * w.n_layers for _ in range(w.P)]
        self.params = [[None] * w.n_layers for _ in range(w.P)]
        for p in range(w.P):
            for l in self.layers:
                self.grads[p][l] = self.host(em.grads[p][l])
                self.params[p][l] = self.host(em.params[p][l]).copy()
        # GPU: first iteration from the same state; keep what will be compared
        em.iteration(w.lr, w.momentum, per_bucket=True)
        torch.cuda.synchronize()
        self.gpu_shards = {}
        for b in self.buckets:
            lo, S = int(op.bucket_shard_base[b]), int(op.bucket_shard_len[b])
            self.gpu_shards[b] = [dev[:, lo:lo + S].cpu().numpy() for dev in (em.shard_grad, em.shard_param, em.shard_mom)]
        self.gpu_params = {(p, l): self.host(em.params[p][l]).copy() for p in (0, w.P - 1) for l in self.layers}

    def run(self):
        np, oracle, w, op = self.np, self.oracle, self.w, self.op
        buckets, grads, params = self.buckets, self.grads, self.params
        row = op.total_shard_len
        sg = np.zeros((w.P, row), np.float32)
        sp = np.zeros_like(sg)
        sm = np.zeros_like(sg)
        for b in buckets:
            oracle.scatter_params(op, params, 0, sp, bucket=b)
        n_sample = int(sum(op.bucket_len[b] for b in buckets))
        sample_bytes = n_sample * (w.grad_elem_bytes * w.P + 4 * w.P + 28)

        # the same oracle calls split by shard / receiving worker over host threads (independent
        # work, identical bits): timed first, on scratch copies, as the all-core figure
        from concurrent.futures import ThreadPoolExecutor
        cores = max(1, min(w.P, os.cpu_count() or 1, 16))
        sg2, sp2, sm2 = sg.copy(), sp.copy(), sm.copy()
        params2 = [[None if a is None else a.copy() for a in r] for r in params]
        with ThreadPoolExecutor(cores) as ex:
            t0 = time.perf_counter()
            for b in buckets:
                list(ex.map(lambda s: oracle.reduce_scatter(op, b, grads, sg2, shards=range(s, s + 1)), range(w.P)))
            for b in buckets:
                list(ex.map(lambda s: oracle.shard_update(op, b, sg2, sp2, sm2, w.lr, w.momentum,
                                                          shards=range(s, s + 1)), range(w.P)))
            for b in reversed(buckets):
                list(ex.map(lambda p: oracle.all_gather(op, b, sp2, params2, workers=range(p, p + 1)), range(w.P)))
            dt_all = time.perf_counter() - t0
        del params2

        t0 = time.perf_counter()
        for b in buckets:
            oracle.reduce_scatter(op, b, grads, sg)
        for b in buckets:
            oracle.shard_update(op, b, sg, sp, sm, w.lr, w.momentum)
        for b in reversed(buckets):
            oracle.all_gather(op, b, sp, params)
        dt = time.perf_counter() - t0
        threads_agree = bool(np.array_equal(sp.view(np.uint32), sp2.view(np.uint32)))

        ok = True
        for b in buckets:
            lo, S = int(op.bucket_shard_base[b]), int(op.bucket_shard_len[b])
            for got, ref in zip(self.gpu_shards[b], (sg, sp, sm)):
                ok = ok and np.array_equal(got.view(np.uint32), ref[:, lo:lo + S].view(np.uint32))
        for (p, l), got in self.gpu_params.items():
            ok = ok and np.array_equal(got.view(np.uint32), params[p][l].view(np.uint32))
        return {
            "value": round(sample_bytes / dt / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "buckets %d..%d of %s (%d of %d elements, all %d workers), one iteration, %.1f s" % (
                buckets[0], buckets[-1], w.name, n_sample, w.N, w.P, dt),
            "gpu_matches_oracle_on_sample": bool(ok),
            "all_cores": {"value": round(sample_bytes / dt_all / 1e9, 3), "unit": "GB/s", "cores": cores,
                          "same_bits_as_single_thread": threads_agree},
        }


def run_hbm_probe():
    from paper_2302_12445_amd import hbm_probe
    torch.cuda.init()
    for row in hbm_probe.sweep():
        print(json.dumps(row), flush=True)


def stats(xs):
    xs = sorted(xs)
    n = len(xs)
    med = xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])
    return {"mean": round(sum(xs) / n, 4), "median": round(med, 4), "min": round(xs[0], 4)}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU's share of the path; runs on more than one GPU are "
              "not part of this build (--gpus %d refused)" % args.gpus, file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (there is no CPU path)", file=sys.stderr)
        sys.exit(2)
    if args.hbm_probe:
        run_hbm_probe()
        return

    from paper_2302_12445_amd.emulation import EmulatedWorkers

    device = "cuda:0"
    torch.cuda.set_device(0)
    w = W.get_workload(args.workload)
    em = EmulatedWorkers(w.sizes, w.P, w.grad_dtype, w.threshold_bytes, device)
    fill_inputs(em, w, device)
    nb = em.plan.n_buckets
    mode = args.launch
    per_bucket = mode != "all_buckets"

    baseline = None
    if not args.no_cpu_baseline:
        baseline = CpuBaseline(em, w, args.sample_buckets)
        baseline.snapshot()

    if args.pmc_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=device)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    graph = em.capture_iteration(w.lr, w.momentum, per_bucket=True) if mode == "graph" else None

    def step(marks=None):
        """One pass of the path; marks = [e0, e1, e2, e3] events recorded at the phase boundaries
        (only the modes whose phases follow each other on one stream have inner boundaries)."""
        if marks:
            marks[0].record()
        if mode == "graph":
            graph.replay()
        elif mode == "per_bucket":
            for b in range(nb):
                em.reduce_scatter(b)
            if marks:
                marks[1].record()
            for b in range(nb):
                em.shard_update(b, w.lr, w.momentum)
            if marks:
                marks[2].record()
            for b in reversed(range(nb)):
                em.all_gather(b)
        else:
            em.reduce_scatter(-1)
            if marks:
                marks[1].record()
            em.shard_update(-1, w.lr, w.momentum)
            if marks:
                marks[2].record()
            em.all_gather(-1)
        if marks:
            marks[3].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # timed region: K steps; step and phase boundaries marked with events on the launch stream
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(ev[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # the same steps with reduce-scatter and update of a bucket in one kernel (gbar stays in
    # registers): reported beside the headline, never as `value`
    fev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    buckets = list(range(nb)) if per_bucket else [-1]
    for _ in range(2):
        em.iteration(w.lr, w.momentum, per_bucket=per_bucket, fused_update=True)
    torch.cuda.synchronize()
    f0 = time.perf_counter()
    for k in range(args.steps):
        fev[k][0].record()
        for b in buckets:
            em.reduce_scatter_update(b, w.lr, w.momentum)
        fev[k][1].record()
        for b in reversed(buckets):
            em.all_gather(b)
        fev[k][2].record()
    torch.cuda.synchronize()
    fwall = time.perf_counter() - f0

    bytes_ = w.algorithmic_bytes()
    ms_per_step = wall * 1e3 / args.steps
    value = bytes_["total"] / (wall / args.steps) / 1e9
    launches = nb if per_bucket else 1
    step_ms = [ev[k][0].elapsed_time(ev[k][3]) for k in range(args.steps)]
    line = {
        "metric": "effective aggregation GB/s (RS+update+AG)", "value": round(value, 1), "unit": "GB/s",
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "step_ms": stats(step_ms),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if w.grad_dtype == "f32" else "f32 (gradients stored as bf16, widened exactly)",
        "data": "synthetic",
        "config": {"workload": w.name, "P": w.P, "N": w.N, "n_layers": w.n_layers, "buckets": nb,
                   "threshold_bytes": w.threshold_bytes if w.threshold_bytes != W.NO_LIMIT else "no limit",
                   "grad_dtype": w.grad_dtype, "launch": args.launch,
                   "algorithmic_bytes_per_step": bytes_["total"]},
    }
    if mode in ("per_bucket", "all_buckets"):
        phase_ms = {}
        for i, name in enumerate(("rs", "update", "ag")):
            phase_ms[name] = sum(ev[k][i].elapsed_time(ev[k][i + 1]) for k in range(args.steps)) / args.steps
        kernel_of = {"rs": "reduce_scatter_kernel", "update": "shard_update_kernel", "ag": "all_gather_kernel"}
        dom = max(phase_ms, key=phase_ms.get)
        achieved = bytes_[dom] / (phase_ms[dom] * 1e-3) / 1e9
        line["roofline"] = {
            "bound": "hbm", "kernel": kernel_of[dom], "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": recorded_traffic(w.name, dom) if mode == "per_bucket" else None,
            "traffic_source": "profiles/hbm_traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, calibrated)",
            "bytes_per_launch": bytes_[dom] // launches, "launches_per_step": launches,
            "avg_launch_ms": round(phase_ms[dom] / launches, 4),
            "phases": {n: {"ms": round(phase_ms[n], 4), "GBps": round(bytes_[n] / (phase_ms[n] * 1e-3) / 1e9, 1)}
                       for n in phase_ms},
        }
    else:  # one graph launch: no inner event boundaries, price the whole step
        med = stats(step_ms)["median"]
        line["roofline"] = {"bound": "hbm", "kernel": "whole step (one graph replay)",
                            "achieved": round(bytes_["total"] / (med * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBPS,
                            "unit": "GB/s", "frac": round(bytes_["total"] / (med * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                            "traffic": None}
    f_rs = sum(fev[k][0].elapsed_time(fev[k][1]) for k in range(args.steps)) / args.steps
    f_ag = sum(fev[k][1].elapsed_time(fev[k][2]) for k in range(args.steps)) / args.steps
    fused_rs_bytes = bytes_["rs"] + bytes_["update"] - 8 * w.N   # gbar neither written nor re-read
    line["fused_rs_update"] = {
        "note": "dear_reduce_scatter_update + dear_all_gather; moves 8N fewer bytes than the headline path",
        "ms_per_step": round(fwall * 1e3 / args.steps, 4),
        "effective_GBps_on_headline_bytes": round(bytes_["total"] / (fwall / args.steps) / 1e9, 1),
        "moved_GBps": round((bytes_["total"] - 8 * w.N) / (fwall / args.steps) / 1e9, 1),
        "phases": {"rs_update": {"ms": round(f_rs, 4), "GBps": round(fused_rs_bytes / (f_rs * 1e-3) / 1e9, 1)},
                   "ag": {"ms": round(f_ag, 4), "GBps": round(bytes_["ag"] / (f_ag * 1e-3) / 1e9, 1)}},
    }
    # and with update and all-gather of a bucket in one kernel (moves 4N fewer bytes, but writes the
    # replicas as P interleaved streams)
    gev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    for _ in range(2):
        em.iteration(w.lr, w.momentum, per_bucket=per_bucket, fused_gather=True)
    torch.cuda.synchronize()
    g0 = time.perf_counter()
    for k in range(args.steps):
        gev[k][0].record()
        for b in buckets:
            em.reduce_scatter(b)
        gev[k][1].record()
        for b in reversed(buckets):
            em.update_all_gather(b, w.lr, w.momentum)
        gev[k][2].record()
    torch.cuda.synchronize()
    gwall = time.perf_counter() - g0
    g_ua = sum(gev[k][1].elapsed_time(gev[k][2]) for k in range(args.steps)) / args.steps
    ua_bytes = bytes_["update"] + bytes_["ag"] - 4 * w.N
    line["fused_update_ag"] = {
        "note": "dear_reduce_scatter + dear_update_all_gather; moves 4N fewer bytes than the headline path",
        "ms_per_step": round(gwall * 1e3 / args.steps, 4),
        "phases": {"update_ag": {"ms": round(g_ua, 4), "GBps": round(ua_bytes / (g_ua * 1e-3) / 1e9, 1)}},
    }
    if baseline is not None:  # the CPU leg runs after every GPU timing
        line["cpu_baseline"] = baseline.run()
    print(json.dumps(line), flush=True)
    em.close()


if __name__ == "__main__":
    main()
