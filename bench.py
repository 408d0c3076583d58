#!/usr/bin/env python3
"""Benchmark of the robust-aggregation hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic batch of peer
gradients: CenteredClip on every partition (btard_cc_begin / _iterate /
_finish == btard_centered_clip) followed by the verification quantities
(btard_verify_projections).  Inputs are resident in HBM before the timed
region.  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E bandwidth


def recorded_traffic(cfg: int):
    """HBM bytes per launch of the CenteredClip pass as measured with rocprofv3 --pmc
    (FETCH_SIZE and WRITE_SIZE, scaled by a copy kernel of known size); the summary of
    those profiler runs is kept under profiles/.  None if no such run is recorded for
    this configuration: a plain bench run cannot read hardware counters itself."""
    import glob
    import re
    tag = re.compile(r"^traffic_bytes_per_launch cc_pass_kernel cfg%d:\s*([0-9.eE+]+)" % cfg)
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        try:
            with open(path) as fh:
                for line in fh:
                    m = tag.match(line.strip())
                    if m:
                        return float(m.group(1))
        except OSError:
            pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="BASELINE configuration 1..5")
    ap.add_argument("--with-delta", action="store_true",
                    help="also materialise the clipped residuals (optional step S8)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--gram", action="store_true",
                    help="time the step with BTARD_FLAG_GRAM (Gram-matrix iteration with "
                         "streaming fallback) instead of one streaming pass per iteration")
    ap.add_argument("--no-host-sync", action="store_true",
                    help="with --gram: stay asynchronous and enqueue max_iters passes blindly")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain device copy of known size (1 GiB read + 1 GiB written) "
                         "so that HBM counters of a profiler run can be scaled")
    ap.add_argument("--cpu-sample-parts", type=int, default=0,
                    help="partitions the oracle is timed on (0 = pick for ~10-30 s)")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one process simulates all n peers); "
              "--gpus must be 1", file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2

    import paper_2106_11257_amd as btard
    from paper_2106_11257_amd import workloads

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = workloads.make_workload(args.config, device=dev)
    G, off = wl.G, wl.offsets
    n, d, P = wl.n, wl.d, wl.parts
    ws = btard.alloc_workspace(n, P, dev)
    v = torch.empty(d, dtype=torch.float32, device=dev)
    iters = torch.empty(P, dtype=torch.int32, device=dev)
    step_norm = torch.empty(P, dtype=torch.float64, device=dev)
    vout = {k: torch.empty((n, P), dtype=torch.float64, device=dev)
            for k in ("norms", "weights", "proj")}
    vout["colsum"] = torch.empty(P, dtype=torch.float64, device=dev)
    if args.with_delta:
        vout["delta"] = torch.empty((n, d), dtype=torch.float32, device=dev)
    flags = btard.BTARD_FLAG_GRAM if args.gram else btard.BTARD_FLAG_NONE
    prob = btard.make_problem(G, off, wl.tau, wl.eps, wl.max_iters, workspace=ws, flags=flags)
    stream = torch.cuda.current_stream(dev)

    def step(events=None):
        if events is not None:
            events[0].record(stream)
        btard.cc_begin(prob)
        passes = wl.max_iters
        if args.gram:
            btard.cc_gram(prob)
            if not args.no_host_sync:
                passes = btard.cc_remaining(prob)    # one stream synchronisation
        if events is not None:
            events[1].record(stream)
        btard.cc_iterate(prob, 0, passes)
        if events is not None:
            events[2].record(stream)
        btard.cc_finish(prob, passes, v, iters, step_norm)
        if events is not None:
            events[3].record(stream)
        btard.verify_projections(G, off, v, wl.tau, wl.seed_z, want_delta=args.with_delta,
                                 workspace=ws, out=vout)
        if events is not None:
            events[4].record(stream)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(evs[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    seg = [[evs[k][s].elapsed_time(evs[k][s + 1]) for k in range(args.steps)] for s in range(4)]
    seg_ms = [sum(x) / len(x) for x in seg]                   # begin, iterate, finish, verify

    it = iters.cpu().tolist()
    sizes = [off[j + 1] - off[j] for j in range(P)]
    applied = sum(sizes[j] * max(it[j], 0) for j in range(P))
    # passes the device made over partition j: one per update, plus the pass that found an
    # update below eps when the partition stopped before the cap
    passes = sum(sizes[j] * (max(it[j], 0) + (1 if 0 <= it[j] < wl.max_iters else 0))
                 for j in range(P))
    agg_bytes = 4.0 * n * applied
    value = agg_bytes / (ms_per_step * 1e-3) / 1e9
    cc_only = agg_bytes / (sum(seg_ms[0:3]) * 1e-3) / 1e9

    # roofline of the dominant kernel (the CenteredClip pass): algorithmic bytes = every peer
    # gradient element of a running partition read once per launch, n*d_j*4
    pass_bytes_total = 4.0 * n * passes
    launches = wl.max_iters
    t_iter_s = seg_ms[1] * 1e-3
    achieved = pass_bytes_total / t_iter_s / 1e9 if t_iter_s > 0 else 0.0
    roofline = {
        "bound": "hbm", "kernel": "cc_pass_kernel",
        "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBPS, 4),
        "traffic": recorded_traffic(args.config),
        "bytes_per_launch": pass_bytes_total / launches,
        "launches_per_step": launches,
        "avg_launch_us": round(t_iter_s / launches * 1e6, 2),
    }
    verify_bytes = 4.0 * (n + 1) * d
    out = {
        "metric": "aggregated peer-gradient GB/s per CenteredClip iteration + % of HBM roofline",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": wl.name, "n": n, "d": d, "parts": P, "tau": wl.tau,
                   "eps": wl.eps, "max_iters": wl.max_iters,
                   "iters_min": min(it), "iters_max": max(it),
                   "seed_inputs": wl.seed_inputs, "seed_z": wl.seed_z,
                   "with_delta": bool(args.with_delta),
                   "mode": "gram + streaming fallback" if args.gram else "streaming"},
        "segments_ms": {"cc_begin": round(seg_ms[0], 4), "cc_iterate": round(seg_ms[1], 4),
                        "cc_finish": round(seg_ms[2], 4), "verify": round(seg_ms[3], 4)},
        "cc_only_GBps": round(cc_only, 1),
        "verify_GBps": round(verify_bytes / (seg_ms[3] * 1e-3) / 1e9, 1),
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        import numpy as np
        import oracle
        # bounded sample: the first k partitions of the same workload, same iteration rule
        k = args.cpu_sample_parts
        if k <= 0:
            budget = 6.0e10       # element-updates, roughly 10-30 s of oracle time
            per_part = 2.0 * n * max(sizes) * wl.max_iters
            k = int(max(1, min(P, budget // max(per_part, 1))))
        lo, hi = off[0], off[k]
        sub = G[:, lo:hi].contiguous().cpu().numpy()
        sub_off = [o - lo for o in off[: k + 1]]
        times = []
        while True:                      # at least one run; repeat short ones (best of <= 5)
            t0 = time.perf_counter()
            _, ito, _, _ = oracle.centered_clip(sub, sub_off, wl.tau, wl.eps, wl.max_iters)
            times.append(time.perf_counter() - t0)
            if sum(times) > 10.0 or len(times) >= 5:
                break
        t_cpu = min(times)
        cpu_bytes = 4.0 * n * sum((sub_off[j + 1] - sub_off[j]) * max(int(ito[j]), 0)
                                  for j in range(k))
        out["cpu_baseline"] = {
            "value": round(cpu_bytes / t_cpu / 1e9, 3), "unit": "GB/s",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"CenteredClip on partitions 0..{k - 1} of {P} of the same workload "
                      f"({(hi - lo)} of {d} coordinates, all {n} peers, same tau/eps/max_iters), "
                      f"best of {len(times)} runs: {t_cpu:.2f} s",
        }
        assert [int(x) for x in ito] == it[:k], "oracle and GPU iteration counts differ"
        del np

    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
