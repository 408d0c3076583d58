#!/usr/bin/env python3
"""Benchmark of the robust-aggregation hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic batch of peer
gradients, resident in HBM before the timed region: CenteredClip on every
partition to its stopping rule, then the verification quantities (norms,
weights, projections on the seed-derived direction z, column sums).

Two ways of running the same step are timed in one invocation:

  headline  the fastest path of the library: the CenteredClip iteration on each
            partition's Gram matrix (BTARD_FLAG_GRAM: one pass over the data for
            all iterations, streaming passes only where its accuracy cannot be
            guaranteed), one stream synchronisation to skip passes nobody
            needs, and the last CenteredClip pass merged with the verification
            pass (btard_cc_finish_verify).  `value`, `ms_per_step` and
            `roofline` (its longest kernel) describe this path.
  streaming one pass over the data per CenteredClip iteration (the per-iteration
            kernel, cc_pass_kernel), then btard_cc_finish and
            btard_verify_projections.  Reported under "streaming"; its roofline
            is the per-iteration HBM fraction.

Both produce the same v, iteration counts and verification outputs (tests).

With no --config the line describes the largest configuration (5: 16 peers, 1.3 G
coordinates, an 84 GB slab) and carries a "per_config" object with the same figures, in
short, for configurations 1-4 (measured with fewer steps).  --config k measures that
configuration alone.

`value` is an algorithmic-equivalent rate: bytes of peer gradients aggregated per
CenteredClip iteration (4 n sum_j d_j iters_j) per second of the whole step.  On the
headline path the iteration runs on the Gram matrix, so the slab itself is read only twice
per step and `value` can exceed the HBM peak; "physical" gives the bytes a step really
moves per second, and `roofline` the dominant kernel against the HBM (or matrix) peak.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5]
                  [--mode both|headline|streaming]
Prints one JSON line.
"""
from __future__ import annotations

import argparse
import gc
import glob
import json
import os
import re
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E bandwidth


def recorded_traffic(kernel: str, cfg: int):
    """HBM bytes per launch of `kernel` as measured with rocprofv3 --pmc (FETCH_SIZE and
    WRITE_SIZE, scaled by a copy kernel of known size); the summaries of those profiler runs
    are kept under profiles/.  None if no such run is recorded for this configuration: a
    plain bench run cannot read hardware counters itself."""
    if _OTHER_LENGTH:
        return None
    tag = re.compile(r"^traffic_bytes_per_launch %s cfg%d:\s*([0-9.eE+]+)" % (re.escape(kernel), cfg))
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


_OTHER_LENGTH = False      # set by --d: the recorded counter runs are for the full lengths


TRAFFIC_NOTE = ("traffic: HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of "
                "this command, recorded in profiles/*.md (a bench run cannot read counters itself)")


def mean(xs):
    return sum(xs) / len(xs) if xs else 0.0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=0,
                    help="BASELINE configuration 1..5 alone (default: 5 as the headline, and "
                         "configurations 1-4 in short under per_config)")
    ap.add_argument("--d", type=int, default=0,
                    help="with --config: the same recipe at another vector length (a sensitivity "
                         "run, e.g. a length that is not a power of two; not a BASELINE workload)")
    ap.add_argument("--entry", action="store_true",
                    help="with --config: print that configuration's entry of the default run's "
                         "per_config block (the default run starts one such process per configuration)")
    ap.add_argument("--no-per-config", action="store_true",
                    help="with no --config: leave out configurations 1-4")
    ap.add_argument("--mode", choices=("both", "headline", "streaming"), default="both")
    ap.add_argument("--host-sync", action="store_true",
                    help="headline path: look at what the Gram iteration left undone (one "
                         "stream synchronisation) before the last pass, instead of running the "
                         "last pass at once and checking afterwards")
    ap.add_argument("--with-delta", action="store_true",
                    help="streaming path: also materialise the clipped residuals (optional)")
    ap.add_argument("--preclip", type=float, default=0.0,
                    help="pre-clipping radius lambda of BTARD-Clipped-SGD as a multiple of the "
                         "median row norm of partition 0 (0: none, the headline configuration)")
    ap.add_argument("--no-graph", action="store_true",
                    help="do not also time the headline step replayed as one HIP graph")
    ap.add_argument("--baselines", action="store_true",
                    help="also time the baseline aggregators of Sec. 4.1 on the same slab "
                         "(coordinate-wise median; geometric median, 20 Weiszfeld iterations)")
    ap.add_argument("--hashes", action="store_true",
                    help="also time the partition hashes (SHA-256 tree) of the slab and of v")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain device copies of known size (1 GiB read + 1 GiB "
                         "written) so that HBM counters of a profiler run can be scaled")
    args = ap.parse_args()
    if args.d > 0:
        if not args.config:
            print("bench.py: --d needs --config", file=sys.stderr)
            return 2
        global _OTHER_LENGTH
        _OTHER_LENGTH = True

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
    def measure(cfg, steps, warmup, brief, cpu_baseline):
        """All figures of one configuration.  brief: the short form used for the per_config
        entries (no comparison variants, no extras).  cpu_baseline: thread counts to time
        the oracle with (0: all the host cores; empty: not at all)."""
        wl = workloads.make_workload(cfg, device=dev, d=(args.d if args.d > 0 and args.config else None))
        G, off = wl.G, wl.offsets
        n, d, P, M = wl.n, wl.d, wl.parts, wl.max_iters
        sizes = [off[j + 1] - off[j] for j in range(P)]
        ws = btard.alloc_workspace(n, P, dev)
        v = torch.empty(d, dtype=torch.float32, device=dev)
        iters = torch.empty(P, dtype=torch.int32, device=dev)
        step_norm = torch.empty(P, dtype=torch.float64, device=dev)
        vout = {k: torch.empty((n, P), dtype=torch.float64, device=dev)
                for k in ("norms", "weights", "proj")}
        vout["colsum"] = torch.empty(P, dtype=torch.float64, device=dev)
        if args.with_delta:
            vout["delta"] = torch.empty((n, d), dtype=torch.float32, device=dev)
        factors = torch.empty((n, P), dtype=torch.float64, device=dev)
        vout_preclipped = dict(vout, factors=torch.empty_like(factors))
        stream = torch.cuda.current_stream(dev)
        slab_bytes = 4.0 * n * d
        lam = 0.0
        if args.preclip > 0.0:
            row_norms = G[:, off[0]:off[1]].double().norm(dim=1)
            lam = float(torch.tensor(args.preclip * float(row_norms.median()), dtype=torch.float32))

        if args.copy_calibration and not brief:
            src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
            dst = torch.empty_like(src)
            for _ in range(3):
                dst.copy_(src)
            torch.cuda.synchronize()
            del src, dst

        def rec(events, i):
            if events is not None:
                events[i].record(stream)

        # ---- the two ways of running a step; events (if given) mark the segment boundaries
        prob_s = btard.make_problem(G, off, wl.tau, wl.eps, M, workspace=ws, preclip=lam)
        seg_s = ("cc_begin", "cc_iterate", "cc_finish", "verify")

        def step_streaming(events=None):
            rec(events, 0)
            btard.cc_begin(prob_s)
            rec(events, 1)
            btard.cc_iterate(prob_s, 0, M)
            rec(events, 2)
            btard.cc_finish(prob_s, M, v, iters, step_norm)
            rec(events, 3)
            if lam > 0.0:
                # (a verifying peer holds the factors of the rows it clipped: they are handed
                # over, not measured again)
                btard.cc_preclip_factors(prob_s, factors)
                btard.verify_projections_preclipped(G, off, v, wl.tau, wl.seed_z, factors=factors,
                                                    want_delta=args.with_delta, workspace=ws,
                                                    out=vout_preclipped)
            else:
                btard.verify_projections(G, off, v, wl.tau, wl.seed_z, want_delta=args.with_delta,
                                         workspace=ws, out=vout)
            rec(events, 4)

        # (the Gram kernels also do the work of btard_cc_begin where they can: P <= 255)
        headline_flags = btard.BTARD_FLAG_GRAM | btard.BTARD_FLAG_GRAM_BEGINS
        prob_h = btard.make_problem(G, off, wl.tau, wl.eps, M, workspace=ws,
                                    flags=headline_flags, preclip=lam)
        seg_h = ("cc_begin", "gram_matrix", "gram_iterate", "fallback_passes", "finish_verify")
        fallback_passes = []

        def step_headline(events=None, host_sync=False):
            # Without host_sync nothing waits for the device: the last pass is enqueued right
            # behind the Gram iteration, and whether that iteration finished every partition
            # (it does on the benchmark configurations) is read back after the timed region,
            # together with the results.  If it did not, the step is completed by
            # complete_headline() and the synchronised variant is what gets reported.
            rec(events, 0)
            rec(events, 1)                                           # (no launch of its own any more)
            btard.cc_gram_matrix(prob_h)
            rec(events, 2)
            btard.cc_gram_iterate(prob_h)
            rec(events, 3)
            passes = 0
            if host_sync:
                passes = btard.cc_remaining(prob_h)                  # one synchronisation
                fallback_passes.append(passes)
                btard.cc_iterate(prob_h, 0, passes)
            rec(events, 4)
            btard.cc_finish_verify(prob_h, passes, wl.seed_z, v, iters, step_norm, out=vout)
            rec(events, 5)

        def complete_headline():
            """After an unsynchronised step: the passes the Gram iteration left, if any."""
            passes = btard.cc_remaining(prob_h)
            if passes > 0:
                btard.cc_iterate(prob_h, 0, passes)
                btard.cc_finish_verify(prob_h, passes, wl.seed_z, v, iters, step_norm, out=vout)
                torch.cuda.synchronize()
            return passes

        def run(step, nseg, steps):
            for _ in range(warmup):
                step()
            torch.cuda.synchronize()
            evs = [[torch.cuda.Event(enable_timing=True) for _ in range(nseg + 1)]
                   for _ in range(steps)]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for k in range(steps):
                step(evs[k])
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            seg_ms = [mean([evs[k][s].elapsed_time(evs[k][s + 1]) for k in range(steps)])
                      for s in range(nseg)]
            return (t1 - t0) * 1e3 / steps, seg_ms

        def work_done():
            it = iters.cpu().tolist()
            applied = sum(sizes[j] * max(it[j], 0) for j in range(P))
            # passes a per-iteration path makes over partition j: one per update, plus the pass
            # that finds an update below eps when the partition stops before the cap
            passes = sum(sizes[j] * (max(it[j], 0) + (1 if 0 <= it[j] < M else 0)) for j in range(P))
            return it, 4.0 * n * applied, 4.0 * n * passes

        out = {
            "metric": "aggregated peer-gradient GB/s per CenteredClip iteration + % of HBM roofline",
            "value": None, "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
            "ms_per_step": None, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f64", "data": "synthetic",
            "config": {"workload": wl.name, "n": n, "d": d, "parts": P, "tau": wl.tau, "eps": wl.eps,
                       "max_iters": M, "seed_inputs": wl.seed_inputs, "seed_z": wl.seed_z},
        }
        if lam > 0.0:
            out["config"]["preclip_lambda"] = lam

        # ---- streaming path: the per-iteration kernel
        if args.mode in ("both", "streaming"):
            steps_s = steps if args.mode == "streaming" else max(3, steps // 4)
            ms, seg = run(step_streaming, 4, steps_s)
            it, agg_bytes, pass_bytes = work_done()
            t_iter = seg[1] * 1e-3
            achieved = pass_bytes / t_iter / 1e9
            streaming = {
                "value": round(agg_bytes / (ms * 1e-3) / 1e9, 1), "unit": "GB/s",
                "ms_per_step": round(ms, 4), "steps": steps_s,
                "segments_ms": {k: round(x, 4) for k, x in zip(seg_s, seg)},
                "cc_only_GBps": round(agg_bytes / (sum(seg[0:3]) * 1e-3) / 1e9, 1),
                "verify_GBps": round(4.0 * (n + 1) * d / (seg[3] * 1e-3) / 1e9, 1),
                "roofline": {
                    "bound": "hbm", "kernel": "cc_pass_kernel", "achieved": round(achieved, 1),
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                    "traffic": recorded_traffic("cc_pass_kernel", cfg),
                    "bytes_per_launch": pass_bytes / M, "launches_per_step": M,
                    "avg_launch_us": round(t_iter / M * 1e6, 2)},
            }
            out["streaming"] = streaming
            out["config"].update({"iters_min": min(it), "iters_max": max(it)})
            if args.mode == "streaming":
                out["value"], out["ms_per_step"] = streaming["value"], streaming["ms_per_step"]
                out["roofline"] = streaming["roofline"]
                out["config"]["mode"] = "streaming: one pass over the data per iteration"

        # ---- headline path
        if args.mode in ("both", "headline"):
            def headline_numbers(host_sync, steps):
                fallback_passes.clear()
                ms, seg = run(lambda ev=None: step_headline(ev, host_sync), 5, steps)
                left = 0 if host_sync else complete_headline()
                return ms, seg, left

            # (the Gram formulation serves n <= 64; beyond that every pass is a streaming pass
            # and the step cannot skip the look at what is left)
            synced = args.host_sync or n > 64
            ms, seg, left = headline_numbers(synced, steps)
            unsync_note = None
            if left > 0:
                # the Gram iteration handed partitions over: only the synchronised variant does
                # the whole job inside the timed region
                unsync_note = f"unsynchronised attempt left {left} passes to run; reporting the synchronised path"
                ms, seg, _ = headline_numbers(True, steps)
                synced = True
            it, agg_bytes, pass_bytes = work_done()
            fb = max(fallback_passes) if fallback_passes else 0
            last = "cc_finish_verify_kernel"       # light body where the Gram iteration finished
            kernels = {
                # name: (ms between the HIP events around its launch(es), algorithmic bytes)
                "gram_pass_kernel": (seg[1], slab_bytes),
                last: (seg[4], slab_bytes + 4.0 * d),
            }
            if fb > 0:
                # partitions the Gram iteration did not finish (or n > 16): per-iteration passes
                kernels["cc_pass_kernel"] = (seg[3], pass_bytes)
            # The kernels by themselves.  An event pair inside a step brackets a whole call (the
            # last one also launches verify_finish_kernel) and adds a few microseconds of marker
            # latency, so the two long kernels are also timed back to back on the finished state
            # of the last step, K launches between two HIP events on the launch stream: the Gram
            # pass alone, and the pair (Gram pass, fused last pass) as it runs in a step -- the
            # last pass finds the end of the slab still in the memory-side cache -- from which
            # the last pass is the difference.
            def back_to_back(fn, reps=16):
                fn()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(reps):
                    fn()
                e1.record(stream)
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / reps

            alone = {}
            if fb == 0 and n <= 64:
                reps = 16 if slab_bytes < 4e9 else 4

                def pair():
                    btard.cc_gram_matrix(prob_h)
                    btard.debug_last_pass(prob_h, 0, wl.seed_z, v)
                # (three rounds, the median of each: one round's difference is at the mercy of a
                # single slow launch)
                t_grams, t_lasts = [], []
                for _ in range(3):
                    t_g = back_to_back(lambda: btard.cc_gram_matrix(prob_h), reps)
                    t_grams.append(t_g)
                    t_lasts.append(back_to_back(pair, reps) - t_g)
                alone = {"gram_pass_kernel": sorted(t_grams)[1], last: sorted(t_lasts)[1]}
                # (v and the outputs are as the last step left them: the same values again)
            table = {}
            for name, (t_ms, nbytes) in kernels.items():
                ach = nbytes / (t_ms * 1e-3) / 1e9 if t_ms > 0 else 0.0
                table[name] = {"us": round(t_ms * 1e3, 2), "algorithmic_bytes": nbytes,
                               "achieved_GBps": round(ach, 1),
                               "frac_of_hbm_peak": round(ach / HBM_PEAK_GBPS, 4)}
                if name in alone:
                    # "us": between the events around the call in the timed steps;
                    # "kernel_us": the kernel alone, back to back -- what the roofline uses
                    k_ms = alone[name]
                    ach = nbytes / (k_ms * 1e-3) / 1e9
                    table[name].update({"kernel_us": round(k_ms * 1e3, 2),
                                        "achieved_GBps": round(ach, 1),
                                        "frac_of_hbm_peak": round(ach / HBM_PEAK_GBPS, 4)})
                    kernels[name] = (k_ms, nbytes)
            dominant = max(kernels, key=lambda name: kernels[name][0])
            out["value"] = round(agg_bytes / (ms * 1e-3) / 1e9, 1)
            out["ms_per_step"] = round(ms, 4)
            out["segments_ms"] = {k: round(x, 4) for k, x in zip(seg_h, seg)}
            out["kernels"] = table
            out["roofline"] = {
                "bound": "hbm", "kernel": dominant, "achieved": table[dominant]["achieved_GBps"],
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": table[dominant]["frac_of_hbm_peak"],
                "traffic": recorded_traffic(dominant, cfg),
                "bytes_per_launch": table[dominant]["algorithmic_bytes"], "launches_per_step": 1,
                "avg_launch_us": table[dominant].get("kernel_us", table[dominant]["us"])}
            if dominant == "gram_pass_kernel" and 16 < n <= 64:
                # 16 < n <= 64: the Gram pass is a dense fp64 contraction bound by the matrix unit:
                # one 16 x 16 x 4 instruction (2048 flop) per pair of 16-peer groups and 4 coordinates
                nb = (n + 15) // 16
                flops = nb * (nb + 1) // 2 * 512.0 * d
                t_s = kernels[dominant][0] * 1e-3
                out["roofline"] = {
                    "bound": "mfma", "kernel": dominant, "achieved": round(flops / t_s / 1e12, 2),
                    "peak": 78.6, "unit": "TFLOP/s", "frac": round(flops / t_s / 1e12 / 78.6, 4),
                    "traffic": recorded_traffic(dominant, cfg),
                    "flops_per_launch": flops, "launches_per_step": 1,
                    "avg_launch_us": table[dominant].get("kernel_us", table[dominant]["us"]),
                    "hbm_frac": table[dominant]["frac_of_hbm_peak"]}
            # what a step really moves: the slab once for the Gram matrices, the slab and v once
            # for the last pass, and whatever per-iteration passes the Gram iteration left
            phys_bytes = sum(nbytes for (_t, nbytes) in kernels.values()) if n <= 64 else \
                pass_bytes + slab_bytes + 4.0 * d
            out["value_kind"] = ("algorithmic-equivalent: bytes of peer gradients aggregated per "
                                 "CenteredClip iteration (4 n sum_j d_j iters_j) per second of the "
                                 "whole step (CenteredClip to its stopping rule + verification); "
                                 "not comparable with the HBM peak, see physical and roofline")
            out["physical"] = {"bytes_per_step": phys_bytes, "unit": "GB/s"}
            out["config"].update({
                "iters_min": min(it), "iters_max": max(it),
                "mode": "headline: Gram-matrix iteration (streaming fallback), "
                        + ("one host sync before the last pass, " if synced else
                           "no host sync inside the step (completeness read back afterwards), ")
                        + "fused finish+verify",
                "fallback_passes_per_step": fb})
            if unsync_note:
                out["config"]["note"] = unsync_note
            if not synced and not args.no_graph:
                # The same four launches captured once into a HIP graph and replayed: nothing in
                # the unsynchronised step depends on the host, so a replay is the whole step.
                # (The library clears its state with kernels, never with memset nodes.)
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    # a problem description that carries the capturing stream
                    prob_g = btard.make_problem(G, off, wl.tau, wl.eps, M, workspace=ws,
                                                flags=headline_flags, preclip=lam)
                    btard.cc_gram_matrix(prob_g)
                    btard.cc_gram_iterate(prob_g)
                    btard.cc_finish_verify(prob_g, 0, wl.seed_z, v, iters, step_norm, out=vout)
                for _ in range(warmup):
                    graph.replay()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(steps):
                    graph.replay()
                torch.cuda.synchronize()
                ms_g = (time.perf_counter() - t0) * 1e3 / steps
                if btard.cc_remaining(prob_g) == 0 and iters.cpu().tolist() == it:
                    out["eager_launches"] = {"value": out["value"], "unit": "GB/s",
                                             "ms_per_step": out["ms_per_step"]}
                    out["value"] = round(agg_bytes / (ms_g * 1e-3) / 1e9, 1)
                    out["ms_per_step"] = round(ms_g, 4)
                    out["config"]["mode"] += ", the step's 4 launches replayed as one HIP graph"
                    out["config"]["note_timing"] = ("value and ms_per_step: graph replays; segments_ms "
                                                    "and kernels[].us: HIP events around the calls of "
                                                    "the eager steps; kernels[].kernel_us and roofline: "
                                                    "the kernel alone, launched back to back")
            if not synced and args.mode == "both" and not brief:
                # the same step with the synchronisation, for comparison
                ms2, seg2, _ = headline_numbers(True, max(3, steps // 2))
                out["with_host_sync"] = {
                    "value": round(agg_bytes / (ms2 * 1e-3) / 1e9, 1), "unit": "GB/s",
                    "ms_per_step": round(ms2, 4),
                    "segments_ms": {k: round(x, 4) for k, x in zip(seg_h, seg2)}}

            rate = out["physical"]["bytes_per_step"] / (out["ms_per_step"] * 1e-3) / 1e9
            out["physical"].update({"GBps": round(rate, 1),
                                    "frac_of_hbm_peak": round(rate / HBM_PEAK_GBPS, 4)})
            out["roofline"]["traffic_note"] = TRAFFIC_NOTE

        # ---- one GPU's share if the partitions were spread over n GPUs: partition 0 alone (all n
        # peers' rows of its columns), the shape one aggregator of the paper's protocol works on
        # (in the default run only: with --config the run is what the profiler commands under
        # profiles/ trace, and these smaller launches of the same kernels would blur their averages)
        if not brief and not args.config and n <= 64 and args.mode != "streaming" and P > 1:
            G1 = G[:, off[0]:off[1]]
            d1 = off[1] - off[0]
            off1 = [0, d1]
            ws1 = btard.alloc_workspace(n, 1, dev)
            v1 = torch.empty(d1, dtype=torch.float32, device=dev)
            it1 = torch.empty(1, dtype=torch.int32, device=dev)
            sn1 = torch.empty(1, dtype=torch.float64, device=dev)
            out1 = {k: torch.empty((n, 1), dtype=torch.float64, device=dev)
                    for k in ("norms", "weights", "proj")}
            out1["colsum"] = torch.empty(1, dtype=torch.float64, device=dev)
            prob1 = btard.make_problem(G1, off1, wl.tau, wl.eps, M, workspace=ws1,
                                       flags=headline_flags, preclip=lam)

            def share_step():
                btard.cc_gram_matrix(prob1)
                btard.cc_gram_iterate(prob1)
                passes1 = btard.cc_remaining(prob1)          # (host sync: the share is timed with it)
                btard.cc_iterate(prob1, 0, passes1)
                btard.cc_finish_verify(prob1, passes1, wl.seed_z, v1, it1, sn1, out=out1)
            for _ in range(2):
                share_step()
            torch.cuda.synchronize()
            reps = 5
            t0 = time.perf_counter()
            for _ in range(reps):
                share_step()
            torch.cuda.synchronize()
            ms1 = (time.perf_counter() - t0) * 1e3 / reps
            iters1 = int(it1.cpu()[0])
            out["one_gpu_share"] = {
                "what": "partition 0 alone: the n x d/P slab one aggregator holds when the partitions "
                        "are spread over P GPUs (no communication timed); whole step with one host "
                        "synchronisation",
                "d": d1, "iters": iters1, "ms_per_step": round(ms1, 4),
                "value": round(4.0 * n * d1 * max(iters1, 0) / (ms1 * 1e-3) / 1e9, 1), "unit": "GB/s",
                "physical_GBps": round((2.0 * 4.0 * n * d1 + 4.0 * d1) / (ms1 * 1e-3) / 1e9, 1)}
            del G1, v1, ws1

        # ---- a plain grid-stride kernel on the same slab: what a straightforward kernel reaches
        # with the traffic of a pass (rows read) and of the last pass (rows read, one row written)
        if not brief:
            def timed_us(fn, reps):
                fn()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(reps):
                    fn()
                e1.record(stream)
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / reps * 1e3
            vp = torch.empty(d, dtype=torch.float32, device=dev)
            reps = 3 if slab_bytes > 4e9 else 20
            best_r, best_w = None, None
            for blocks in (2048, 4096, 16384):
                t_r = timed_us(lambda: btard.debug_plain_stream(G, None, blocks), reps)
                t_w = timed_us(lambda: btard.debug_plain_stream(G, vp, blocks), reps)
                if best_r is None or t_r < best_r[0]:
                    best_r = (t_r, blocks)
                if best_w is None or t_w < best_w[0]:
                    best_w = (t_w, blocks)
            del vp
            out["plain_kernel"] = {
                "what": "btard_debug_plain_stream: a grid-stride kernel, one 16-byte load per row and "
                        "thread, fp32 sums, non-temporal loads and stores; best of 2048, 4096 and "
                        "16384 workgroups",
                "rows_read": {"us": round(best_r[0], 2), "workgroups": best_r[1],
                              "GBps": round(slab_bytes / (best_r[0] * 1e-6) / 1e9, 1)},
                "rows_read_one_written": {"us": round(best_w[0], 2), "workgroups": best_w[1],
                                          "GBps": round((slab_bytes + 4.0 * d) / (best_w[0] * 1e-6) / 1e9, 1)},
            }
            # the method's kernels beside it (time of the plain kernel with the same traffic /
            # time of the kernel: above 1 = faster than the plain kernel), which does not depend
            # on how fast this particular machine's memory is
            rel = {}
            if ("streaming" in out and out["streaming"]["roofline"].get("avg_launch_us")
                    and out["streaming"]["roofline"]["bytes_per_launch"] >= 0.999 * slab_bytes):
                rel["cc_pass_kernel"] = round(best_r[0] / out["streaming"]["roofline"]["avg_launch_us"], 3)
            kk = out.get("kernels", {})
            if "gram_pass_kernel" in kk:
                rel["gram_pass_kernel"] = round(best_r[0] / kk["gram_pass_kernel"].get("kernel_us", kk["gram_pass_kernel"]["us"]), 3)
            if "cc_finish_verify_kernel" in kk:
                rel["cc_finish_verify_kernel"] = round(best_w[0] / kk["cc_finish_verify_kernel"].get("kernel_us", kk["cc_finish_verify_kernel"]["us"]), 3)
            out["plain_kernel"]["plain_time_over_kernel_time"] = rel

        # ---- the baseline aggregators on the same slab (not part of the headline step)
        if args.baselines and not brief:
            def timed(fn, reps):
                fn()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(reps):
                    fn()
                e1.record(stream)
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / reps
            vm = torch.empty(d, dtype=torch.float32, device=dev)
            t_med = timed(lambda: btard.coordinate_median(G, vm), 5)
            gm_iters = 20
            t_gm = timed(lambda: btard.geometric_median(G, off, 1e-6, 0.0, gm_iters, workspace=ws), 2)
            med_bytes = slab_bytes + 4.0 * d
            out["baselines"] = {
                "coordinate_median": {
                    "us": round(t_med * 1e3, 2), "algorithmic_bytes": med_bytes,
                    "achieved_GBps": round(med_bytes / (t_med * 1e-3) / 1e9, 1),
                    "frac_of_hbm_peak": round(med_bytes / (t_med * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)},
                "geometric_median": {
                    "iterations": gm_iters, "ms": round(t_gm, 4),
                    # gm_iters passes and the pass that writes v
                    "us_per_pass": round(t_gm * 1e3 / (gm_iters + 1), 2),
                    "achieved_GBps": round(slab_bytes * (gm_iters + 1) / (t_gm * 1e-3) / 1e9, 1)},
            }

        # ---- the commitments hash(g_i[j]) and hash(v[j]) (not part of the headline step)
        if args.hashes and not brief:
            hws = torch.empty(max(btard.hash_workspace_bytes(n, off), 256), dtype=torch.uint8, device=dev)
            dig = torch.empty((n, P, 32), dtype=torch.uint8, device=dev)
            dig_v = torch.empty((1, P, 32), dtype=torch.uint8, device=dev)

            def timed_ms(fn, reps):
                fn()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(reps):
                    fn()
                e1.record(stream)
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / reps
            t_h = timed_ms(lambda: btard.partition_hashes(G, off, hws, dig), 3)
            t_v = timed_ms(lambda: btard.partition_hashes(v, off, hws, dig_v), 3)
            # 1402 vector instructions per 64-byte SHA-256 block (counted in the kernel's code);
            # blocks by the tree's rule: chunks of 1024 bytes, then runs of 32 digests
            def sha_blocks(nbytes):
                return (nbytes + 8) // 64 + 1

            def tree_blocks(words):
                nbytes = 4 * words
                cnt = max(1, -(-nbytes // 1024))
                total = (cnt - 1) * sha_blocks(1024) + sha_blocks(nbytes - (cnt - 1) * 1024)
                while cnt > 1:
                    groups = -(-cnt // 32)
                    total += (groups - 1) * sha_blocks(32 * 32) + sha_blocks((cnt - (groups - 1) * 32) * 32)
                    cnt = groups
                return total
            blocks = n * sum(tree_blocks(w) for w in sizes)
            lane_ops = blocks * 1402.0
            alu_peak = 256 * 4 * 16 * 2.4e9          # lanes x clock: one 32-bit instruction per lane and cycle
            out["hashes"] = {
                "slab_ms": round(t_h, 4), "slab_GBps": round(slab_bytes / (t_h * 1e-3) / 1e9, 1),
                "aggregate_ms": round(t_v, 4),
                "roofline": {"bound": "alu", "achieved": round(lane_ops / (t_h * 1e-3) / 1e12, 2),
                             "peak": round(alu_peak / 1e12, 2), "unit": "T lane-instructions/s",
                             "frac": round(lane_ops / (t_h * 1e-3) / alu_peak, 4)},
            }

        # ---- the oracle on the host cores, as a baseline only
        if cpu_baseline:
            import oracle
            k = int(max(1, min(P, 6.0e10 // max(2.0 * n * max(sizes) * M, 1))))
            lo, hi = off[0], off[k]
            sub = torch.empty((n, hi - lo), dtype=torch.float32, pin_memory=True)
            for i in range(n):
                sub[i].copy_(G[i, lo:hi], non_blocking=True)
            torch.cuda.synchronize()
            sub = sub.numpy()
            sub_off = [o - lo for o in off[: k + 1]]
            all_threads = oracle.num_threads()

            def time_oracle(threads, budget_s):
                oracle.set_num_threads(threads)
                times = []
                while True:                  # at least one run; repeat short ones (best of <= 15)
                    t0 = time.perf_counter()
                    scale = oracle.preclip_scales(sub, sub_off, lam)[0] if lam > 0.0 else None
                    _, ito, _, _ = oracle.centered_clip(sub, sub_off, wl.tau, wl.eps, M, scale=scale)
                    times.append(time.perf_counter() - t0)
                    if sum(times) > budget_s or len(times) >= 15:
                        break
                oracle.set_num_threads(all_threads)
                t_cpu = min(times)
                cpu_bytes = 4.0 * n * sum((sub_off[j + 1] - sub_off[j]) * max(int(ito[j]), 0)
                                          for j in range(k))
                assert [int(x) for x in ito] == iters.cpu().tolist()[:k], \
                    "oracle and GPU iteration counts differ"
                return {
                    "value": round(cpu_bytes / t_cpu / 1e9, 3), "unit": "GB/s",
                    "cores": threads, "kind": "oracle",
                    "sample": f"CenteredClip (no verification) on partitions 0..{k - 1} of {P} of "
                              f"the same workload ({hi - lo} of {d} coordinates, all {n} peers, same "
                              f"tau/eps/max_iters), best of {len(times)} runs: {t_cpu:.2f} s",
                }
            for threads in cpu_baseline:
                key = "cpu_baseline" if threads in (0, all_threads) else f"cpu_baseline_{threads}_thread"
                out[key] = time_oracle(threads if threads > 0 else all_threads,
                                       10.0 if threads != 1 else 4.0)
            del sub
        return out

    def fits(cfg):
        name, n_c, d_c, _tau, _m = workloads._SHAPES[cfg]
        free, _total = torch.cuda.mem_get_info()
        return free >= 4.0 * n_c * d_c * 1.08 + (2 << 30)

    def measured(*a, release=True):
        r = measure(*a)
        gc.collect()                      # (the slab and the outputs of this configuration)
        if release:
            torch.cuda.empty_cache()
        return r

    cpu = [] if args.no_cpu_baseline else [0]
    if args.config and args.entry:
        # one entry of the default run's per_config block (see below)
        c = args.config
        small = c in (1, 2)          # (more, shorter steps: their kernels are tens of microseconds)
        r = measured(c, 40 if small else max(4, args.steps // 2),
                     10 if small else max(2, args.warmup), True, [1] if (c == 1 and cpu) else [])
        keys = ("value", "ms_per_step", "physical", "roofline", "kernels", "segments_ms")
        out = {"workload": r["config"]["workload"],
               "iters_min": r["config"].get("iters_min"), "iters_max": r["config"].get("iters_max"),
               "mode": r["config"].get("mode")}
        out.update({k: r[k] for k in keys if k in r})
        if "streaming" in r:
            out["streaming"] = {k: r["streaming"][k] for k in ("ms_per_step", "roofline")}
        for k in r:
            if k.startswith("cpu_baseline"):
                out[k] = r[k]
    elif args.config:
        out = measured(args.config, args.steps, args.warmup, False,
                       cpu + ([1] if cpu and args.config == 1 else []))
    else:
        # The largest configuration that fits this GPU is the headline and is measured first,
        # on the device as it was handed over.  The others are measured in short (same recipe,
        # fewer steps), each in a process of its own, while this process still holds the
        # headline's memory (in torch's allocator): a slab that is allocated after others have
        # been allocated and given back to the driver -- by this process or by an earlier one --
        # lands where every kernel on it runs 2-7 % slower (64 MiB slab after the 84 GB one:
        # 17.3 against 16.1 us per pass; the 84 GB slab after the four others, in this or in
        # other processes: 26.5-27.7 against 25.8-26.3 ms per step).
        head = next((c for c in (5, 4, 3, 2, 1) if fits(c)), 1)
        out = measured(head, args.steps, args.warmup, False, cpu, release=False)
        per = {}
        if not args.no_per_config:
            import subprocess
            for c in (1, 2, 3, 4, 5):
                if c == head or not fits(c):
                    continue
                cmd = [sys.executable, os.path.abspath(__file__), "--config", str(c), "--entry",
                       "--steps", str(args.steps), "--warmup", str(args.warmup)]
                if args.no_cpu_baseline:
                    cmd.append("--no-cpu-baseline")
                try:
                    done = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE,
                                          timeout=300, check=False)
                    lines = [l for l in done.stdout.decode(errors="replace").splitlines()
                             if l.startswith("{")]
                    if done.returncode == 0 and lines:
                        per[f"cfg{c}"] = json.loads(lines[-1])
                    else:
                        per[f"cfg{c}"] = {"error": f"exit status {done.returncode}",
                                          "stderr": done.stderr.decode(errors="replace")[-400:]}
                except subprocess.TimeoutExpired:
                    per[f"cfg{c}"] = {"error": "no result within 300 s"}
        if per:
            out["per_config"] = per
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
