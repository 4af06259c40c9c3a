#!/usr/bin/env python3
"""Benchmark of the transposition hot path on one MI355X.

A "step" is one pass over the 15-case suite (5 workloads; see paper_1603_02297_amd/workloads.py):
plan -> (search) -> kernel, inputs resident in HBM.  Each case is timed with HIP events on the
launch stream over K launches (buffer pairs rotating so the last-level cache cannot hold the
working set); ms_per_step is the sum over cases.  The headline value is the BASELINE metric:
effective bandwidth (bytes read + written) / time per permutation, median over the cases, also
as a fraction of a device-to-device copy of the same size measured in the same run.

Prints ONE JSON line on stdout.  Progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth


def log(msg: str) -> None:
    print(msg, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--max-candidates", type=int, default=0,
                    help="plan search cap: 0 = library default (200), 1 = heuristic only, -1 = all")
    ap.add_argument("--cases", type=str, default="", help="comma-separated substrings of case names (default: all)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-heuristic", action="store_true",
                    help="do not time the heuristic's first candidate separately (keeps a profile to one configuration)")
    ap.add_argument("--plan-cache", type=str, default="",
                    help="file of stored search results (TTC_PLAN_CACHE): cases found there are not searched again")
    return ap.parse_args()


def cpu_baseline(cases, budget_s: float = 25.0):
    """The oracle as it stands, timed on the host cores: every case of the suite once on one
    thread (while the budget lasts) and three times on all available threads (best kept)."""
    import oracle
    from paper_1603_02297_amd import workloads as wl
    cores = len(os.sched_getaffinity(0))
    threads = max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", cores))))
    multi, single, spent = {}, {}, 0.0
    cache = {}
    for c in cases:
        if spent > budget_s:
            break
        if c.config not in cache:
            cache = {c.config: wl.case_inputs(c)}
        A, B0 = cache[c.config]
        best = None
        for _ in range(3):
            B = B0.copy()
            t0 = time.perf_counter()
            oracle.transpose(c.dtype, c.sizes, c.perm, c.alpha, c.beta, A, B, threads)
            dt = time.perf_counter() - t0
            spent += dt
            best = dt if best is None else min(best, dt)
        multi[c.name] = c.traffic_bytes / best / 1e9
        if spent < budget_s * 0.6:
            B = B0.copy()
            t0 = time.perf_counter()
            oracle.transpose(c.dtype, c.sizes, c.perm, c.alpha, c.beta, A, B, 1)
            dt = time.perf_counter() - t0
            spent += dt
            single[c.name] = c.traffic_bytes / dt / 1e9
        log(f"[cpu] {c.name}: {multi[c.name]:.2f} GB/s on {threads} threads"
            + (f", {single[c.name]:.2f} GB/s on 1" if c.name in single else ""))
    return {"value": round(statistics.median(multi.values()), 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"{len(multi)} of {len(cases)} suite cases at full size, best of 3 runs each on {threads} threads "
                      f"(median over cases); {len(single)} of them also once on 1 thread; {spent:.0f} s of CPU wall time",
            "single_thread_median": round(statistics.median(single.values()), 3) if single else None,
            "per_case": {k: round(v, 3) for k, v in multi.items()}}


def measured_traffic(case_name: str):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if there is one."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    try:
        for line in open(path):
            parts = line.split()
            if len(parts) >= 2 and parts[0] == case_name:
                return int(float(parts[1]))
    except OSError:
        pass
    return None


def main() -> int:
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); sharding over several GPUs is not built",
              file=sys.stderr)
        return 2
    import numpy as np
    import torch

    import paper_1603_02297_amd as ttc
    from paper_1603_02297_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    if args.plan_cache:
        os.environ["TTC_PLAN_CACHE"] = os.path.abspath(args.plan_cache)
    ttc.lib()                                   # fail loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    sel = [s for s in args.cases.split(",") if s]
    cases = [c for c in wl.CASES if not sel or any(s in c.name for s in sel)]
    K, W = args.steps, args.warmup

    # bring the clocks up before anything is timed
    warm = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=dev)
    warm2 = torch.empty_like(warm)
    ttc.ttc_time_ceiling(0, warm.numel() * 4, [warm.data_ptr()], [warm2.data_ptr()], stream, 5, 100)
    del warm, warm2

    results = []
    ceil_cache = {}
    for c in cases:
        nbytes = c.tensor_bytes
        npairs = 3 if nbytes < 400e6 else 2
        if nbytes < 64e6:
            npairs = 8
        A_host, B_host = wl.case_inputs(c)
        A_dev = [torch.from_numpy(A_host).to(dev) for _ in range(npairs)]
        B_dev = [torch.from_numpy(B_host).to(dev) for _ in range(npairs)]
        a_ptrs = [t.data_ptr() for t in A_dev]
        b_ptrs = [t.data_ptr() for t in B_dev]
        # ceilings of the same byte size, measured the same way
        if nbytes not in ceil_cache:
            ck = ttc.ttc_time_ceiling(0, nbytes, a_ptrs, b_ptrs, stream, W, K)
            cm = ttc.ttc_time_ceiling(1, nbytes, a_ptrs, b_ptrs, stream, W, K)
            cx = ttc.ttc_time_ceiling(2, nbytes, a_ptrs, b_ptrs, stream, W, K)
            cs = ttc.ttc_time_ceiling(3, nbytes, a_ptrs, b_ptrs, stream, W, K)
            ceil_cache[nbytes] = (2 * nbytes / ck / 1e6, 2 * nbytes / cm / 1e6, 3 * nbytes / cx / 1e6, 2 * nbytes / cs / 1e6)
            for t, h in zip(B_dev, [B_host] * npairs):          # the axpby ceiling changed B
                t.copy_(torch.from_numpy(h))
        copy_k, copy_m, axpby, copy_s = ceil_cache[nbytes]
        d2d = max(copy_k, copy_m, copy_s)           # the fastest known way to copy is the ceiling

        plan = ttc.ttc_plan_create(c.dtype, len(c.sizes), c.sizes, c.perm, c.alpha, c.beta)
        heur = ttc.ttc_plan_get_info(plan)
        ms_heur = None if args.no_heuristic else ttc.ttc_time_execute(plan, a_ptrs, b_ptrs, stream, W, K)
        t0 = time.perf_counter()
        ttc.ttc_plan_tune_pairs(plan, a_ptrs, b_ptrs, stream, args.max_candidates)
        tune_s = time.perf_counter() - t0
        info = ttc.ttc_plan_get_info(plan)
        ms = ttc.ttc_time_execute(plan, a_ptrs, b_ptrs, stream, W, K)
        if ms_heur is not None and ms_heur < ms:   # the search is noisy: never do worse than the heuristic
            ttc.ttc_plan_select_candidate(plan, 0)
            info = ttc.ttc_plan_get_info(plan)
            ms = ms_heur
        ttc.ttc_plan_destroy(plan)
        gbps = c.traffic_bytes / ms / 1e6
        r = {
            "case": c.name, "ms": round(ms, 5), "GBps": round(gbps, 1),
            "frac_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4),
            "frac_d2d_copy": round(gbps / d2d, 4),
            "frac_axpby_stream": round(gbps / axpby, 4) if not c.beta_is_zero else None,
            "d2d_copy_GBps": round(d2d, 1), "copy_kernel_GBps": round(copy_k, 1),
            "memcpy_GBps": round(copy_m, 1), "copy_stream_kernel_GBps": round(copy_s, 1),
            "axpby_stream_GBps": round(axpby, 1),
            "heuristic_GBps": round(c.traffic_bytes / ms_heur / 1e6, 1) if ms_heur is not None else None,
            "candidate": info["candidate_index"], "candidates": info["candidate_count"],
            "tune_s": round(tune_s, 2),
            "kernel_class": "direct" if info["kernel_class"] == ttc.TTC_KERNEL_DIRECT else "lds",
            "tile": info["tile"], "vec": [info["vec_a"], info["vec_b"]], "threads": info["threads"],
            "lds_bytes": info["lds_bytes"], "tiles": info["num_tiles"], "traffic_bytes": c.traffic_bytes,
        }
        results.append(r)
        log(f"[gpu] {c.name}: {gbps:.0f} GB/s = {100 * r['frac_d2d_copy']:.1f}% of D2D copy ({d2d:.0f}), "
            f"heuristic {r['heuristic_GBps'] or 0:.0f}, cand {r['candidate']}/{r['candidates']}, "
            f"{r['kernel_class']} tile {r['tile']} vec {r['vec']} thr {r['threads']}")
        del A_dev, B_dev
        torch.cuda.empty_cache()

    median_gbps = statistics.median(r["GBps"] for r in results)
    median_frac = statistics.median(r["frac_d2d_copy"] for r in results)
    ms_per_step = sum(r["ms"] for r in results)
    # roofline: the staged kernel on the quoted workload (3-D fp32 384^3, full index reversal)
    dom = next((r for r in results if r["case"].startswith("cfg2-f32-p210")), results[0])
    roofline = {"bound": "hbm", "achieved": dom["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(dom["GBps"] / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(dom["case"]),
                "kernel": "box_kernel (" + dom["kernel_class"] + ")", "case": dom["case"],
                "algorithmic_bytes_per_launch": dom["traffic_bytes"], "avg_launch_ms": dom["ms"]}
    out = {
        "metric": "effective HBM bandwidth (bytes read + written / time) per permutation, median over the suite",
        "value": round(median_gbps, 1), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32/f64/c64", "data": "synthetic",
        "config": {"workload": f"{len(results)}-case suite: 2-D/3-D fp32, 4-D fp64, 6-D fp32, 5-D complex64 "
                               "(about 200-630 MB per tensor), one launch of every case per step",
                   "cases": len(results)},
        "median_frac_of_d2d_copy": round(median_frac, 4),
        "roofline": roofline,
        "cases": results,
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(cases)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
