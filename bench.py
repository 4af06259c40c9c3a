#!/usr/bin/env python3
"""Benchmark of the transposition hot path on one MI355X.

A "step" is one pass over the 15-case suite (5 workloads; see paper_1603_02297_amd/workloads.py):
plan -> stored or searched configuration -> kernel, inputs resident in HBM.  Each case is timed with HIP
events on the launch stream over K launches (buffer pairs rotating so that the last-level cache cannot
hold the working set); ms_per_step is the sum over cases.  The headline value is the effective bandwidth
(bytes read + written) / time per permutation, median over the cases, also as a fraction of a
device-to-device copy of the same size measured next to each case.

What is timed is what is checked: after the timing, the selected configuration runs once more from a fresh
B and the result is compared element by element with the CPU oracle (the run that also gives the
cpu_baseline figure); a mismatch makes the exit status non-zero.

Plans come from the tracked store of search results (paper_1603_02297_amd/plans/gfx950_suite.txt) so that
the bench, the profiles under profiles/ and the full-size parity tests run one and the same configuration;
a case the store does not hold is searched in the run.  --search ignores the store.

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
LAST_LEVEL_CACHE_BYTES = 256 * 1024 * 1024
STEADY_MS = 12.0                # untimed work before a timing, so that the GPU has left its idle state
MAX_WARM = 400                  # ... but no more launches than this (microsecond kernels)
DEFAULT_STORE = os.path.join(ROOT, "paper_1603_02297_amd", "plans", "gfx950_suite.txt")


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
    ap.add_argument("--no-cpu", action="store_true",
                    help="skip the oracle: no cpu_baseline figure and no check of the results")
    ap.add_argument("--no-heuristic", action="store_true",
                    help="do not time the heuristic's first candidate separately (keeps a profile to one configuration)")
    ap.add_argument("--plan-cache", type=str, default=DEFAULT_STORE,
                    help="file of stored search results: cases found there are not searched again; several files, comma "
                         "separated: every stored plan of a case is timed and the fastest kept (with --store-plans: a way "
                         "to validate searches from several machines on one more)")
    ap.add_argument("--search", action="store_true", help="search every case in the run, whatever the store holds")
    ap.add_argument("--problem", type=str, default="",
                    help="time this problem instead of the suite: dtype:sizes:perm[:alpha:beta], e.g. f32:85x85x85x85:3210:1:0 "
                         "(what profiles/ uses for shapes outside the suite; not a bench line)")
    ap.add_argument("--force-class", type=str, default="", choices=("", "direct", "lds", "rows", "micro"),
                    help="run the best-ranked candidate of this kernel family instead of the stored or searched plan")
    ap.add_argument("--store-plans", type=str, default="",
                    help="append what the run selected for every case to this file (the format of --plan-cache)")
    return ap.parse_args()


def ulp_distance(x, y) -> int:
    """Largest distance in units in the last place between two float arrays of one dtype."""
    import numpy as np
    if np.array_equal(x, y):
        return 0
    it = {4: np.int32, 8: np.int64}[x.dtype.itemsize]
    xi, yi = x.view(it).astype(np.int64), y.view(it).astype(np.int64)
    lowest = np.int64(np.iinfo(it).min)
    xi = np.where(xi < 0, lowest - xi, xi)          # sign-magnitude -> one monotone integer line
    yi = np.where(yi < 0, lowest - yi, yi)
    return int(np.abs(xi - yi).max())


class CpuLeg:
    """The oracle as it stands on the host cores: the expected result of every case (what the GPU result is
    compared with) and, from the same runs, the cpu_baseline figure."""

    def __init__(self):
        import oracle
        self.oracle = oracle
        cores = len(os.sched_getaffinity(0))
        self.threads = max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", cores))))
        self.multi, self.single, self.spent = {}, {}, 0.0

    def expected(self, c, A, B0, budget_s: float = 30.0):
        best, want = None, None
        for _ in range(3 if self.spent < budget_s else 1):
            B = B0.copy()
            t0 = time.perf_counter()
            self.oracle.transpose(c.dtype, c.sizes, c.perm, c.alpha, c.beta, A, B, self.threads)
            dt = time.perf_counter() - t0
            self.spent += dt
            best = dt if best is None else min(best, dt)
            want = B
        self.multi[c.name] = c.traffic_bytes / best / 1e9
        if self.spent < budget_s * 0.6:
            B = B0.copy()
            t0 = time.perf_counter()
            self.oracle.transpose(c.dtype, c.sizes, c.perm, c.alpha, c.beta, A, B, 1)
            dt = time.perf_counter() - t0
            self.spent += dt
            self.single[c.name] = c.traffic_bytes / dt / 1e9
        log(f"[cpu] {c.name}: {self.multi[c.name]:.2f} GB/s on {self.threads} threads"
            + (f", {self.single[c.name]:.2f} GB/s on 1" if c.name in self.single else ""))
        return want

    def summary(self, ncases: int):
        return {"value": round(statistics.median(self.multi.values()), 3), "unit": "GB/s", "cores": self.threads,
                "kind": "oracle",
                "sample": f"{len(self.multi)} of {ncases} suite cases at full size, best of 3 on {self.threads} threads, "
                          f"median over cases; {self.spent:.0f} s CPU wall",
                "single_thread_median": round(statistics.median(self.single.values()), 3) if self.single else None}


def plan_text(info, ttc) -> str:
    """The selected configuration in one short string (the fields that name it in the plan store and the profiles)."""
    cls = {ttc.TTC_KERNEL_DIRECT: "direct", ttc.TTC_KERNEL_LDS: "lds", ttc.TTC_KERNEL_ROWS: "rows", ttc.TTC_KERNEL_MICRO: "micro"}[info["kernel_class"]]
    tile = "x".join(str(t) for t in info["tile"])
    return (f"{cls} t{tile} v{info['vec_a']}/{info['vec_b']} th{info['threads']} wg{info['wg_per_cu']} u{info['unroll']} m{info['merged']} "
            f"buf{info['lds_buffers']} lds{info['lds_bytes']} nt{info['nt_a']}{info['nt_b']} x{info['xcd_remap']} "
            f"cf{info['lds_conflict_a']}/{info['lds_conflict_b']} cand{info['candidate_index']}/{info['candidate_count']}")


def measured_traffic(case_name: str, plan: str):
    """HBM bytes per launch from the committed rocprofv3 counter summary, if it was taken on this configuration."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    key = plan.split(" cand")[0]
    try:
        for line in open(path):
            parts = line.rstrip("\n").split("\t")
            if len(parts) >= 3 and parts[0] == case_name and parts[2].split(" cand")[0] == key:
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
    ttc.lib()                                   # fail loudly if the HIP library is not built
    os.environ.pop("TTC_PLAN_CACHE", None)      # the store is consulted explicitly below, never written behind our back
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    sel = [s for s in args.cases.split(",") if s]
    cases = [c for c in wl.CASES if not sel or any(s in c.name for s in sel)]
    if args.problem:
        f = args.problem.split(":")
        dt = {v: k for k, v in wl.DTYPE_NAME.items()}[f[0]]
        al = complex(f[3]) if len(f) > 3 else 1.0
        be = complex(f[4]) if len(f) > 4 else 0.0
        if dt in (wl.F32, wl.F64, wl.F32_F64, wl.F64_F32):
            al, be = al.real, be.real
        cases = [wl.Case(9, dt, tuple(int(x) for x in f[1].split("x")), tuple(int(x) for x in f[2]), al, be)]
    K, W = args.steps, args.warmup
    cpu = None if args.no_cpu else CpuLeg()

    # bring the clocks up before anything is timed
    warm = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=dev)
    warm2 = torch.empty_like(warm)
    ttc.ttc_time_ceiling(0, warm.numel() * 4, [warm.data_ptr()], [warm2.data_ptr()], stream, 5, 100)
    del warm, warm2

    results, failed = [], []
    for c in cases:
        nbytes = c.tensor_bytes
        # enough buffer pairs in rotation that the last-level cache cannot hold them (every launch meets HBM)
        npairs = max(2, min(48, -(-int(1.25 * LAST_LEVEL_CACHE_BYTES) // (2 * nbytes)) + 1))
        A_host, B_host = wl.case_inputs(c)
        A_dev = [torch.from_numpy(A_host).to(dev) for _ in range(npairs)]
        B_dev = [torch.from_numpy(B_host).to(dev) for _ in range(npairs)]
        a_ptrs = [t.data_ptr() for t in A_dev]
        b_ptrs = [t.data_ptr() for t in B_dev]
        reps = K if nbytes > 64e6 else max(K, 10 * npairs)       # microsecond launches: more of them per timing
        # ceilings of the same byte size, measured the same way, next to the case
        cbytes = nbytes - nbytes % 16                            # the copy helpers move whole 16-byte units
        # Untimed launches before every timing: W, and at least STEADY_MS of work.  Kernels made of very many small
        # workgroups take 10 ms of launches to reach their steady rate after the GPU has idled (measured: 5500 ->
        # 6100 GB/s over the first 50 launches of a 0.2 ms kernel, 5200 again after 0.2 s of idling; the copies do
        # not care), and the host work between the timings of a case is long enough for that.
        Wc = max(W, min(MAX_WARM, int(STEADY_MS / (2 * cbytes / 6.0e9) + 1)))
        ck = ttc.ttc_time_ceiling(0, cbytes, a_ptrs, b_ptrs, stream, Wc, reps)
        cm = ttc.ttc_time_ceiling(1, cbytes, a_ptrs, b_ptrs, stream, Wc, reps)
        cs = ttc.ttc_time_ceiling(3, cbytes, a_ptrs, b_ptrs, stream, Wc, reps)
        co = ttc.ttc_time_ceiling(4, cbytes, a_ptrs, b_ptrs, stream, Wc, reps)
        copy_k, copy_m, copy_s, copy_o = (2 * cbytes / t / 1e6 for t in (ck, cm, cs, co))
        axpby = None
        if not c.beta_is_zero:
            cx = min(ttc.ttc_time_ceiling(2, cbytes, a_ptrs, b_ptrs, stream, Wc, reps),
                     ttc.ttc_time_ceiling(5, cbytes, a_ptrs, b_ptrs, stream, Wc, reps))      # plain persistent, non-temporal one-shot
            axpby = 3 * cbytes / cx / 1e6
            for t in B_dev:                                      # the axpby ceiling changed B
                t.copy_(torch.from_numpy(B_host))
        d2d = max(copy_k, copy_m, copy_s, copy_o)   # the fastest known way to copy is the ceiling

        plan = ttc.ttc_plan_create(c.dtype, len(c.sizes), c.sizes, c.perm, c.alpha, c.beta)
        ms_heur = None if args.no_heuristic else ttc.ttc_time_execute(plan, a_ptrs, b_ptrs, stream, Wc, reps)
        t0 = time.perf_counter()
        source = "search"
        if args.force_class:
            want_cls = {"direct": ttc.TTC_KERNEL_DIRECT, "lds": ttc.TTC_KERNEL_LDS, "rows": ttc.TTC_KERNEL_ROWS, "micro": ttc.TTC_KERNEL_MICRO}[args.force_class]
            source = "first " + args.force_class
            for k in range(ttc.ttc_plan_candidate_count(plan)):
                ttc.ttc_plan_select_candidate(plan, k)
                if ttc.ttc_plan_get_info(plan)["kernel_class"] == want_cls:
                    break
            else:
                raise SystemExit(f"bench.py: {c.name} has no candidate of class {args.force_class}")
        elif not args.search and "," in args.plan_cache:
            # several stores (searches run on different machines): time what each holds for the case, keep the fastest
            timed = []
            for path in args.plan_cache.split(","):
                if path and ttc.ttc_plan_cache_lookup(plan, path):
                    timed.append((ttc.ttc_time_execute(plan, a_ptrs, b_ptrs, stream, Wc, reps), path))
                    log(f"[gpu] {c.name}: {path}: {c.traffic_bytes / timed[-1][0] / 1e6:.0f} GB/s, {plan_text(ttc.ttc_plan_get_info(plan), ttc)}")
            if not timed:
                raise SystemExit(f"bench.py: none of the stores holds {c.name}")
            ttc.ttc_plan_cache_lookup(plan, min(timed)[1])
            source = "store " + os.path.basename(min(timed)[1])
        elif not args.search and args.plan_cache and ttc.ttc_plan_cache_lookup(plan, args.plan_cache):
            source = "store"
        else:
            ttc.ttc_plan_tune_pairs(plan, a_ptrs, b_ptrs, stream, args.max_candidates)
        tune_s = time.perf_counter() - t0
        if args.store_plans:
            ttc.ttc_plan_cache_store(plan, args.store_plans)
        info = ttc.ttc_plan_get_info(plan)
        ms = ttc.ttc_time_execute(plan, a_ptrs, b_ptrs, stream, Wc, reps)      # the plan as finally selected
        # the same plan once more, from a fresh B, against the oracle
        max_ulp = None
        if cpu is not None:
            B_dev[0].copy_(torch.from_numpy(B_host))
            ttc.ttc_execute(plan, a_ptrs[0], b_ptrs[0], stream)
            torch.cuda.synchronize()
            got = B_dev[0].cpu().numpy()
            want = cpu.expected(c, A_host, B_host)
            max_ulp = ulp_distance(got, want)
            allowed = 0 if (complex(c.alpha) == 1 and complex(c.beta) == 0) else 1
            if max_ulp > allowed:
                failed.append((c.name, max_ulp))
            del got, want
        ttc.ttc_plan_destroy(plan)
        gbps = c.traffic_bytes / ms / 1e6
        r = {
            "case": c.name, "ms": round(ms, 5), "GBps": round(gbps, 1),
            "frac_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4),
            "frac_d2d_copy": round(gbps / d2d, 4),
            "frac_axpby_stream": round(gbps / axpby, 4) if axpby else None,
            "d2d_copy_GBps": round(d2d, 1),
            "heuristic_GBps": round(c.traffic_bytes / ms_heur / 1e6, 1) if ms_heur is not None else None,
            "max_ulp": max_ulp, "plan": plan_text(info, ttc), "plan_source": source, "tune_s": round(tune_s, 2),
            "pairs": npairs, "traffic_bytes": c.traffic_bytes,
            "working_set": "HBM" if 2 * nbytes * npairs > LAST_LEVEL_CACHE_BYTES else "cache-resident",
        }
        results.append(r)
        log(f"[gpu] {c.name}: {gbps:.0f} GB/s = {100 * r['frac_d2d_copy']:.1f}% of D2D copy ({d2d:.0f}; kernel {copy_k:.0f}, "
            f"nt kernel {copy_s:.0f}, one-shot nt {copy_o:.0f}, memcpy {copy_m:.0f}), heuristic {r['heuristic_GBps'] or 0:.0f}, max_ulp {max_ulp}, "
            f"{source}: {r['plan']}")
        del A_dev, B_dev
        torch.cuda.empty_cache()

    median_gbps = statistics.median(r["GBps"] for r in results)
    median_frac = statistics.median(r["frac_d2d_copy"] for r in results)
    ms_per_step = sum(r["ms"] for r in results)
    worst = min(results, key=lambda r: r["frac_d2d_copy"])
    low = min(results, key=lambda r: r["frac_hbm_peak"])
    # roofline: the staged kernel on the quoted workload (3-D fp32 384^3, full index reversal)
    dom = next((r for r in results if r["case"].startswith("cfg2-f32-p210")), results[0])
    roofline = {"bound": "hbm", "achieved": dom["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(dom["GBps"] / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(dom["case"], dom["plan"]),
                "kernel": {"micro": "micro_kernel", "rows": "rows_kernel"}.get(dom["plan"].split(" ")[0], "box_kernel"),
                "case": dom["case"], "plan": dom["plan"],
                "algorithmic_bytes_per_launch": dom["traffic_bytes"], "avg_launch_ms": dom["ms"],
                "median_frac_of_d2d_copy": round(median_frac, 4),
                "worst_case_vs_copy": worst["case"], "worst_frac_of_d2d_copy": worst["frac_d2d_copy"],
                "lowest_case_vs_peak": low["case"], "lowest_achieved": low["GBps"], "lowest_frac": low["frac_hbm_peak"],
                "lowest_traffic": measured_traffic(low["case"], low["plan"]),
                "all_results_match_oracle": (not failed) if cpu is not None else None}
    # one short entry per case, flat, so that every fraction and every max_ulp survives in the record
    for k, r in enumerate(results, 1):
        short = r["case"].replace("-f32", "").replace("-f64", "").replace("-c64", "")
        roofline[f"case{k:02d}"] = (f"{short} {r['GBps']:.0f}GB/s copy={r['frac_d2d_copy']:.3f} peak={r['frac_hbm_peak']:.3f} "
                                     f"ulp={r['max_ulp']} {r['working_set']}")
    out = {
        "metric": "effective HBM bandwidth (bytes read + written / time) per permutation, median over the suite",
        "value": round(median_gbps, 1), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32/f64/c64", "data": "synthetic",
        "config": {"workload": f"{len(results)}-case suite (2-D/3-D fp32, 4-D fp64, 6-D fp32, 5-D complex64), one launch per case per step",
                   "cases": len(results), "untimed_ms_before_each_timing": STEADY_MS},
        "roofline": roofline,
    }
    if cpu is not None:
        out["cpu_baseline"] = cpu.summary(len(cases))
    # per-case rows, compact: [case, ms, GB/s, frac of copy, frac of peak, frac of axpby stream, heuristic GB/s, max_ulp, source, plan]
    out["case_columns"] = "case,ms,GBps,frac_copy,frac_peak,frac_axpby,heur_GBps,max_ulp,source,plan"
    out["cases"] = [[r["case"], r["ms"], r["GBps"], r["frac_d2d_copy"], r["frac_hbm_peak"], r["frac_axpby_stream"],
                     r["heuristic_GBps"], r["max_ulp"], r["plan_source"], r["plan"]] for r in results]
    print(json.dumps(out, separators=(",", ":")), flush=True)
    if failed:
        log("bench.py: RESULT MISMATCH against the oracle: " + ", ".join(f"{n} ({u} ulp)" for n, u in failed))
        return 1
    return 0


if __name__ == "__main__":
    sys.exit(main())
