"""Two measurement studies on the GPU, modelled on the paper's evaluation (Sections 4 and 6).

    python -m paper_1603_02297_amd.studies search  [--out FILE]     search-space reduction
    python -m paper_1603_02297_amd.studies sweep   [--out FILE]     57-case benchmark, classes, ablations

search: how close the first 1 / 10 / 100 / 200 candidates of the ranked list come to the best
of all candidates (the paper reports 94.58 / 97.35 / 99.10 % for 1 / 10 / 100 on its CPUs).

sweep: a benchmark built by the paper's rules (Section 4.1): 19 permutations -- one 2-D, three
3-D, five each for 4-D, 5-D, 6-D, none with mergeable indices, each dimension with its inverse
permutation and exactly one permutation that keeps the stride-1 index -- times three shapes
(about equal extents; extents growing by a factor 6 from first to last index; the same
shrinking), fp32, about 200 MiB per tensor.  The paper's own list is not published in the text,
so the permutations are drawn here from a fixed seed.  Reported per class (stride-1 / inverse /
general), with the gain of each search dimension (tile shape, vector width, tile order, LDS
buffering, launch shape) measured as in the paper's Figure 6: best candidate overall over the
best candidate with that dimension held at its default.

Everything is timed with HIP events through the library's own helpers; tensors hold uniform
random values; buffer pairs rotate so that the last-level cache cannot hold the working set.
"""
from __future__ import annotations

import argparse
import itertools
import json
import statistics
import sys
import time

import numpy as np

from . import binding as ttc
from . import workloads as wl

TARGET_BYTES = 200 * 1024 * 1024


def log(msg):
    print(msg, file=sys.stderr, flush=True)


# ---- problems -----------------------------------------------------------------------------------
def mergeable(perm):
    return any(perm[j + 1] == perm[j] + 1 for j in range(len(perm) - 1))


def benchmark_permutations(seed=1603):
    """19 permutations by the paper's rules; class of each: 'stride-1', 'inverse' or 'general'."""
    rng = np.random.default_rng(seed)
    out = []
    for n, count in ((2, 1), (3, 3), (4, 5), (5, 5), (6, 5)):
        inverse = tuple(range(n - 1, -1, -1))
        chosen = [(inverse, "inverse")]
        if count > 1:
            fixed = [p for p in itertools.permutations(range(n)) if p[0] == 0 and not mergeable(p)]
            chosen.append((fixed[int(rng.integers(len(fixed)))], "stride-1"))
            general = [p for p in itertools.permutations(range(n))
                       if p[0] != 0 and p != inverse and not mergeable(p)]
            for k in rng.choice(len(general), size=count - 2, replace=False):
                chosen.append((general[int(k)], "general"))
        out += chosen
    return out


def shape_for(n, config, elem_bytes=4):
    """Extents of an n-index tensor of about TARGET_BYTES: config 0 equal, 1 growing x6, 2 shrinking x6."""
    vol = TARGET_BYTES / elem_bytes
    if config == 0 or n == 1:
        ratios = [1.0] * n
    else:
        ratios = [6.0 ** (k / (n - 1)) for k in range(n)]
        if config == 2:
            ratios.reverse()
    geo = float(np.prod(ratios)) ** (1.0 / n)
    base = (vol ** (1.0 / n)) / geo
    return tuple(max(2, int(round(base * r))) for r in ratios)


# ---- timing -------------------------------------------------------------------------------------
class Buffers:
    """Rotating A/B pairs of one size, reused while the size stays the same."""

    def __init__(self):
        self.key, self.a, self.b = None, [], []

    def get(self, torch, elements, elem_bytes, pairs=3):
        key = (elements, elem_bytes)
        if key != self.key:
            self.a, self.b = [], []
            torch.cuda.empty_cache()
            n32 = elements * elem_bytes // 4
            dev = torch.device("cuda:0")
            self.a = [torch.rand(n32, dtype=torch.float32, device=dev) * 2 - 1 for _ in range(pairs)]
            self.b = [torch.rand(n32, dtype=torch.float32, device=dev) * 2 - 1 for _ in range(pairs)]
            self.key = key
        return [t.data_ptr() for t in self.a], [t.data_ptr() for t in self.b]


def time_candidates(plan, a_ptrs, b_ptrs, stream, warm=1, reps=4):
    """(info, ms) of every candidate of the plan, in rank order."""
    rows = []
    for k in range(ttc.ttc_plan_candidate_count(plan)):
        ttc.ttc_plan_select_candidate(plan, k)
        ms = ttc.ttc_time_execute(plan, a_ptrs, b_ptrs, stream, warm, reps)
        rows.append((ttc.ttc_plan_get_info(plan), ms))
    return rows


def retime_best(plan, rows, a_ptrs, b_ptrs, stream, keep=8):
    """Time the fastest few again, longer, with the streaming hints by rule, off and on, then with the other
    tile mappings (as the library's own search does), and return rows with those entries replaced by their best."""
    order = sorted(range(len(rows)), key=lambda i: rows[i][1])[:keep]
    rows = list(rows)
    for i in order:
        ttc.ttc_plan_select_candidate(plan, i)
        best = None
        for sa, sb in ((-1, -1), (0, 0), (1, 1)):
            ttc.ttc_plan_set_streaming(plan, sa, sb)
            ms = ttc.ttc_time_execute(plan, a_ptrs, b_ptrs, stream, 2, 12)
            if best is None or ms < best[1]:
                best = (ttc.ttc_plan_get_info(plan), ms)
        info = best[0]
        ttc.ttc_plan_set_streaming(plan, info["nt_a"], info["nt_b"])
        for mode in (1, 3):                      # tiles dealt to the XCDs: one range each, chunks of 8 (default: chunks of 32)
            ttc.ttc_plan_set_tile_mapping(plan, mode)
            ms = ttc.ttc_time_execute(plan, a_ptrs, b_ptrs, stream, 2, 12)
            if ms < best[1]:
                best = (ttc.ttc_plan_get_info(plan), ms)
        ttc.ttc_plan_set_tile_mapping(plan, -1)
        ttc.ttc_plan_set_streaming(plan, -1, -1)
        rows[i] = best
    return rows


def d2d_copy_gbps(nbytes, a_ptrs, b_ptrs, stream):
    nbytes -= nbytes % 16                       # the copy helpers move whole 16-byte units
    ck = ttc.ttc_time_ceiling(0, nbytes, a_ptrs, b_ptrs, stream, 2, 10)
    cm = ttc.ttc_time_ceiling(1, nbytes, a_ptrs, b_ptrs, stream, 2, 10)
    cs = ttc.ttc_time_ceiling(3, nbytes, a_ptrs, b_ptrs, stream, 2, 10)
    return 2 * nbytes / min(ck, cm, cs) / 1e6


# ---- study 1: reduction of the search space -------------------------------------------------------
def study_search(out, dump=None):
    import torch
    stream = torch.cuda.current_stream().cuda_stream
    bufs = Buffers()
    caps = (1, 10, 100, 200)
    table = []
    problems = [(c.name, c.dtype, c.sizes, c.perm, c.alpha, c.beta) for c in wl.CASES if c.config != 1]
    for (perm, cls), cfg in itertools.product(benchmark_permutations(), (0, 1)):
        if len(perm) in (3, 5):
            sizes = shape_for(len(perm), cfg)
            problems.append((f"bench-{len(perm)}d-{cls}-cfg{cfg}-p{''.join(map(str, perm))}", wl.F32, sizes, perm, 1.0, 0.0))
    for name, dtype, sizes, perm, alpha, beta in problems:
        n = int(np.prod(sizes))
        a_ptrs, b_ptrs = bufs.get(torch, n, wl.ELEM_BYTES[dtype])
        plan = ttc.ttc_plan_create(dtype, len(sizes), sizes, perm, alpha, beta)
        rows = retime_best(plan, time_candidates(plan, a_ptrs, b_ptrs, stream), a_ptrs, b_ptrs, stream)
        ttc.ttc_plan_destroy(plan)
        ms = np.array([r[1] for r in rows])
        if dump is not None:        # every candidate's configuration and time, one JSON line per problem
            dump.write(json.dumps({"problem": name, "rows": [dict(r[0], ms=r[1]) for r in rows]}) + "\n")
        best = ms.min()
        frac = [best / ms[:k].min() for k in caps]
        table.append((name, len(rows), rows[0][0]["bytes_moved"] / best / 1e6, frac))
        log(f"{name}: {len(rows)} candidates, best {table[-1][2]:.0f} GB/s, " +
            ", ".join(f"first {k}: {100 * f:.1f}%" for k, f in zip(caps, frac)))
    w = max(len(t[0]) for t in table)
    print(f"{'problem':<{w}}  cands  best GB/s  " + "  ".join(f"first {k:>3}" for k in caps), file=out)
    for name, n, gbps, frac in table:
        print(f"{name:<{w}}  {n:5d}  {gbps:9.0f}  " + "  ".join(f"{100 * f:8.2f}%" for f in frac), file=out)
    mean = [statistics.mean(t[3][i] for t in table) for i in range(len(caps))]
    low = [min(t[3][i] for t in table) for i in range(len(caps))]
    print(f"{'mean':<{w}}  {'':5}  {'':9}  " + "  ".join(f"{100 * f:8.2f}%" for f in mean), file=out)
    print(f"{'minimum':<{w}}  {'':5}  {'':9}  " + "  ".join(f"{100 * f:8.2f}%" for f in low), file=out)
    print("paper (Section 6, its CPUs): first 1: 94.58%, first 10: 97.35%, first 100: 99.10% of the full search",
          file=out)


# ---- study 2: the 57-case benchmark, classes and ablations ------------------------------------------
def ablations(rows):
    """Gain of searching each dimension: best time with the dimension at its default / best time overall."""
    ms = np.array([r[1] for r in rows])
    infos = [r[0] for r in rows]
    best = ms.min()
    first = infos[0]

    def best_where(pred):
        sel = [m for i, m in zip(infos, ms) if pred(i)]
        return (min(sel) / best) if sel else float("nan")

    return {
        "tile shape": best_where(lambda i: i["tile"] == first["tile"] and i["kernel_class"] == first["kernel_class"]),
        "vector width": best_where(lambda i: i["vec_a"] == 1 and i["vec_b"] == 1),
        "tile order": best_where(lambda i: i["tile_order"] == i["perm"]),
        "LDS buffering": best_where(lambda i: i["kernel_class"] == ttc.TTC_KERNEL_DIRECT or i["lds_buffers"] == 2),
        "launch shape": best_where(lambda i: i["threads"] == 256 and i["wg_per_cu"] == 16),
    }


def study_sweep(out, limit=None, dump=None):
    import torch
    stream = torch.cuda.current_stream().cuda_stream
    bufs = Buffers()
    results = []
    cases = [(perm, cls, cfg) for perm, cls in benchmark_permutations() for cfg in (0, 1, 2)]
    if limit:
        cases = cases[:limit]
    for perm, cls, cfg in cases:
        sizes = shape_for(len(perm), cfg)
        n = int(np.prod(sizes))
        a_ptrs, b_ptrs = bufs.get(torch, n, 4)
        copy = d2d_copy_gbps(n * 4, a_ptrs, b_ptrs, stream)
        plan = ttc.ttc_plan_create(wl.F32, len(sizes), sizes, perm, 1.0, 0.0)
        rows = retime_best(plan, time_candidates(plan, a_ptrs, b_ptrs, stream), a_ptrs, b_ptrs, stream)
        ttc.ttc_plan_select_candidate(plan, 0)
        heur_ms = ttc.ttc_time_execute(plan, a_ptrs, b_ptrs, stream, 2, 12)
        ttc.ttc_plan_destroy(plan)
        ms = np.array([r[1] for r in rows])
        k = int(ms.argmin())
        nbytes = rows[0][0]["bytes_moved"]
        if dump is not None:
            name = f"sweep-{len(perm)}d-{cls}-cfg{cfg}-p{''.join(map(str, perm))}"
            dump.write(json.dumps({"problem": name, "rows": [dict(r[0], ms=r[1]) for r in rows]}) + "\n")
        res = {"perm": perm, "class": cls, "cfg": cfg, "sizes": sizes, "copy": copy,
               "best": nbytes / ms[k] / 1e6, "heur": nbytes / heur_ms / 1e6, "info": rows[k][0],
               "abl": ablations(rows), "cands": len(rows)}
        results.append(res)
        log(f"{len(perm)}-D {cls:9s} cfg{cfg} {sizes} p{perm}: best {res['best']:.0f} GB/s = "
            f"{100 * res['best'] / copy:.1f}% of copy, heuristic {res['heur']:.0f}")
    print("dim class     cfg  sizes / perm                                          cands  copy GB/s  heur GB/s  best GB/s"
          "  best/copy  tile of the best", file=out)
    for r in results:
        sp = f"{'x'.join(map(str, r['sizes']))} p{''.join(map(str, r['perm']))}"
        print(f"{len(r['perm'])}-D {r['class']:9s} {r['cfg']}    {sp:<52}  {r['cands']:5d}  {r['copy']:9.0f}  {r['heur']:9.0f}"
              f"  {r['best']:9.0f}  {100 * r['best'] / r['copy']:8.1f}%  {r['info']['tile']}", file=out)
    print("", file=out)
    print("class      cases  median best/copy  min best/copy  median heur/copy  median best GB/s", file=out)
    for cls in ("stride-1", "inverse", "general", "all"):
        sel = [r for r in results if cls == "all" or r["class"] == cls]
        if not sel:
            continue
        fb = [r["best"] / r["copy"] for r in sel]
        fh = [r["heur"] / r["copy"] for r in sel]
        print(f"{cls:9s}  {len(sel):5d}  {100 * statistics.median(fb):15.1f}%  {100 * min(fb):12.1f}%"
              f"  {100 * statistics.median(fh):15.1f}%  {statistics.median(r['best'] for r in sel):16.0f}", file=out)
    print("", file=out)
    print("gain of searching one dimension (best time with it held at its default / best time overall; "
          "paper Figure 6 reports up to +35% for blocking, +22% for loop order on its CPUs)", file=out)
    print("dimension       default held                                   mean gain  max gain", file=out)
    held = {"tile shape": "tile of the heuristic's first candidate", "vector width": "one element per lane",
            "tile order": "tiles numbered in B's index order", "LDS buffering": "two tile buffers",
            "launch shape": "256 threads, 16 workgroups per CU"}
    for name in held:
        g = [r["abl"][name] - 1.0 for r in results if r["abl"][name] == r["abl"][name]]
        if g:
            print(f"{name:14s}  {held[name]:45s}  {100 * statistics.mean(g):+8.1f}%  {100 * max(g):+7.1f}%", file=out)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("study", choices=("search", "sweep"))
    ap.add_argument("--out", default="", help="write the table to this file (default: stdout)")
    ap.add_argument("--limit", type=int, default=0, help="sweep: only the first LIMIT cases")
    ap.add_argument("--dump", default="", help="also write every candidate's configuration and time (JSON lines; .gz compresses)")
    args = ap.parse_args(argv)
    import torch
    if not torch.cuda.is_available():
        print("studies: no GPU visible", file=sys.stderr)
        return 2
    ttc.lib()
    out = open(args.out, "w") if args.out else sys.stdout
    t0 = time.time()
    print(f"# python -m paper_1603_02297_amd.studies {args.study}" + (f" --limit {args.limit}" if args.limit else ""), file=out)
    dump = None
    if args.dump:
        import gzip
        dump = gzip.open(args.dump, "wt") if args.dump.endswith(".gz") else open(args.dump, "w")
    if args.study == "search":
        study_search(out, dump)
    else:
        study_sweep(out, args.limit or None, dump)
    if dump:
        dump.close()
    print(f"# {time.time() - t0:.0f} s", file=out)
    if args.out:
        out.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
