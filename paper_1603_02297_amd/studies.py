"""Measurement studies on the GPU, modelled on the paper's evaluation (Sections 4 and 6), and the fit of the ranking model.

    python -m paper_1603_02297_amd.studies search  [--out FILE]     search-space reduction
    python -m paper_1603_02297_amd.studies sweep   [--out FILE]     57-case benchmark, classes, ablations
    python -m paper_1603_02297_amd.studies fit DUMP [DUMP ...]      weights of the ranking model from --dump files (no GPU)

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
best candidate with that dimension held at its default; and the gain of the pads in the LDS
tile: the best configuration laid out again without pads (TTC_LDS_PAD=0) and timed.

Results are checked elsewhere: tests/test_gpu_sweep_shapes.py runs these very shapes (same generator,
host-drawn seeded values) against the CPU oracle; nothing in this package touches the oracle.

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
    """(info, ms) of every candidate of the plan, in rank order (ms: the better of the rule's streaming hints and both sides streamed)."""
    rows = []
    for k in range(ttc.ttc_plan_candidate_count(plan)):
        ttc.ttc_plan_select_candidate(plan, k)
        ms = ttc.ttc_time_execute(plan, a_ptrs, b_ptrs, stream, warm, reps)
        info = ttc.ttc_plan_get_info(plan)
        if not (info["nt_a"] == 1 and info["nt_b"] == 1):     # like the library's search: the better of the rule's hints and both sides streamed
            ttc.ttc_plan_set_streaming(plan, 1, 1)
            ms_nt = ttc.ttc_time_execute(plan, a_ptrs, b_ptrs, stream, warm, reps)
            if ms_nt < ms:
                ms, info = ms_nt, ttc.ttc_plan_get_info(plan)
            ttc.ttc_plan_set_streaming(plan, -1, -1)
        rows.append((info, ms))
    return rows


def retime_best(plan, rows, a_ptrs, b_ptrs, stream, keep=8):
    """Time the fastest few again, longer, with the streaming hints by rule, off, on and on one side only, then with
    the other tile mappings (as the library's own search does), and return rows with those entries replaced by their best."""
    order = sorted(range(len(rows)), key=lambda i: rows[i][1])[:keep]
    rows = list(rows)
    for i in order:
        ttc.ttc_plan_select_candidate(plan, i)
        best = None
        for sa, sb in ((-1, -1), (0, 0), (1, 1), (1, 0), (0, 1)):
            ttc.ttc_plan_set_streaming(plan, sa, sb)
            ms = ttc.ttc_time_execute(plan, a_ptrs, b_ptrs, stream, 2, 12)
            if best is None or ms < best[1]:
                best = (ttc.ttc_plan_get_info(plan), ms)
        info = best[0]
        ttc.ttc_plan_set_streaming(plan, info["nt_a"], info["nt_b"])
        for mode in (1, 3):                      # tiles dealt to the XCDs: one range each, chunks of 8 (default: chunks of 32)
            if info["kernel_class"] == ttc.TTC_KERNEL_ROWS:
                break                            # no tiles to deal
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
    co = ttc.ttc_time_ceiling(4, nbytes, a_ptrs, b_ptrs, stream, 2, 10)
    return 2 * nbytes / min(ck, cm, cs, co) / 1e6


# ---- study 1: reduction of the search space -------------------------------------------------------
def search_set(families, cap):
    """Ranks the library's search times when capped at `cap` candidates (the rule of ttc_plan_tune_pairs): the
    first `cap` of the ranking, a fifth of the places going to the best-ranked micro-tile candidates over single
    indices and another fifth to those over merged indices where the ranking would have left them out.
    families: per candidate in rank order, 0 = other kernels, 1 = micro-tile, 2 = micro-tile over merged indices."""
    total = len(families)
    cap = min(cap, total)
    chosen = list(range(cap))
    if 10 <= cap < total:
        extra = []
        for fam in (1, 2):
            seen = 0
            for i, f in enumerate(families):
                if seen >= cap // 5:
                    break
                if f == fam:
                    seen += 1
                    if i >= cap:
                        extra.append(i)
        k = cap - 1
        while k >= 1 and extra:
            if families[chosen[k]] == 0:
                chosen[k] = extra.pop()
            k -= 1
    return chosen


def micro_family(info):
    """0: not the micro-tile kernel; 1: its tile is over single indices; 2: two indices taken as one on a side."""
    if info["kernel_class"] != ttc.TTC_KERNEL_MICRO:
        return 0
    return 2 if info["merged"] else 1


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
        families = [micro_family(r[0]) for r in rows]
        frac = [best / ms[search_set(families, k)].min() for k in caps]
        table.append((name, len(rows), rows[0][0]["bytes_moved"] / best / 1e6, frac))
        log(f"{name}: {len(rows)} candidates, best {table[-1][2]:.0f} GB/s, " +
            ", ".join(f"first {k}: {100 * f:.1f}%" for k, f in zip(caps, frac)))
    w = max(len(t[0]) for t in table)
    print("best time among the candidates a search capped at 1 / 10 / 100 / 200 would time, relative to the best of all", file=out)
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
def unpadded_ms(dtype, sizes, perm, alpha, beta, best_info, a_ptrs, b_ptrs, stream, tmp):
    """Time of the configuration `best_info` names when its LDS tile is laid out without pads (without the swizzle), or None."""
    import os
    if best_info["kernel_class"] not in (ttc.TTC_KERNEL_LDS, ttc.TTC_KERNEL_MICRO):
        return None                              # no LDS tile (the micro-tile kernel's is swizzled, not padded: the swizzle goes)
    plan = ttc.ttc_plan_create(dtype, len(sizes), sizes, perm, alpha, beta)
    ttc.ttc_plan_select_candidate(plan, best_info["candidate_index"])
    ttc.ttc_plan_set_streaming(plan, best_info["nt_a"], best_info["nt_b"])
    ttc.ttc_plan_set_tile_mapping(plan, best_info["xcd_remap"])
    open(tmp, "w").close()
    ttc.ttc_plan_cache_store(plan, tmp)
    ttc.ttc_plan_destroy(plan)
    os.environ["TTC_LDS_PAD"] = "0"
    try:
        plan = ttc.ttc_plan_create(dtype, len(sizes), sizes, perm, alpha, beta)
        if not ttc.ttc_plan_cache_lookup(plan, tmp):
            ttc.ttc_plan_destroy(plan)
            return None
        info = ttc.ttc_plan_get_info(plan)
        ms = ttc.ttc_time_execute(plan, a_ptrs, b_ptrs, stream, 2, 12)
        ttc.ttc_plan_destroy(plan)
    finally:
        del os.environ["TTC_LDS_PAD"]
    return ms, info


ONE_SHOT = (ttc.TTC_KERNEL_ROWS, ttc.TTC_KERNEL_MICRO)      # one tile (chunk) per workgroup: no workgroups-per-CU knob


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
        "LDS buffering": best_where(lambda i: i["kernel_class"] != ttc.TTC_KERNEL_LDS or i["lds_buffers"] == 2),
        "launch shape": best_where(lambda i: i["threads"] == 256 and (i["wg_per_cu"] == 16 or i["kernel_class"] in ONE_SHOT)),
        "kernel family": best_where(lambda i: i["kernel_class"] in (ttc.TTC_KERNEL_LDS, ttc.TTC_KERNEL_DIRECT)),
    }


def study_sweep(out, limit=None, dump=None):
    import torch
    stream = torch.cuda.current_stream().cuda_stream
    import tempfile
    bufs = Buffers()
    results = []
    tmp_store = tempfile.NamedTemporaryFile(prefix="ttc_sweep_", suffix=".txt", delete=False).name
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
        ms = np.array([r[1] for r in rows])
        k = int(ms.argmin())
        ttc.ttc_plan_select_candidate(plan, rows[k][0]["candidate_index"])
        ttc.ttc_plan_set_streaming(plan, rows[k][0]["nt_a"], rows[k][0]["nt_b"])
        ttc.ttc_plan_set_tile_mapping(plan, rows[k][0]["xcd_remap"])
        best_again = ttc.ttc_time_execute(plan, a_ptrs, b_ptrs, stream, 2, 12)     # timed next to its unpadded twin
        ttc.ttc_plan_destroy(plan)
        nopad = unpadded_ms(wl.F32, sizes, perm, 1.0, 0.0, rows[k][0], a_ptrs, b_ptrs, stream, tmp_store)
        nbytes = rows[0][0]["bytes_moved"]
        if dump is not None:
            name = f"sweep-{len(perm)}d-{cls}-cfg{cfg}-p{''.join(map(str, perm))}"
            dump.write(json.dumps({"problem": name, "rows": [dict(r[0], ms=r[1]) for r in rows]}) + "\n")
        res = {"perm": perm, "class": cls, "cfg": cfg, "sizes": sizes, "copy": copy,
               "best": nbytes / ms[k] / 1e6, "heur": nbytes / heur_ms / 1e6, "info": rows[k][0],
               "abl": ablations(rows), "cands": len(rows)}
        res["abl"]["LDS pads"] = (nopad[0] / best_again) if nopad else float("nan")
        res["conflict"] = (rows[k][0]["lds_conflict_a"], rows[k][0]["lds_conflict_b"],
                           nopad[1]["lds_conflict_a"] if nopad else 0, nopad[1]["lds_conflict_b"] if nopad else 0)
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
            "launch shape": "256 threads, 16 workgroups per CU",
            "LDS pads": "the best configuration with an unpadded LDS tile",
            "kernel family": "box kernels only (no row kernel, no micro-tile kernel)"}
    for name in held:
        g = [r["abl"][name] - 1.0 for r in results if r["abl"][name] == r["abl"][name]]
        if g:
            print(f"{name:14s}  {held[name]:45s}  {100 * statistics.mean(g):+8.1f}%  {100 * max(g):+7.1f}%", file=out)


# ---- study 3: fitting the ranking model ------------------------------------------------------------
FREE_SIGN = {"alA*A<256", "alA*A<1K", "tile>16K", "tile>32K", "t128", "t512", "wg4", "wg8", "ordA", "ordMix", "direct",
             "nbuf1", "nt", "conf", "partB", "b*nbuf1", "b*t128"}


def fit_features(r):
    """Features of one timed candidate (a row of a --dump file: ttc_plan_get_info plus its time).  They mirror the
    terms of heuristic_cost() in csrc/ttc_plan.cpp: contiguous run and per-instruction piece per side (octaves below
    1 KB / 256 B / 64 B), how much of a 128-byte line a run shares with its neighbours, extra line and 64-byte write
    requests, tile size, occupancy, idle lanes, vector width, remainder tiles, launch shape, tile order, streaming."""
    eba, ebb = wl.ELEM_BYTES[r["dtype"]], wl.ELEM_BYTES_B[r["dtype"]]
    n, sizes, tile = r["ndim"], r["sizes"], r["tile"]
    vol = float(np.prod(tile[:n]))
    tb = vol * eba
    direct = r["kernel_class"] == ttc.TTC_KERNEL_DIRECT
    ra, rb, sa, sb, aa, ab = (r[k] for k in ("run_bytes_a", "run_bytes_b", "seg_bytes_a", "seg_bytes_b", "align_a", "align_b"))

    def idle(dt, dl, vec, nd):
        it = 1
        for t_, l_ in zip(dt[:nd], dl[:nd]):
            it *= -(-t_ // l_)
        return it * 64 * vec / vol - 1.0

    la = idle(r["digit_tile_a"], r["digit_lane_a"], r["vec_a"], r["digits_a"])
    lb = 0.0 if direct else idle(r["digit_tile_b"], r["digit_lane_b"], r["vec_b"], r["digits_b"])
    wv = r["threads"] // 64
    waves = min(32, (160 * 1024 // max(r["lds_bytes"], 1)) * wv) if not direct else 32
    wgs = min(16, 160 * 1024 // max(r["lds_bytes"], 1))
    pad = 1.0
    for k in range(n):
        pad *= (-(-sizes[k] // tile[k]) * tile[k]) / sizes[k]
    vb = r["vec_b"] if not direct else r["vec_a"]
    lg = lambda x: float(np.log2(x))
    order, perm = r["tile_order"][:n], r["perm"][:n]
    okind = 0 if order == perm else (1 if order == list(range(n)) else 2)
    f = {
        "A<1K": max(0, lg(1024 / ra)), "B<1K": max(0, lg(1024 / rb)), "A<256": max(0, lg(256 / ra)), "B<256": max(0, lg(256 / rb)),
        "A<64": max(0, lg(64 / ra)), "B<64": max(0, lg(64 / rb)),
        "Aun": (1 - aa / 128) * 128 / ra, "Bun": (1 - ab / 128) * 128 / rb,
        "sA<256": max(0, lg(256 / sa)), "sB<256": max(0, lg(256 / sb)), "sA<64": max(0, lg(64 / sa)), "sB<64": max(0, lg(64 / sb)),
        "tile<8K": max(0, lg(8192 / tb)), "tile>16K": max(0, lg(tb / 16384)), "tile>32K": max(0, lg(tb / 32768)),
        "occ": max(0, 16 - waves) / 16, "occ8": max(0, 8 - waves) / 8, "wgs<4": max(0, 4 - wgs) / 4, "laneA": la, "laneB": lb,
        "conf": 0 if direct else (r["lds_conflict_a"] + r["lds_conflict_b"] - 4),
        "vbytesA<16": float(r["vec_a"] * eba < 16), "vbytesB<16": float(vb * ebb < 16),
        "vbytesA<8": float(r["vec_a"] * eba < 8), "vbytesB<8": float(vb * ebb < 8),
        "partA": float(r["partial_a"]), "partB": float(r["partial_b"]), "pad": pad - 1,
        "t128": float(r["threads"] == 128), "t512": float(r["threads"] == 512),
        "wg4": float(r["wg_per_cu"] == 4), "wg8": float(r["wg_per_cu"] == 8),
        "ordA": float(okind == 1), "ordMix": float(okind == 2), "direct": float(direct),
        "few": max(0, (2048 - r["num_tiles"]) / 2048), "nbuf1": float((not direct) and r["lds_buffers"] == 1),
        "dirun": float(direct) * ((1 - aa / 128) * 128 / sa + (1 - ab / 128) * 128 / sb),
    }
    beta = float(r["epilogue"] == ttc.TTC_EPI_AXPBY)
    req_a = ((ra + 128 - min(aa, 128)) / 128) * 128 / ra - 1
    req_b = ((rb + 64 - min(ab, 64)) / 64) * 64 / rb - 1
    f.update({"reqA": req_a, "reqB": req_b, "b*B<256": beta * f["B<256"], "b*Bun": beta * f["Bun"], "b*reqB": beta * req_b,
              "oA*Bun": f["ordA"] * f["Bun"], "oA*reqB": f["ordA"] * req_b, "oM*Bun": f["ordMix"] * f["Bun"],
              "alB*B<1K": float(ab >= 128) * max(0, lg(1024 / rb)), "alB*B<2K": float(ab >= 128) * max(0, lg(2048 / rb)),
              "alA*A<256": float(aa >= 128) * max(0, lg(256 / ra)), "alA*A<1K": float(aa >= 128) * max(0, lg(1024 / ra)),
              "nt": float(r["nt_a"] + r["nt_b"]) / 2, "b*nbuf1": beta * f["nbuf1"], "b*t128": beta * f["t128"]})
    return f


FREE_SIGN_MICRO = {"A>1K", "B>1K", "t128", "t64", "ordNotB", "blocks", "lds", "mergeA", "mergeB", "beta"}


def fit_micro_features(r):
    """Features of one timed micro-tile candidate; they mirror the terms of micro_cost() in csrc/ttc_plan.cpp: run
    length per side (octaves below 128 / 256 / 512 bytes, above 1 KB), remainder tiles, runs that start inside
    cache lines, workgroup size, tile order, blocks per lane, LDS per workgroup, merged indices and tiles that cut
    the inner index of a merged pair, idle lanes."""
    eb = wl.ELEM_BYTES[r["dtype"]]
    n, sizes, perm = r["ndim"], r["sizes"], r["perm"]
    p0 = perm[0]
    ta, tb = r["digit_tile_a"][0], r["digit_tile_a"][1]
    ma, mb = r["merged"] & 1, (r["merged"] >> 1) & 1
    cols = sizes[0] * (sizes[1] if ma else 1)
    rows = sizes[p0] * (sizes[perm[1]] if mb else 1)
    ra, rb = ta * eb, tb * eb
    below = lambda v, ref: max(0.0, float(np.log2(ref / v)))
    above = lambda v, ref: max(0.0, float(np.log2(v / ref)))
    line = 128 // eb
    un_a = float(cols % line != 0 or ta % line != 0)
    un_b = float(rows % line != 0 or tb % line != 0)
    vec = 16 // eb
    blocks, th = max(1, r["unroll"]), r["threads"]
    return {
        "A<128": below(ra, 128), "A<256": below(ra, 256), "A<512": below(ra, 512), "A>1K": above(ra, 1024),
        "B<128": below(rb, 128), "B<256": below(rb, 256), "B<512": below(rb, 512), "B>1K": above(rb, 1024),
        "pad": (-(-cols // ta) * ta / cols) * (-(-rows // tb) * tb / rows) - 1.0,
        "unA*A<512": un_a * below(ra, 512), "unB*B<512": un_b * below(rb, 512),
        "t128": float(th == 128), "t64": float(th == 64), "ordNotB": float(r["tile_order"][:n] != perm[:n]),
        "blocks": float(np.log2(blocks)), "lds": r["lds_bytes"] / 65536.0,
        "mergeA": float(ma), "mergeB": float(mb),
        "cutA": float(ma and ta % sizes[0] != 0), "cutB": float(mb and tb % sizes[p0] != 0),
        "idle": 1.0 - (ta // vec) * (tb // vec) / (blocks * th),
    }


def study_fit(out, dumps, ridge=0.05, sharpness=3.0, folds=8, family="box"):
    """Weights of heuristic_cost() (family "box") or micro_cost() (family "micro") from per-candidate timings (the
    --dump files of `search` and `sweep`).

    Model: log(time / best time of the problem) = sum_k w_k * feature_k + one free intercept per problem.
    Objective: least squares, each row weighted by exp(-sharpness * log-slowdown) so that the fast candidates, whose
    order matters, count most; a ridge term keeps collinear features apart.  Constraints: every weight that prices
    a loss (short runs, shared lines, idle lanes, ...) is >= 0; only the preferences in FREE_SIGN may take either
    sign.  Checked by cross-validation over whole problems: how close the first 1 / 10 / 100 / 200 candidates of the
    predicted order come to the best candidate of problems the fit has not seen.  Row kernels and workgroup shapes
    the model has no term for are left out of the fit.  The printed weights are rounded by hand into the source,
    where guard rails outside the measured range (runs under 64 bytes, small problems) are added."""
    import gzip
    from scipy.optimize import lsq_linear
    data = []
    for path in dumps:
        with (gzip.open(path, "rt") if path.endswith(".gz") else open(path)) as fh:
            for line in fh:
                d = json.loads(line)
                if family == "micro":
                    d["rows"] = [r for r in d["rows"] if r["kernel_class"] == ttc.TTC_KERNEL_MICRO]
                else:
                    d["rows"] = [r for r in d["rows"] if r["kernel_class"] not in ONE_SHOT]
                if len(d["rows"]) >= 4:
                    data.append(d)
    features, free_sign = (fit_micro_features, FREE_SIGN_MICRO) if family == "micro" else (fit_features, FREE_SIGN)
    names, X, y, grp = None, [], [], []
    for d in data:
        best = min(r["ms"] for r in d["rows"])
        for r in d["rows"]:
            f = features(r)
            names = names or list(f)
            X.append([f[k] for k in names])
            y.append(np.log(r["ms"] / best))
            grp.append(d["problem"])
    X, y = np.array(X), np.array(y)
    cases = sorted(set(grp))
    index = {c: i for i, c in enumerate(cases)}
    G = np.zeros((len(grp), len(cases)))
    G[np.arange(len(grp)), [index[g] for g in grp]] = 1
    wts = np.exp(-sharpness * y)
    lo = np.array([(-np.inf if k in free_sign else 0.0) for k in names] + [-np.inf] * len(cases))
    hi = np.full(len(lo), np.inf)
    full = np.hstack([X, G]) * wts[:, None]

    def solve(Am, ym):
        keep = np.abs(Am).sum(0) > 0
        x = np.zeros(Am.shape[1])
        nk = int(keep.sum())
        aug = np.vstack([Am[:, keep], ridge * np.eye(nk)])
        x[keep] = lsq_linear(aug, np.concatenate([ym, np.zeros(nk)]), bounds=(lo[keep], hi[keep]), method="trf",
                             lsq_solver="exact").x
        return x

    coef = solve(full, y * wts)
    print(f"# {len(data)} problems, {len(y)} timed candidates, {len(names)} features", file=out)
    print("feature        weight", file=out)
    for k, c in zip(names, coef):
        print(f"{k:12s}  {c:+.4f}", file=out)
    starts = np.cumsum([0] + [len(d["rows"]) for d in data])
    caps = (1, 10, 100, 200)
    q = [None] * len(data)
    for fold in range(folds):
        m = np.ones(len(y), bool)
        held = [j for j in range(len(data)) if j % folds == fold]
        for j in held:
            m[starts[j]:starts[j + 1]] = False
        cf = solve(full[m], (y * wts)[m])
        for j in held:
            pr = X[starts[j]:starts[j + 1]] @ cf[:len(names)]
            ms = np.array([r["ms"] for r in data[j]["rows"]])
            order = np.argsort(pr, kind="stable")
            q[j] = [ms.min() / ms[order[:k]].min() for k in caps] + [ms.min() / ms[:k].min() for k in caps]
    q = np.array(q)
    print("", file=out)
    print("cross-validation over whole problems: best time / best time among the first k candidates", file=out)
    print("                        " + "  ".join(f"first {k:>3}" for k in caps), file=out)
    print("refitted order, mean    " + "  ".join(f"{100 * v:8.2f}%" for v in q[:, :4].mean(0)), file=out)
    print("refitted order, minimum " + "  ".join(f"{100 * v:8.2f}%" for v in q[:, :4].min(0)), file=out)
    print("order in the dump, mean " + "  ".join(f"{100 * v:8.2f}%" for v in q[:, 4:].mean(0)), file=out)
    print("(within the family: the candidates of the other kernel families are left out of both orders)", file=out)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("study", choices=("search", "sweep", "fit"))
    ap.add_argument("dumps", nargs="*", help="fit: the --dump files of earlier search / sweep runs")
    ap.add_argument("--out", default="", help="write the table to this file (default: stdout)")
    ap.add_argument("--limit", type=int, default=0, help="sweep: only the first LIMIT cases")
    ap.add_argument("--family", choices=("box", "micro"), default="box", help="fit: the box kernels' model or the micro-tile kernel's")
    ap.add_argument("--dump", default="", help="also write every candidate's configuration and time (JSON lines; .gz compresses)")
    args = ap.parse_args(argv)
    out = open(args.out, "w") if args.out else sys.stdout
    if args.study == "fit":                      # host only: no GPU, no library call
        if not args.dumps:
            print("studies fit: name at least one --dump file", file=sys.stderr)
            return 2
        print("# python -m paper_1603_02297_amd.studies fit " + " ".join(args.dumps) + f" --family {args.family}", file=out)
        study_fit(out, args.dumps, family=args.family)
        if args.out:
            out.close()
        return 0
    import torch
    if not torch.cuda.is_available():
        print("studies: no GPU visible", file=sys.stderr)
        return 2
    ttc.lib()
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
