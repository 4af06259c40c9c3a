"""Host logic of the library (no GPU): validation, size-1 removal, index fusion, case split,
candidate list, and -- through the library's host-side replay of its own index arithmetic --
that every candidate's walk stays in bounds and realises the element map of Eq. 1."""
import itertools

import numpy as np
import pytest

import oracle
import paper_1603_02297_amd as ttc
from paper_1603_02297_amd import workloads as wl


def plan(dtype, sizes, perm, alpha=None, beta=None):
    return ttc.ttc_plan_create(dtype, len(sizes), sizes, perm, alpha, beta)


def info_of(dtype, sizes, perm, alpha=None, beta=None):
    p = plan(dtype, sizes, perm, alpha, beta)
    try:
        return ttc.ttc_plan_get_info(p)
    finally:
        ttc.ttc_plan_destroy(p)


# ---- validation -------------------------------------------------------------------
@pytest.mark.parametrize("args,status", [
    ((ttc.TTC_F32, 0, (), ()), ttc.TTC_ERR_INVALID_VALUE),
    ((ttc.TTC_F32, 7, (2,) * 7, tuple(range(7))), ttc.TTC_ERR_INVALID_VALUE),
    ((ttc.TTC_F32, 2, (4, 0), (1, 0)), ttc.TTC_ERR_INVALID_VALUE),
    ((ttc.TTC_F32, 2, (4, -3), (1, 0)), ttc.TTC_ERR_INVALID_VALUE),
    ((ttc.TTC_F32, 2, (4, 4), (1, 1)), ttc.TTC_ERR_INVALID_PERM),
    ((ttc.TTC_F32, 2, (4, 4), (0, 2)), ttc.TTC_ERR_INVALID_PERM),
    ((ttc.TTC_F32, 2, (4, 4), (-1, 0)), ttc.TTC_ERR_INVALID_PERM),
    ((8, 2, (4, 4), (1, 0)), ttc.TTC_ERR_UNSUPPORTED_DTYPE),
    ((-1, 2, (4, 4), (1, 0)), ttc.TTC_ERR_UNSUPPORTED_DTYPE),
    ((ttc.TTC_F64, 3, (2 ** 31, 2 ** 31, 2 ** 10), (2, 1, 0)), ttc.TTC_ERR_OVERFLOW),
])
def test_create_rejects(args, status):
    with pytest.raises(ttc.TtcError) as e:
        ttc.ttc_plan_create(*args)
    assert e.value.status == status
    assert ttc.ttc_last_status() == status


def test_create_ex_rejects_short_leading_dimensions():
    for lda, ldb in [((3, 5), None), (None, (4, 4)), ((4, 5), (5, 3))]:
        with pytest.raises(ttc.TtcError) as e:
            ttc.ttc_plan_create_ex(ttc.TTC_F32, 2, (4, 5), (1, 0), lda, ldb)
        assert e.value.status == ttc.TTC_ERR_INVALID_VALUE
    p = ttc.ttc_plan_create_ex(ttc.TTC_F32, 2, (4, 5), (1, 0), (4, 5), (5, 4))
    i = ttc.ttc_plan_get_info(p)
    assert i["span_a"] == 20 and i["span_b"] == 20
    ttc.ttc_plan_destroy(p)


def test_destroy_null_is_noop():
    ttc.ttc_plan_destroy(None)


def test_defaults_are_alpha_one_beta_zero():
    # defaults of the paper's Table 1
    assert info_of(ttc.TTC_F32, (8, 8), (1, 0))["epilogue"] == ttc.TTC_EPI_COPY
    assert info_of(ttc.TTC_F32, (8, 8), (1, 0), 1.5, 0.0)["epilogue"] == ttc.TTC_EPI_SCALE
    assert info_of(ttc.TTC_F32, (8, 8), (1, 0), 1.0, 1.0)["epilogue"] == ttc.TTC_EPI_AXPBY
    assert info_of(ttc.TTC_C64, (8, 8), (1, 0), 1.0 + 0j, 0.0)["epilogue"] == ttc.TTC_EPI_COPY
    assert info_of(ttc.TTC_C64, (8, 8), (1, 0), 1.0 + 1j, 0.0)["epilogue"] == ttc.TTC_EPI_SCALE


# ---- index fusion (paper Section 3, stage (1)) ---------------------------------------
def test_paper_merge_example():
    # Pi(i1,i2,i3) = (i2,i3,i1) becomes the 2-D (i~2, i1) with size(i~2) = size(i2)*size(i3)
    i = info_of(ttc.TTC_F32, (5, 6, 7), (1, 2, 0))
    assert i["ndim"] == 2 and i["sizes"] == [5, 42] and i["perm"] == [1, 0]


def test_config_fusions():
    i = info_of(ttc.TTC_F64, (72,) * 4, (2, 3, 0, 1))
    assert i["ndim"] == 2 and i["sizes"] == [5184, 5184] and i["perm"] == [1, 0]
    i = info_of(ttc.TTC_F32, (24, 20, 16, 18, 22, 17), (1, 0, 2, 3, 5, 4))
    assert i["ndim"] == 5 and i["sizes"] == [24, 20, 288, 22, 17] and i["perm"] == [1, 0, 2, 4, 3]
    i = info_of(ttc.TTC_F32, (4, 5, 6), (0, 1, 2))
    assert i["ndim"] == 1 and i["sizes"] == [120] and i["perm"] == [0] and i["stride1_fixed"] == 1
    for perm in [(5, 3, 1, 0, 4, 2), (5, 4, 3, 2, 1, 0)]:
        assert info_of(ttc.TTC_F32, (24, 20, 16, 18, 22, 17), perm)["ndim"] == 6      # nothing merges


def test_size_one_extents_are_dropped_then_fused():
    i = info_of(ttc.TTC_F32, (4, 1, 5, 1, 6), (2, 1, 4, 3, 0))     # without the 1s: (4,5,6) perm (1,2,0)
    assert i["ndim"] == 2 and i["sizes"] == [4, 30] and i["perm"] == [1, 0]
    i = info_of(ttc.TTC_F32, (1, 1, 1), (2, 0, 1))
    assert i["ndim"] == 1 and i["sizes"] == [1] and i["elements"] == 1


def test_fusion_is_maximal_and_consistent():
    rng = np.random.default_rng(7)
    for _ in range(200):
        n = int(rng.integers(1, 7))
        sizes = tuple(int(x) for x in rng.integers(1, 5, n))
        perm = tuple(int(x) for x in rng.permutation(n))
        i = info_of(ttc.TTC_F32, sizes, perm)
        m, fs, fp = i["ndim"], i["sizes"], i["perm"]
        assert sorted(fp) == list(range(m))
        assert int(np.prod(fs)) == int(np.prod(sizes)) == i["elements"]
        for j in range(m - 1):
            assert fp[j + 1] != fp[j] + 1          # nothing left to merge
        if m > 1:
            assert all(s > 1 for s in fs)
        # the fused problem has the same element map as the original one
        if i["elements"] <= 400:
            assert oracle.element_map(sizes, perm) == oracle.element_map(tuple(fs), tuple(fp))


def test_fusion_respects_leading_dimensions():
    # footnote of Section 3 stage (1): i_m, i_{m+1} merge only if ld(i_{m+1}) = size(i_m) * ld(i_m), in A and in B
    def fused(lda, ldb):
        p = ttc.ttc_plan_create_ex(ttc.TTC_F32, 3, (5, 6, 7), (1, 2, 0), lda, ldb)
        try:
            return ttc.ttc_plan_get_info(p)
        finally:
            ttc.ttc_plan_destroy(p)
    i = fused(None, None)
    assert i["ndim"] == 2 and i["sizes"] == [5, 42]
    i = fused((8, 6, 7), (6, 7, 9))                # padding only on indices that do not sit inside the merged pair
    assert i["ndim"] == 2 and i["sizes"] == [5, 42] and i["stride_a"] == [1, 8] and i["stride_b"] == [42, 1]
    i = fused((5, 9, 7), None)                     # A's index 1 is padded: 1 and 2 are not contiguous in A
    assert i["ndim"] == 3 and i["stride_a"] == [1, 5, 45]
    i = fused(None, (8, 7, 5))                     # B's index 0 (= i1) is padded: not contiguous in B
    assert i["ndim"] == 3 and i["stride_b"] == [56, 1, 8]
    assert i["span_b"] == 1 + 5 * 1 + 6 * 8 + 4 * 56


def test_size_one_extent_with_padding_keeps_the_strides():
    p = ttc.ttc_plan_create_ex(ttc.TTC_F32, 3, (4, 1, 6), (2, 1, 0), (5, 3, 6), (7, 2, 4))
    i = ttc.ttc_plan_get_info(p)
    ttc.ttc_plan_destroy(p)
    assert i["ndim"] == 2 and i["sizes"] == [4, 6] and i["stride_a"] == [1, 15] and i["stride_b"] == [14, 1]


# ---- case split (paper Section 3.1) ------------------------------------------------------
def test_case_split_on_the_benchmark_cases():
    for c in wl.CASES:
        i = info_of(c.dtype, c.sizes, c.perm, c.alpha, c.beta)
        fixed = (i["perm"][0] == 0)
        assert i["stride1_fixed"] == int(fixed)
        assert fixed == (c.perm == (0, 2, 1))
        if fixed:
            assert i["kernel_class"] == ttc.TTC_KERNEL_ROWS          # 1536-byte rows: gathered whole
        else:
            assert i["kernel_class"] in (ttc.TTC_KERNEL_LDS, ttc.TTC_KERNEL_MICRO)     # both stage the tile through LDS
        assert i["bytes_moved"] == c.traffic_bytes
        assert i["lds_bytes"] <= 160 * 1024
        assert 0 < i["candidate_count"]


def test_candidates_are_ranked_and_have_a_scalar_fallback():
    p = plan(ttc.TTC_F32, (48, 36, 20), (2, 0, 1))
    n = ttc.ttc_plan_candidate_count(p)
    costs, scalar = [], False
    for k in range(n):
        ttc.ttc_plan_select_candidate(p, k)
        i = ttc.ttc_plan_get_info(p)
        costs.append(i["heuristic_cost"])
        scalar |= (i["vec_a"] == 1 and i["vec_b"] == 1)
        assert i["tile"][0] % i["vec_a"] == 0 and i["tile"][i["perm"][0]] % i["vec_b"] == 0
    assert scalar
    # candidate 0 is the one the plan was created with (the best of a short list); the appended fallback may sit out of order
    assert costs[1:-1] == sorted(costs[1:-1]) and costs[0] <= 1.25 * costs[1]
    with pytest.raises(ttc.TtcError):
        ttc.ttc_plan_select_candidate(p, n)
    ttc.ttc_plan_destroy(p)


# ---- every candidate's walk, replayed on the host, is the element map of Eq. 1 ----------------
def check_all_candidates(dtype, sizes, perm, max_candidates=None, lda=None, ldb=None):
    p = ttc.ttc_plan_create_ex(dtype, len(sizes), sizes, perm, lda, ldb)
    total = oracle.span([sizes[perm[j]] for j in range(len(sizes))], ldb)
    assert total == ttc.ttc_plan_get_info(p)["span_b"]
    want = [-1] * total
    for off_a, off_b in oracle.element_pairs(sizes, perm, lda, ldb):
        want[off_b] = off_a
    n = ttc.ttc_plan_candidate_count(p)
    idx = range(n) if max_candidates is None or n <= max_candidates else \
        sorted(set(np.linspace(0, n - 1, max_candidates).astype(int).tolist()))
    for k in idx:
        ttc.ttc_plan_select_candidate(p, k)
        got = ttc.ttc_debug_emulate_map(p, total)
        assert list(got) == want, (sizes, perm, k, ttc.ttc_plan_get_info(p))
    ttc.ttc_plan_destroy(p)
    return n


@pytest.mark.parametrize("n", [1, 2, 3, 4])
def test_walks_all_perms_small_odd_extents(n):
    ext = [3, 5, 7, 2]
    for perm in itertools.permutations(range(n)):
        sizes = tuple(ext[(k + perm[0]) % 4] for k in range(n))
        check_all_candidates(ttc.TTC_F32, sizes, perm, max_candidates=12)


@pytest.mark.parametrize("dtype", [ttc.TTC_F32, ttc.TTC_F64, ttc.TTC_C64, ttc.TTC_C128, ttc.TTC_F32_F64,
                                   ttc.TTC_F64_F32, ttc.TTC_C64_C128, ttc.TTC_C128_C64])
@pytest.mark.parametrize("sizes,perm", [
    ((70, 66), (1, 0)),                 # several tiles, ragged tails on both indices
    ((64, 64), (1, 0)),
    ((129, 3, 67), (2, 1, 0)),
    ((40, 36, 5), (0, 2, 1)),           # stride-1 index fixed, long rows
    ((4, 50, 30), (0, 2, 1)),           # stride-1 index fixed, short rows
    ((6, 5, 4, 7, 3, 5), (5, 3, 1, 0, 4, 2)),
    ((12, 10, 9, 11), (1, 0, 3, 2)),
    ((8, 16, 6, 5, 10), (4, 1, 3, 0, 2)),
    ((1000,), (0,)),
    ((2, 3, 5, 7, 11, 13), (5, 4, 3, 2, 1, 0)),
])
def test_walks_shapes_with_tails(dtype, sizes, perm):
    check_all_candidates(dtype, sizes, perm, max_candidates=24)


@pytest.mark.parametrize("dtype,sizes,perm", [
    (ttc.TTC_F32, (70, 50), (1, 0)),            # ragged on both indices: last vectors and blocks moved back
    (ttc.TTC_F32, (133, 67), (1, 0)),           # remainder tiles of less than one vector
    (ttc.TTC_F64, (35, 35, 35), (2, 1, 0)),
    (ttc.TTC_F64, (72, 3, 72), (2, 1, 0)),      # tiles of 72: 36 vectors a row, no power of two
    (ttc.TTC_F32, (96, 2, 96), (2, 0, 1)),
    (ttc.TTC_F32, (12, 5, 7, 9), (3, 2, 1, 0)),         # short leading extents: two indices taken as one, on both sides
    (ttc.TTC_F64, (6, 7, 5, 9), (3, 1, 0, 2)),          # ... on one side only (B's second index is A's second index)
    (ttc.TTC_C64, (8, 5, 4, 10), (3, 1, 2, 0)),
])
def test_walks_of_every_micro_tile_candidate(dtype, sizes, perm):
    p = ttc.ttc_plan_create_ex(dtype, len(sizes), sizes, perm)
    want = [-1] * int(np.prod(sizes))
    for off_a, off_b in oracle.element_pairs(sizes, perm, None, None):
        want[off_b] = off_a
    seen = 0
    for k in range(ttc.ttc_plan_candidate_count(p)):
        ttc.ttc_plan_select_candidate(p, k)
        if ttc.ttc_plan_get_info(p)["kernel_class"] != ttc.TTC_KERNEL_MICRO:
            continue
        seen += 1
        assert list(ttc.ttc_debug_emulate_map(p, len(want))) == want, (sizes, perm, k, ttc.ttc_plan_get_info(p))
    assert seen >= 8
    ttc.ttc_plan_destroy(p)


def test_micro_tile_kernel_updates_every_element_of_a_ragged_tensor_once():
    """beta != 0: moved-back vectors and blocks must not update an element twice; the replay then insists on one
    write per element (without an update of B a second write with the same source is allowed)."""
    for sizes, perm in (((70, 50), (1, 0)), ((133, 67), (1, 0)), ((12, 5, 7, 9), (3, 2, 1, 0))):
        want = [-1] * int(np.prod(sizes))
        for off_a, off_b in oracle.element_pairs(sizes, perm, None, None):
            want[off_b] = off_a
        p = ttc.ttc_plan_create(ttc.TTC_F32, len(sizes), sizes, perm, 1.0, 0.5)
        seen = 0
        for k in range(ttc.ttc_plan_candidate_count(p)):
            ttc.ttc_plan_select_candidate(p, k)
            if ttc.ttc_plan_get_info(p)["kernel_class"] != ttc.TTC_KERNEL_MICRO:
                continue
            seen += 1
            assert list(ttc.ttc_debug_emulate_map(p, len(want))) == want, (sizes, perm, k, ttc.ttc_plan_get_info(p))
        assert seen >= 8
        ttc.ttc_plan_destroy(p)


def test_walks_random_5d_6d():
    rng = np.random.default_rng(11)
    for _ in range(12):
        n = int(rng.integers(5, 7))
        sizes, perm = wl.random_problem(rng, n, 20000, 12)
        check_all_candidates(ttc.TTC_F32, sizes, perm, max_candidates=6)


def test_library_walks_realise_the_listing_address_map():
    """The golden address map of the paper's Section 3.5 listing, against every candidate's replayed walk."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "listing_address_map_2x3x4.txt")
    pairs = [tuple(int(x) for x in line.split()) for line in open(path) if not line.startswith("#")]
    want = [-1] * 24
    for off_a, off_b in pairs:
        want[off_b] = off_a
    p = plan(ttc.TTC_F32, (2, 3, 4), (2, 1, 0))
    for k in range(ttc.ttc_plan_candidate_count(p)):
        ttc.ttc_plan_select_candidate(p, k)
        assert list(ttc.ttc_debug_emulate_map(p)) == want
    ttc.ttc_plan_destroy(p)


# ---- sub-tensors (paper Table 1, --lda / --ldb) ------------------------------------------------
@pytest.mark.parametrize("dtype", [ttc.TTC_F32, ttc.TTC_F64, ttc.TTC_C128_C64])
@pytest.mark.parametrize("sizes,perm,lda,ldb", [
    ((70, 66), (1, 0), (75, 66), (67, 70)),
    ((64, 64), (1, 0), (64, 64), (96, 64)),
    ((33, 5, 40), (2, 1, 0), (36, 5, 41), (40, 7, 33)),
    ((40, 36, 5), (0, 2, 1), (43, 36, 5), (40, 6, 36)),          # stride-1 index fixed
    ((4, 50, 30), (0, 2, 1), (4, 51, 30), (5, 30, 50)),
    ((6, 5, 4, 7, 3), (4, 1, 3, 0, 2), (7, 5, 5, 7, 3), (3, 6, 8, 6, 4)),
    ((12, 10, 9, 11), (0, 1, 3, 2), (13, 10, 9, 11), (12, 10, 11, 9)),   # indices 0,1 adjacent but A padded
    ((500,), (0,), (700,), (512,)),
    ((9, 1, 8), (2, 1, 0), (9, 4, 8), (8, 3, 10)),
    ((1, 8, 6, 10), (1, 2, 0, 3), (2, 9, 8, 10), (9, 7, 3, 14)),     # size-1 first index, padded: no stride-1 index in A
    ((8, 1, 6), (1, 0, 2), (8, 3, 6), (2, 9, 6)),                    # the same in B
])
def test_walks_subtensors(dtype, sizes, perm, lda, ldb):
    check_all_candidates(dtype, sizes, perm, max_candidates=16, lda=lda, ldb=ldb)


def test_walks_random_subtensors():
    rng = np.random.default_rng(23)
    for i in range(48):
        n = int(rng.integers(1, 7))
        sizes, perm = wl.random_problem(rng, n, 12000, 14)
        lda = tuple(s + int(x) for s, x in zip(sizes, rng.integers(0, 4, n)))
        ldb = tuple(sizes[perm[j]] + int(x) for j, x in zip(range(n), rng.integers(0, 4, n)))
        check_all_candidates(i % 8, sizes, perm, max_candidates=5, lda=lda, ldb=ldb)


# ---- persistent store of search results (paper Section 3: the database of previous solutions) --------
CONFIG_FIELDS = ("kernel_class", "tile", "tile_order", "vec_a", "vec_b", "threads", "wg_per_cu", "lds_buffers",
                 "digit_tile_a", "digit_lane_a", "digit_tile_b", "digit_lane_b", "lds_bytes")


def config_of(p):
    i = ttc.ttc_plan_get_info(p)
    return {k: i[k] for k in CONFIG_FIELDS}


def test_plan_store_round_trip(tmp_path):
    path = str(tmp_path / "plans.txt")
    sizes, perm = (48, 36, 20), (2, 0, 1)
    p = plan(ttc.TTC_F32, sizes, perm, 1.5, 0.0)
    assert ttc.ttc_plan_cache_lookup(p, path) is False                 # no file yet
    n = ttc.ttc_plan_candidate_count(p)
    ttc.ttc_plan_select_candidate(p, n // 3)
    ttc.ttc_plan_set_tile_mapping(p, 3)                                # the stored solution carries its tile mapping
    chosen = config_of(p)
    ttc.ttc_plan_cache_store(p, path)
    ttc.ttc_plan_destroy(p)

    q = plan(ttc.TTC_F32, sizes, perm, 1.5, 0.0)
    assert ttc.ttc_plan_get_info(q)["candidate_index"] == 0
    assert ttc.ttc_plan_cache_lookup(q, path) is True
    assert config_of(q) == chosen and ttc.ttc_plan_get_info(q)["candidate_index"] == n // 3
    assert ttc.ttc_plan_get_info(q)["xcd_remap"] == 3
    ttc.ttc_plan_destroy(q)

    # alpha does not enter the key, beta == 0 does; neither do unrelated problems match
    q = plan(ttc.TTC_F32, sizes, perm, 1.0, 0.0)
    assert ttc.ttc_plan_cache_lookup(q, path) is True
    ttc.ttc_plan_destroy(q)
    for other in [plan(ttc.TTC_F32, sizes, perm, 1.5, 0.5), plan(ttc.TTC_F64, sizes, perm, 1.5, 0.0),
                  plan(ttc.TTC_F32, sizes, (1, 0, 2), 1.5, 0.0), plan(ttc.TTC_F32, (48, 36, 21), perm, 1.5, 0.0),
                  ttc.ttc_plan_create_ex(ttc.TTC_F32, 3, sizes, perm, (50, 36, 20), None, 1.5, 0.0)]:
        assert ttc.ttc_plan_cache_lookup(other, path) is False
        assert ttc.ttc_plan_get_info(other)["candidate_index"] == 0
        ttc.ttc_plan_destroy(other)


def test_plan_store_later_entry_wins_and_damage_is_ignored(tmp_path):
    path = str(tmp_path / "plans.txt")
    p = plan(ttc.TTC_F64, (40, 30), (1, 0))
    ttc.ttc_plan_select_candidate(p, 5)
    ttc.ttc_plan_cache_store(p, path)
    ttc.ttc_plan_select_candidate(p, 9)
    second = config_of(p)
    ttc.ttc_plan_cache_store(p, path)
    ttc.ttc_plan_select_candidate(p, 0)
    assert ttc.ttc_plan_cache_lookup(p, path) is True and config_of(p) == second
    # an entry naming a configuration this library does not build is skipped
    lines = open(path).read().splitlines()
    key, sig, us = lines[-1].split("|")
    broken = sig.split()
    broken[1] = "192"                                                  # a workgroup size no candidate has
    with open(path, "w") as f:
        f.write(key + "| " + " ".join(broken) + " |" + us + "\n")
    ttc.ttc_plan_select_candidate(p, 0)
    assert ttc.ttc_plan_cache_lookup(p, path) is False
    with open(path, "w") as f:
        f.write(key + "| 1 2 x |" + us + "\n")
    assert ttc.ttc_plan_cache_lookup(p, path) is False
    assert ttc.ttc_plan_get_info(p)["candidate_index"] == 0
    ttc.ttc_plan_destroy(p)
    with pytest.raises(ttc.TtcError) as e:
        q = plan(ttc.TTC_F64, (40, 30), (1, 0))
        try:
            ttc.ttc_plan_cache_store(q, str(tmp_path / "no_such_dir" / "plans.txt"))
        finally:
            ttc.ttc_plan_destroy(q)
    assert e.value.status == ttc.TTC_ERR_IO


def test_walks_with_cut_vectors():
    """Odd extents: candidates that use full-width vectors and cut the last one of every run."""
    seen = 0
    for dtype, sizes, perm in [(ttc.TTC_F32, (35, 37), (1, 0)), (ttc.TTC_F32, (19, 19, 19), (2, 1, 0)),
                               (ttc.TTC_F64, (21, 5, 33), (2, 0, 1)), (ttc.TTC_F32, (45, 9, 7), (0, 2, 1)),
                               (ttc.TTC_C64, (27, 31), (1, 0)), (ttc.TTC_F64_F32, (17, 3, 23), (2, 1, 0))]:
        p = plan(dtype, sizes, perm)
        want = [-1] * int(np.prod(sizes))
        for off_a, off_b in oracle.element_pairs(sizes, perm):
            want[off_b] = off_a
        for k in range(ttc.ttc_plan_candidate_count(p)):
            ttc.ttc_plan_select_candidate(p, k)
            i = ttc.ttc_plan_get_info(p)
            if not (i["partial_a"] or i["partial_b"]) or seen % 7:
                seen += bool(i["partial_a"] or i["partial_b"])
                continue
            seen += 1
            assert list(ttc.ttc_debug_emulate_map(p)) == want, (sizes, perm, k, i)
        ttc.ttc_plan_destroy(p)
    assert seen > 50


def test_cut_vectors_never_overlap_where_b_is_read():
    """beta != 0: an overlapping vector would read elements of B its neighbour may already have updated."""
    for dtype, sizes, perm in [(ttc.TTC_F32, (35, 37), (1, 0)), (ttc.TTC_F32, (45, 9, 7), (0, 2, 1)),
                               (ttc.TTC_F64, (21, 5, 33), (2, 0, 1))]:
        p = plan(dtype, sizes, perm, 0.75, 1.25)
        want = [-1] * int(np.prod(sizes))
        for off_a, off_b in oracle.element_pairs(sizes, perm):
            want[off_b] = off_a
        cut_a = 0
        for k in range(ttc.ttc_plan_candidate_count(p)):
            ttc.ttc_plan_select_candidate(p, k)
            i = ttc.ttc_plan_get_info(p)
            assert i["partial_b"] == 0
            if i["kernel_class"] == ttc.TTC_KERNEL_DIRECT:
                assert i["partial_a"] == 0
            if i["partial_a"] and cut_a % 5 == 0:
                assert list(ttc.ttc_debug_emulate_map(p)) == want, (sizes, perm, k, i)
            cut_a += i["partial_a"]
        ttc.ttc_plan_destroy(p)


# ---- non-temporal accesses (paper Table 1: streaming stores) -----------------------------------
def test_streaming_rule_and_override():
    p = plan(ttc.TTC_F32, (384, 384, 384), (2, 1, 0), 1.5, 0.0)         # every run is whole 128-byte lines
    i = ttc.ttc_plan_get_info(p)
    assert i["nt_a"] == 1 and i["nt_b"] == 1
    ttc.ttc_plan_set_streaming(p, 0, -1)
    i = ttc.ttc_plan_get_info(p)
    assert i["nt_a"] == 0 and i["nt_b"] == 1
    ttc.ttc_plan_set_streaming(p, -1, 0)
    i = ttc.ttc_plan_get_info(p)
    assert i["nt_a"] == 1 and i["nt_b"] == 0
    with pytest.raises(ttc.TtcError):
        ttc.ttc_plan_set_streaming(p, 2, 0)
    ttc.ttc_plan_destroy(p)
    p = plan(ttc.TTC_F32, (85, 85, 85), (2, 1, 0))                      # 340-byte rows: lines are shared
    i = ttc.ttc_plan_get_info(p)
    assert i["nt_a"] == 0 and i["nt_b"] == 0
    ttc.ttc_plan_destroy(p)
    p = plan(ttc.TTC_F32, (384, 24, 24), (0, 2, 1))                     # direct kernel: both sides or neither
    for k in range(ttc.ttc_plan_candidate_count(p)):
        ttc.ttc_plan_select_candidate(p, k)
        if ttc.ttc_plan_get_info(p)["kernel_class"] == ttc.TTC_KERNEL_DIRECT:
            break
    assert ttc.ttc_plan_get_info(p)["kernel_class"] == ttc.TTC_KERNEL_DIRECT
    ttc.ttc_plan_set_streaming(p, 1, 0)
    i = ttc.ttc_plan_get_info(p)
    assert i["nt_a"] == 0 and i["nt_b"] == 0
    ttc.ttc_plan_set_streaming(p, 1, 1)
    i = ttc.ttc_plan_get_info(p)
    assert i["nt_a"] == 1 and i["nt_b"] == 1
    ttc.ttc_plan_destroy(p)


@pytest.mark.parametrize("sizes,perm", [((256, 256), (1, 0)), ((512, 512), (1, 0)), ((1024, 1024), (1, 0)), ((384, 24, 24), (0, 2, 1)),
                                        ((64, 64, 64), (2, 1, 0)), ((24, 24, 24, 24), (3, 2, 1, 0)), ((17, 19, 23, 29), (2, 0, 3, 1))])
def test_first_candidate_of_a_small_problem_spreads_over_the_chip(sizes, perm):
    # outside the range the cost model was fitted on, guard rails keep the first candidate from a few giant tiles
    i = info_of(ttc.TTC_F32, sizes, perm)
    nbytes = 4 * int(np.prod(sizes))
    assert i["num_tiles"] >= min(128, nbytes // 8192), i


@pytest.mark.parametrize("sizes,perm", [((70, 33, 45), (2, 0, 1)), ((19, 7, 23, 5), (3, 1, 0, 2)), ((300, 11), (1, 0)),
                                        ((96, 20, 31), (0, 2, 1)), ((5, 4, 3, 6, 2, 7), (5, 3, 1, 0, 4, 2))])
def test_every_tile_mapping_covers_the_tensor(sizes, perm):
    """How tiles are dealt to the XCDs (round robin, one range each, chunks of 2**k in turn) changes which
    workgroup takes which tile, never what is computed: the replay of every workgroup's walk still writes
    every element of B once, from the element of A the oracle names."""
    want = [-1] * int(np.prod(sizes))
    for off_a, off_b in oracle.element_pairs(sizes, perm, None, None):
        want[off_b] = off_a
    def default_mode(tiles):         # chunks of 32; round robin where a workgroup gets one or two tiles at most
        return 5 if tiles >= 2048 else 0
    p = plan(ttc.TTC_F32, sizes, perm)
    n = ttc.ttc_plan_candidate_count(p)
    for k in sorted({0, n // 7, n // 2, n - 1}):
        ttc.ttc_plan_select_candidate(p, k)
        tiles = ttc.ttc_plan_get_info(p)["num_tiles"]
        assert ttc.ttc_plan_get_info(p)["xcd_remap"] == default_mode(tiles)
        for mode in (0, 1, 2, 3, 5, 8, 10, -1):
            ttc.ttc_plan_set_tile_mapping(p, mode)
            assert ttc.ttc_plan_get_info(p)["xcd_remap"] == (default_mode(tiles) if mode < 0 else mode)
            assert list(ttc.ttc_debug_emulate_map(p)) == want, (k, mode)
    for bad in (-2, 11):
        with pytest.raises(ttc.TtcError):
            ttc.ttc_plan_set_tile_mapping(p, bad)
    ttc.ttc_plan_destroy(p)


def test_default_tile_mapping_follows_the_tile_count():
    # 200 MB problems get chunks of 32 tiles; a problem with a few hundred tiles is dealt round robin, so that
    # no XCD is left without work
    big = info_of(ttc.TTC_F32, (384, 384, 384), (2, 1, 0))
    assert big["num_tiles"] >= 2048 and big["xcd_remap"] == 5
    small = info_of(ttc.TTC_F32, (256, 256), (1, 0))
    assert small["num_tiles"] < 256 and small["xcd_remap"] == 0
