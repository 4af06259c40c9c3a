"""Parity of the HIP path against the CPU oracle for the extensions of the basic operation
(paper Table 1): tensors that are parts of larger ones (--lda / --ldb), complex128, and the
mixed-precision types.  Same bar as the basic parity tests: bit-exact where the result has a
single rounding at most (pure permutations, conversions), at most 1 ulp of B's type otherwise.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
import paper_1603_02297_amd as ttc
from paper_1603_02297_amd import workloads as wl

pytestmark = pytest.mark.gpu

INT_OF = {np.dtype(np.float32): np.int32, np.dtype(np.float64): np.int64}
ALL_TYPES = [wl.F32, wl.F64, wl.C64, wl.C128, wl.F32_F64, wl.F64_F32, wl.C64_C128, wl.C128_C64]
NEW_TYPES = [wl.C128, wl.F32_F64, wl.F64_F32, wl.C64_C128, wl.C128_C64]
REAL_SCALARS = [(1.0, 0.0), (1.5, 0.0), (0.75, 1.25), (1.0 / 3.0, -2.0 / 7.0)]
COMPLEX_SCALARS = [(1.0, 0.0), (0.5 + 0.5j, 0.0), (0.5 + 0.5j, 1.0 + 0.0j), (-1.25 + 2j, 0.5 - 0.75j)]


def scalars(dtype, k):
    table = COMPLEX_SCALARS if wl.COMPONENTS[dtype] == 2 else REAL_SCALARS
    return table[k % len(table)]


def ulp_distance(x, y):
    if np.array_equal(x, y, equal_nan=True):
        return 0
    it = INT_OF[x.dtype]
    xi, yi = x.view(it).astype(np.int64), y.view(it).astype(np.int64)
    lowest = np.int64(np.iinfo(it).min)
    xi = np.where(xi < 0, lowest - xi, xi)
    yi = np.where(yi < 0, lowest - yi, yi)
    return int(np.abs(xi - yi).max())


def prod(xs):
    n = 1
    for x in xs:
        n *= int(x)
    return n


def check(dtype, sizes, perm, alpha, beta, lda=None, ldb=None, seed=0, candidate=None, tune=False, threads=8):
    """A and B are whole enclosing tensors (prod(ld) elements); every element of B is compared,
    inside and outside the sub-tensor."""
    n = len(sizes)
    comps = wl.COMPONENTS[dtype]
    na = prod(lda) if lda is not None else prod(sizes)
    nb = prod(ldb) if ldb is not None else prod(sizes)
    A = wl.uniform_tensor(dtype, na, 3000 + seed, "a")
    B0 = wl.uniform_tensor(dtype, nb, 4000 + seed, "b")
    want = oracle.transpose(dtype, sizes, perm, alpha, beta, A, B0.copy(), threads, lda=lda, ldb=ldb)
    dev = torch.device("cuda:0")
    dA, dB = torch.from_numpy(A).to(dev), torch.from_numpy(B0).to(dev)
    stream = torch.cuda.current_stream().cuda_stream
    plan = ttc.ttc_plan_create_ex(dtype, n, sizes, perm, lda, ldb, alpha, beta)
    try:
        info = ttc.ttc_plan_get_info(plan)
        assert info["span_a"] * comps <= A.size and info["span_b"] * comps <= B0.size
        if candidate is not None:
            ttc.ttc_plan_select_candidate(plan, candidate % info["candidate_count"])
        if tune:
            scratch = dB.clone()
            ttc.ttc_plan_tune(plan, dA.data_ptr(), scratch.data_ptr(), stream, 0)
        ttc.ttc_execute(plan, dA.data_ptr(), dB.data_ptr(), stream)
        torch.cuda.synchronize()
        info = ttc.ttc_plan_get_info(plan)
    finally:
        ttc.ttc_plan_destroy(plan)
    got = dB.cpu().numpy()
    exact = (complex(alpha) == 1 and complex(beta) == 0)         # a move, or one conversion
    d = ulp_distance(got, want)
    assert d <= (0 if exact else 1), (dtype, sizes, perm, lda, ldb, alpha, beta, candidate, d, info)
    return info


SHAPES = [
    ((200, 150), (1, 0)),
    ((129, 3, 67), (2, 1, 0)),
    ((96, 50, 31), (0, 2, 1)),
    ((4, 50, 30), (0, 2, 1)),
    ((6, 5, 4, 7, 3, 5), (5, 3, 1, 0, 4, 2)),
    ((8, 16, 6, 5, 10), (4, 1, 3, 0, 2)),
    ((3000,), (0,)),
]


@pytest.mark.parametrize("dtype", NEW_TYPES, ids=[wl.DTYPE_NAME[d] for d in NEW_TYPES])
@pytest.mark.parametrize("sizes,perm", SHAPES)
def test_new_types_candidates_and_epilogues(dtype, sizes, perm):
    p = ttc.ttc_plan_create_ex(dtype, len(sizes), sizes, perm)
    ncand = ttc.ttc_plan_candidate_count(p)
    ttc.ttc_plan_destroy(p)
    picks = range(ncand) if ncand <= 20 else sorted(set(np.linspace(0, ncand - 1, 20).astype(int).tolist()))
    for k in picks:
        al, be = scalars(dtype, k)
        check(dtype, sizes, perm, al, be, seed=k, candidate=k)


LD_SHAPES = [
    ((200, 150), (1, 0), (203, 150), (151, 200)),
    ((64, 64), (1, 0), (64, 64), (96, 64)),
    ((129, 3, 67), (2, 1, 0), (131, 4, 67), (70, 3, 129)),
    ((96, 50, 31), (0, 2, 1), (100, 50, 31), (96, 33, 50)),           # stride-1 index fixed, both padded
    ((4, 50, 30), (0, 2, 1), (4, 51, 30), (5, 30, 50)),
    ((6, 5, 4, 7, 3, 5), (5, 3, 1, 0, 4, 2), (6, 6, 4, 8, 3, 5), (7, 7, 5, 6, 3, 4)),
    ((12, 10, 9, 11), (0, 1, 3, 2), (13, 10, 9, 11), (12, 10, 11, 9)),
    ((3000,), (0,), (3500,), (3001,)),
    ((9, 1, 8), (2, 1, 0), (9, 4, 8), (8, 3, 10)),
]


@pytest.mark.parametrize("dtype", [wl.F32, wl.F64, wl.C64, wl.C128_C64, wl.F32_F64],
                         ids=["f32", "f64", "c64", "c128c64", "f32f64"])
@pytest.mark.parametrize("sizes,perm,lda,ldb", LD_SHAPES)
def test_subtensors_candidates_and_epilogues(dtype, sizes, perm, lda, ldb):
    p = ttc.ttc_plan_create_ex(dtype, len(sizes), sizes, perm, lda, ldb)
    ncand = ttc.ttc_plan_candidate_count(p)
    ttc.ttc_plan_destroy(p)
    picks = range(ncand) if ncand <= 16 else sorted(set(np.linspace(0, ncand - 1, 16).astype(int).tolist()))
    for k in picks:
        al, be = scalars(dtype, k)
        check(dtype, sizes, perm, al, be, lda, ldb, seed=k, candidate=k)


def test_random_subtensors_all_types():
    rng = np.random.default_rng(29)
    for i in range(24):
        n = int(rng.integers(2, 7))
        sizes, perm = wl.random_problem(rng, n, 200000, 14)
        lda = tuple(s + int(x) for s, x in zip(sizes, rng.integers(0, 3, n)))
        ldb = tuple(sizes[perm[j]] + int(x) for j, x in zip(range(n), rng.integers(0, 3, n)))
        dtype = ALL_TYPES[i % len(ALL_TYPES)]
        al, be = scalars(dtype, i)
        check(dtype, sizes, perm, al, be, lda, ldb, seed=i)


def test_packing_a_panel_of_a_matrix():
    """The use the paper names for leading dimensions (Section 3): pack a panel of a larger matrix
    into a contiguous, transposed buffer.  The panel starts in the middle of the matrix: the
    caller passes the address of its corner."""
    rows, cols, m, k, r0, c0 = 1000, 800, 192, 256, 300, 100
    M = wl.uniform_tensor(wl.F64, rows * cols, 61)
    dev = torch.device("cuda:0")
    dM = torch.from_numpy(M).to(dev)
    dP = torch.full((m * k,), float("nan"), dtype=torch.float64, device=dev)
    plan = ttc.ttc_plan_create_ex(wl.F64, 2, (m, k), (1, 0), (rows, cols), None)
    ttc.ttc_execute(plan, dM.data_ptr() + 8 * (r0 + c0 * rows), dP.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    ttc.ttc_plan_destroy(plan)
    corner = M[r0 + c0 * rows:]
    want = oracle.transpose(wl.F64, (m, k), (1, 0), 1.0, 0.0, corner, np.full(m * k, np.nan), 4, lda=(rows, cols))
    assert np.array_equal(dP.cpu().numpy(), want)
    # and against numpy's own slicing
    assert np.array_equal(want.reshape((k, m), order="F"), M.reshape((rows, cols), order="F")[r0:r0 + m, c0:c0 + k].T)


FULL_SIZE = [
    (wl.F32, (384, 384, 384), (2, 1, 0), (400, 392, 384), (388, 384, 400), 1.5, 0.0),
    (wl.F64, (72, 72, 72, 72), (3, 2, 1, 0), (80, 72, 75, 72), (72, 76, 72, 72), 0.75, 1.25),
    (wl.C128, (72, 40, 72, 72), (3, 0, 2, 1), None, None, 0.5 + 0.5j, 1.0 + 0.0j),
    (wl.F32_F64, (384, 384, 384), (2, 1, 0), None, None, 1.5, 0.0),
    (wl.F64_F32, (24, 20, 16, 18, 22, 17), (5, 3, 1, 0, 4, 2), None, None, 2.0, -1.0),
    (wl.C64_C128, (8, 64, 48, 40, 40), (4, 1, 3, 0, 2), None, None, 0.5 + 0.5j, 0.0),
    (wl.C128_C64, (8, 64, 48, 40, 40), (2, 0, 4, 3, 1), None, None, 1.0, 0.0),
]


@pytest.mark.parametrize("dtype,sizes,perm,lda,ldb,alpha,beta", FULL_SIZE,
                         ids=[f"{wl.DTYPE_NAME[c[0]]}-{'ld' if c[3] else 'dense'}" for c in FULL_SIZE])
def test_full_size_heuristic_and_tuned(dtype, sizes, perm, lda, ldb, alpha, beta):
    """Benchmark-sized tensors, every element compared, heuristic and tuned plan."""
    check(dtype, sizes, perm, alpha, beta, lda, ldb, threads=16)
    check(dtype, sizes, perm, alpha, beta, lda, ldb, threads=16, tune=True)


def test_new_types_reject_misaligned_and_alias():
    dev = torch.device("cuda:0")
    buf = torch.zeros(1 << 16, dtype=torch.float64, device=dev)
    s = torch.cuda.current_stream().cuda_stream
    plan = ttc.ttc_plan_create_ex(wl.C128, 2, (32, 32), (1, 0))
    for a, b, status in [(buf.data_ptr(), buf.data_ptr() + 16 * 512, ttc.TTC_ERR_ALIAS),
                         (buf.data_ptr() + 4, buf.data_ptr() + 65536, ttc.TTC_ERR_MISALIGNED)]:
        with pytest.raises(ttc.TtcError) as e:
            ttc.ttc_execute(plan, a, b, s)
        assert e.value.status == status
    ttc.ttc_plan_destroy(plan)
    # sub-tensors: the ranges up to the last element count, not the element totals
    plan = ttc.ttc_plan_create_ex(wl.F64, 2, (16, 16), (1, 0), (64, 16), None)
    with pytest.raises(ttc.TtcError) as e:
        ttc.ttc_execute(plan, buf.data_ptr(), buf.data_ptr() + 8 * 512, s)      # inside A's span of 976 elements
    assert e.value.status == ttc.TTC_ERR_ALIAS
    ttc.ttc_execute(plan, buf.data_ptr(), buf.data_ptr() + 8 * 1024, s)
    torch.cuda.synchronize()
    ttc.ttc_plan_destroy(plan)


def test_search_results_persist_through_the_plan_store(tmp_path, monkeypatch):
    """With TTC_PLAN_CACHE set, a search stores what it selected and the next plan for the same
    problem takes it from the store without timing anything (paper Section 3)."""
    path = tmp_path / "plans.txt"
    monkeypatch.setenv("TTC_PLAN_CACHE", str(path))
    dev = torch.device("cuda:0")
    sizes, perm = (96, 40, 24), (2, 0, 1)
    n = prod(sizes)
    A = wl.uniform_tensor(wl.F32, n, 7)
    dA = torch.from_numpy(A).to(dev)
    dB = torch.zeros(n, dtype=torch.float32, device=dev)
    s = torch.cuda.current_stream().cuda_stream
    p = ttc.ttc_plan_create(wl.F32, 3, sizes, perm, 1.5, 0.0)
    ttc.ttc_plan_tune(p, dA.data_ptr(), dB.data_ptr(), s, 0)
    first = ttc.ttc_plan_get_info(p)
    ttc.ttc_plan_destroy(p)
    assert path.exists() and len(path.read_text().splitlines()) == 1
    q = ttc.ttc_plan_create(wl.F32, 3, sizes, perm, 1.5, 0.0)
    ttc.ttc_plan_tune(q, dA.data_ptr(), dB.data_ptr(), s, 0)
    second = ttc.ttc_plan_get_info(q)
    assert len(path.read_text().splitlines()) == 1                      # a hit stores nothing new
    assert second["candidate_index"] == first["candidate_index"]
    assert abs(second["tuned_ms"] - first["tuned_ms"]) < 1e-3           # the stored time, not a new measurement
    ttc.ttc_execute(q, dA.data_ptr(), dB.data_ptr(), s)
    torch.cuda.synchronize()
    ttc.ttc_plan_destroy(q)
    want = oracle.transpose(wl.F32, sizes, perm, 1.5, 0.0, A, np.zeros(n, np.float32))
    assert np.array_equal(dB.cpu().numpy(), want)


@pytest.mark.parametrize("dtype,sizes,perm", [
    (wl.F32, (135, 137), (1, 0)), (wl.F32, (19, 19, 19, 19), (3, 2, 1, 0)), (wl.F64, (21, 5, 33, 9), (2, 0, 3, 1)),
    (wl.F32, (45, 9, 37), (0, 2, 1)), (wl.C64, (27, 31, 5), (1, 2, 0)), (wl.F64_F32, (17, 3, 23, 11), (3, 1, 0, 2)),
    (wl.F32_F64, (85, 85, 7), (1, 0, 2)),
], ids=["f32-2d", "f32-4d", "f64-4d", "f32-fixed", "c64-3d", "f64f32-4d", "f32f64-3d"])
def test_cut_vectors(dtype, sizes, perm):
    """Odd extents: the candidates that keep full-width vectors and cut the last one of every run."""
    p = ttc.ttc_plan_create_ex(dtype, len(sizes), sizes, perm)
    picks = []
    for k in range(ttc.ttc_plan_candidate_count(p)):
        ttc.ttc_plan_select_candidate(p, k)
        i = ttc.ttc_plan_get_info(p)
        if i["partial_a"] or i["partial_b"]:
            picks.append(k)
    ttc.ttc_plan_destroy(p)
    assert picks
    for n, k in enumerate(picks[::max(1, len(picks) // 24)]):
        al, be = scalars(dtype, n)
        check(dtype, sizes, perm, al, be, seed=n, candidate=k)


def test_tensor_beyond_4_gib():
    """Byte offsets past 2^32: a 4.5 GB fp32 tensor, every element compared."""
    sizes, perm = (1040, 1024, 1056), (2, 1, 0)
    n = prod(sizes)
    assert n * 4 > 2 ** 32
    A = np.random.default_rng(2 ** 32 + 1).random(n, dtype=np.float32)
    want = oracle.transpose(wl.F32, sizes, perm, 1.0, 0.0, A, np.empty(n, np.float32), 16)
    dev = torch.device("cuda:0")
    dA = torch.from_numpy(A).to(dev)
    dB = torch.empty(n, dtype=torch.float32, device=dev)
    plan = ttc.ttc_plan_create(wl.F32, 3, sizes, perm, None, None)
    ttc.ttc_execute(plan, dA.data_ptr(), dB.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    ttc.ttc_plan_destroy(plan)
    got = dB.cpu().numpy()
    del dA, dB
    assert np.array_equal(got, want)


def test_search_cap_semantics(monkeypatch):
    """max_candidates: 1 keeps the heuristic's choice untimed, a positive cap times that many, -1 all;
    0 takes TTC_MAX_CANDIDATES from the environment (paper Table 1, --maxImplementations)."""
    monkeypatch.delenv("TTC_PLAN_CACHE", raising=False)
    dev = torch.device("cuda:0")
    sizes, perm = (48, 36, 20), (2, 0, 1)
    n = prod(sizes)
    dA = torch.rand(n, dtype=torch.float32, device=dev)
    dB = torch.empty(n, dtype=torch.float32, device=dev)
    s = torch.cuda.current_stream().cuda_stream

    def timed(cap):
        p = ttc.ttc_plan_create(wl.F32, 3, sizes, perm, None, None)
        ttc.ttc_plan_tune(p, dA.data_ptr(), dB.data_ptr(), s, cap)
        count, sel = 0, ttc.ttc_plan_get_info(p)["candidate_index"]
        total = ttc.ttc_plan_candidate_count(p)
        for k in range(total):
            ttc.ttc_plan_select_candidate(p, k)
            count += ttc.ttc_plan_get_info(p)["tuned_ms"] > 0
        ttc.ttc_plan_destroy(p)
        return count, sel, total

    count, sel, total = timed(1)
    assert count == 0 and sel == 0
    count, sel, _ = timed(7)
    assert count == 7 and sel < 7
    count, _, _ = timed(-1)
    assert count == total
    monkeypatch.setenv("TTC_MAX_CANDIDATES", "5")
    count, sel, _ = timed(0)
    assert count == 5 and sel < 5


@pytest.mark.parametrize("dtype,sizes,perm,alpha,beta", [
    (wl.F32, (128, 96, 40), (2, 1, 0), 1.5, 0.0), (wl.F32, (85, 33, 47), (1, 2, 0), 1.0, 0.0),
    (wl.F64, (64, 20, 48), (0, 2, 1), 0.75, 1.25), (wl.C64, (32, 24, 40), (2, 0, 1), 0.5 + 0.5j, 1.0),
], ids=["f32-aligned", "f32-odd", "f64-direct", "c64"])
def test_streaming_accesses_change_nothing_in_the_result(dtype, sizes, perm, alpha, beta):
    n = prod(sizes)
    A = wl.uniform_tensor(dtype, n, 11, "a")
    B0 = wl.uniform_tensor(dtype, n, 12, "b")
    want = oracle.transpose(dtype, sizes, perm, alpha, beta, A, B0.copy(), 4)
    dev = torch.device("cuda:0")
    dA = torch.from_numpy(A).to(dev)
    s = torch.cuda.current_stream().cuda_stream
    plan = ttc.ttc_plan_create(dtype, len(sizes), sizes, perm, alpha, beta)
    for sa, sb in ((0, 0), (1, 1), (1, 0), (0, 1), (-1, -1)):
        ttc.ttc_plan_set_streaming(plan, sa, sb)
        dB = torch.from_numpy(B0).to(dev)
        ttc.ttc_execute(plan, dA.data_ptr(), dB.data_ptr(), s)
        torch.cuda.synchronize()
        assert ulp_distance(dB.cpu().numpy(), want) <= 1, (sa, sb, ttc.ttc_plan_get_info(plan))
    ttc.ttc_plan_destroy(plan)


@pytest.mark.parametrize("dtype,sizes,perm,alpha,beta", [
    (wl.F32, (85, 33, 47), (2, 1, 0), 1.0, 0.0), (wl.F32, (200, 150, 9), (1, 0, 2), 1.5, 0.0),
    (wl.F64, (64, 20, 48), (0, 2, 1), 0.75, 1.25), (wl.C64, (8, 33, 12, 30), (3, 1, 0, 2), 0.5 + 0.5j, 1.0),
], ids=["f32-odd", "f32-ragged", "f64-direct", "c64"])
def test_tile_mappings_change_nothing_in_the_result(dtype, sizes, perm, alpha, beta):
    n = prod(sizes)
    A = wl.uniform_tensor(dtype, n, 31, "a")
    B0 = wl.uniform_tensor(dtype, n, 32, "b")
    want = oracle.transpose(dtype, sizes, perm, alpha, beta, A, B0.copy(), 4)
    dev = torch.device("cuda:0")
    dA = torch.from_numpy(A).to(dev)
    s = torch.cuda.current_stream().cuda_stream
    plan = ttc.ttc_plan_create(dtype, len(sizes), sizes, perm, alpha, beta)
    count = ttc.ttc_plan_candidate_count(plan)
    for k in sorted({0, count // 5, count // 2, count - 1}):
        ttc.ttc_plan_select_candidate(plan, k)
        for mode in (0, 1, 2, 3, 5, 9, -1):
            ttc.ttc_plan_set_tile_mapping(plan, mode)
            dB = torch.from_numpy(B0).to(dev)
            ttc.ttc_execute(plan, dA.data_ptr(), dB.data_ptr(), s)
            torch.cuda.synchronize()
            exact = (complex(alpha) == 1 and complex(beta) == 0)
            assert ulp_distance(dB.cpu().numpy(), want) <= (0 if exact else 1), (k, mode, ttc.ttc_plan_get_info(plan))
    ttc.ttc_plan_destroy(plan)
