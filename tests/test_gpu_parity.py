"""Parity of the HIP path against the CPU oracle, element by element, through the C ABI.

Bar: bit-exact for alpha=1, beta=0 (a pure permutation); at most 1 ulp otherwise (both sides
follow one evaluation order with the same fused multiply-adds, so 0 is what is expected).
"""
import itertools
import os

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
import paper_1603_02297_amd as ttc
from paper_1603_02297_amd import workloads as wl

pytestmark = pytest.mark.gpu

REAL = wl.REAL_DTYPE
COMPS = wl.COMPONENTS
INT_OF = {np.dtype(np.float32): np.int32, np.dtype(np.float64): np.int64}


def ulp_distance(x: np.ndarray, y: np.ndarray) -> int:
    """Largest distance in units in the last place between two float arrays of one dtype."""
    if np.array_equal(x, y):
        return 0
    it = INT_OF[x.dtype]
    xi, yi = x.view(it).astype(np.int64), y.view(it).astype(np.int64)
    lowest = np.int64(np.iinfo(it).min)
    xi = np.where(xi < 0, lowest - xi, xi)          # map sign-magnitude to a monotone integer line
    yi = np.where(yi < 0, lowest - yi, yi)
    return int(np.abs(xi - yi).max())


STORE = os.path.join(os.path.dirname(os.path.abspath(ttc.__file__)), "plans", "gfx950_suite.txt")


def gpu_run(dtype, sizes, perm, alpha, beta, A, B0, candidate=None, tune=False, store=None):
    """One ttc_execute on the GPU; returns the resulting B as a numpy array."""
    dev = torch.device("cuda:0")
    dA = torch.from_numpy(A).to(dev)
    dB = torch.from_numpy(B0).to(dev)
    plan = ttc.ttc_plan_create(dtype, len(sizes), sizes, perm, alpha, beta)
    try:
        if candidate is not None:       # the list depends on whether beta is 0: wrap
            ttc.ttc_plan_select_candidate(plan, candidate % ttc.ttc_plan_candidate_count(plan))
        if store is not None:
            assert ttc.ttc_plan_cache_lookup(plan, store), f"{store} holds no usable plan for {sizes} {perm}"
        if tune:
            scratch = torch.empty_like(dB)
            ttc.ttc_plan_tune(plan, dA.data_ptr(), scratch.data_ptr(), torch.cuda.current_stream().cuda_stream, 0)
        ttc.ttc_execute(plan, dA.data_ptr(), dB.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        info = ttc.ttc_plan_get_info(plan)
    finally:
        ttc.ttc_plan_destroy(plan)
    return dB.cpu().numpy(), info


def check(dtype, sizes, perm, alpha, beta, seed=0, candidate=None, nan_b=False, threads=8, tune=False):
    n = int(np.prod(sizes))
    A = wl.uniform_tensor(dtype, n, 1000 + seed)
    B0 = wl.uniform_tensor(dtype, n, 2000 + seed)
    if nan_b:
        B0[:] = np.nan
    want = oracle.transpose(dtype, sizes, perm, alpha, beta, A, B0.copy(), threads)
    got, info = gpu_run(dtype, sizes, perm, alpha, beta, A, B0, candidate, tune)
    pure = (complex(alpha) == 1 and complex(beta) == 0)
    d = ulp_distance(got, want)
    assert d <= (0 if pure else 1), (sizes, perm, alpha, beta, candidate, d, info)
    return d, info


SCALARS = {
    wl.F32: [(1.0, 0.0), (1.5, 0.0), (0.75, 1.25), (2.0, -1.0)],
    wl.F64: [(1.0, 0.0), (1.5, 0.0), (0.75, 1.25)],
    wl.C64: [(1.0, 0.0), (0.5 + 0.5j, 0.0), (0.5 + 0.5j, 1.0 + 0.0j), (-1.25 + 2j, 0.5 - 0.75j)],
}


@pytest.mark.parametrize("dtype", [wl.F32, wl.F64, wl.C64])
@pytest.mark.parametrize("n", [1, 2, 3, 4])
def test_all_perms_small_odd_extents(dtype, n):
    ext = [37, 5, 19, 6]
    for pi, perm in enumerate(itertools.permutations(range(n))):
        sizes = tuple(ext[(k + perm[0]) % 4] for k in range(n))
        al, be = SCALARS[dtype][pi % len(SCALARS[dtype])]
        check(dtype, sizes, perm, al, be, seed=pi)


@pytest.mark.parametrize("dtype", [wl.F32, wl.F64, wl.C64])
@pytest.mark.parametrize("sizes,perm", [
    ((200, 150), (1, 0)),
    ((129, 3, 67), (2, 1, 0)),
    ((96, 50, 31), (0, 2, 1)),
    ((4, 50, 30), (0, 2, 1)),
    ((6, 5, 4, 7, 3, 5), (5, 3, 1, 0, 4, 2)),
    ((12, 10, 9, 11), (1, 0, 3, 2)),
    ((8, 16, 6, 5, 10), (4, 1, 3, 0, 2)),
    ((5000,), (0,)),
    ((2, 3, 5, 7, 11, 13), (5, 4, 3, 2, 1, 0)),
])
def test_every_candidate_every_epilogue(dtype, sizes, perm):
    """Ragged shapes spanning several tiles; the plan's candidate configurations (all of them, or
    48 spread evenly over the ranked list when there are more)."""
    p = ttc.ttc_plan_create(dtype, len(sizes), sizes, perm, None, None)
    ncand = ttc.ttc_plan_candidate_count(p)
    ttc.ttc_plan_destroy(p)
    picks = range(ncand) if ncand <= 48 else sorted(set(np.linspace(0, ncand - 1, 48).astype(int).tolist()))
    for k in picks:
        al, be = SCALARS[dtype][k % len(SCALARS[dtype])]
        check(dtype, sizes, perm, al, be, seed=k, candidate=k)


def test_random_5d_6d():
    rng = np.random.default_rng(5)
    for i in range(20):
        n = int(rng.integers(5, 7))
        sizes, perm = wl.random_problem(rng, n, 300000, 14)
        dtype = (wl.F32, wl.F64, wl.C64)[i % 3]
        al, be = SCALARS[dtype][i % len(SCALARS[dtype])]
        check(dtype, sizes, perm, al, be, seed=i)


def test_beta_zero_never_reads_b():
    for dtype in (wl.F32, wl.F64, wl.C64):
        for al in (1.0, 1.5):
            check(dtype, (70, 33, 9), (2, 0, 1), al, 0.0, nan_b=True)
            check(dtype, (70, 33, 9), (0, 2, 1), al, 0.0, nan_b=True)


def test_size_one_and_degenerate_shapes():
    check(wl.F32, (1,), (0,), 1.0, 0.0)
    check(wl.F32, (1, 1, 1), (2, 0, 1), 2.0, -1.0)
    check(wl.F64, (1, 77, 1, 5), (3, 2, 1, 0), 0.75, 1.25)
    check(wl.F32, (2, 1, 3, 1, 4, 1), (5, 4, 3, 2, 1, 0), 1.0, 0.0)
    check(wl.C64, (3, 2), (1, 0), 0.5 + 0.5j, 1.0)


def test_rejects_alias_null_and_misaligned():
    dev = torch.device("cuda:0")
    buf = torch.zeros(4096, dtype=torch.float32, device=dev)
    plan = ttc.ttc_plan_create(wl.F32, 2, (32, 32), (1, 0), None, None)
    s = torch.cuda.current_stream().cuda_stream
    for a, b, status in [(buf.data_ptr(), buf.data_ptr(), ttc.TTC_ERR_ALIAS),
                         (buf.data_ptr(), buf.data_ptr() + 4 * 512, ttc.TTC_ERR_ALIAS),
                         (0, buf.data_ptr(), ttc.TTC_ERR_NULL_POINTER),
                         (buf.data_ptr() + 2, buf.data_ptr() + 8192, ttc.TTC_ERR_MISALIGNED)]:
        with pytest.raises(ttc.TtcError) as e:
            ttc.ttc_execute(plan, a, b, s)
        assert e.value.status == status
    ttc.ttc_plan_destroy(plan)


def test_pointers_aligned_to_the_element_only():
    """Pointers aligned to the element but not to 16 bytes: the vector kernels still apply and
    give the exact result, writing nothing outside B."""
    dev = torch.device("cuda:0")
    sizes, perm = (64, 48, 5), (1, 0, 2)
    n = int(np.prod(sizes))
    A = wl.uniform_tensor(wl.F32, n, 77)
    want = oracle.transpose(wl.F32, sizes, perm, 1.0, 0.0, A, np.zeros(n, np.float32))
    dA = torch.zeros(n + 8, dtype=torch.float32, device=dev)
    dB = torch.zeros(n + 8, dtype=torch.float32, device=dev)
    dA[1:n + 1] = torch.from_numpy(A).to(dev)
    plan = ttc.ttc_plan_create(wl.F32, 3, sizes, perm, None, None)
    assert ttc.ttc_plan_get_info(plan)["vec_a"] == 4
    ttc.ttc_execute(plan, dA.data_ptr() + 4, dB.data_ptr() + 12, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    ttc.ttc_plan_destroy(plan)
    got = dB.cpu().numpy()
    assert np.array_equal(got[3:n + 3], want)
    assert not got[:3].any() and not got[n + 3:].any()          # nothing written outside B


def test_tuned_plan_is_still_exact():
    d, info = check(wl.F32, (96, 40, 24), (2, 0, 1), 1.5, 0.0, tune=True)
    assert info["tuned_ms"] > 0


def test_non_default_stream():
    dev = torch.device("cuda:0")
    sizes, perm = (80, 60), (1, 0)
    A = wl.uniform_tensor(wl.F64, 4800, 5)
    want = oracle.transpose(wl.F64, sizes, perm, 1.0, 0.0, A, np.zeros(4800))
    dA = torch.from_numpy(A).to(dev)
    dB = torch.zeros(4800, dtype=torch.float64, device=dev)
    st = torch.cuda.Stream()                      # default priority
    torch.cuda.synchronize()
    plan = ttc.ttc_plan_create(wl.F64, 2, sizes, perm, None, None)
    ttc.ttc_execute(plan, dA.data_ptr(), dB.data_ptr(), st.cuda_stream)
    st.synchronize()
    ttc.ttc_plan_destroy(plan)
    assert np.array_equal(dB.cpu().numpy(), want)


@pytest.mark.parametrize("case", wl.CASES, ids=[c.name for c in wl.CASES])
def test_benchmark_cases_full_size(case):
    """The 15 headline cases at full size, every element compared: the heuristic's plan, a plan searched
    here, and the plan of the tracked store -- the launch configuration bench.py times and profiles/ describe."""
    A, B0 = wl.case_inputs(case)
    want = oracle.transpose(case.dtype, case.sizes, case.perm, case.alpha, case.beta, A, B0.copy(), 16)
    for how in ({}, {"tune": True}, {"store": STORE}):
        got, info = gpu_run(case.dtype, case.sizes, case.perm, case.alpha, case.beta, A, B0, **how)
        pure = (complex(case.alpha) == 1 and complex(case.beta) == 0)
        d = ulp_distance(got, want)
        assert d <= (0 if pure else 1), (case.name, how, d, info)


# The weakest shapes of the 57-case benchmark built by the rules of the paper's Section 4.1 (about 200 MiB,
# extents that are multiples of nothing): runs share cache lines with their neighbours and every vector is cut.
ODD_BENCHMARK_SHAPES = [
    ((7241, 7241), (1, 0)),
    ((85, 85, 85, 85), (3, 2, 1, 0)),
    ((35, 35, 35, 35, 35), (4, 3, 2, 1, 0)),
    ((19, 19, 19, 19, 19, 19), (5, 4, 3, 2, 1, 0)),
]


@pytest.mark.parametrize("sizes,perm", ODD_BENCHMARK_SHAPES, ids=["x".join(map(str, s)) for s, _ in ODD_BENCHMARK_SHAPES])
def test_odd_benchmark_shapes_full_size(sizes, perm):
    """Inverse permutations of odd extents at benchmark size, heuristic and searched plan, bit-exact."""
    n = int(np.prod(sizes))
    A = wl.uniform_tensor(wl.F32, n, 5700 + len(sizes))
    B0 = wl.uniform_tensor(wl.F32, n, 5800 + len(sizes))
    want = oracle.transpose(wl.F32, sizes, perm, 1.0, 0.0, A, B0.copy(), 16)
    for tune in (False, True):
        got, info = gpu_run(wl.F32, sizes, perm, 1.0, 0.0, A, B0, tune=tune)
        assert np.array_equal(got, want), (sizes, perm, tune, info)


# ---- every candidate of the one-shot kernel families on ragged shapes -----------------------------------------
@pytest.mark.gpu
@pytest.mark.parametrize("dtype,sizes,perm,alpha,beta", [
    (wl.F32, (70, 50), (1, 0), 1.0, 0.0),              # moved-back vectors and blocks on both indices
    (wl.F32, (133, 67), (1, 0), 1.5, 0.0),             # remainder tiles narrower than a vector
    (wl.F32, (133, 67), (1, 0), 0.75, 1.25),           # ... with B read as well: every element updated once
    (wl.F64, (35, 35, 35), (2, 1, 0), 2.0, -1.0),
    (wl.F64, (35, 35, 35), (2, 1, 0), 1.0, 0.0),
    (wl.F64, (72, 5, 72), (2, 1, 0), 0.75, 1.25),      # tiles of 72 (36 vectors a row), B read as well
    (wl.C64, (24, 7, 40), (2, 0, 1), 0.5 + 0.5j, 1.0 + 0.0j),
    (wl.F32, (12, 10, 7, 9, 11), (4, 3, 2, 1, 0), 1.0, 0.0),     # two indices taken as one on both sides, ragged
    (wl.F32, (12, 10, 7, 9, 11), (4, 3, 2, 1, 0), 0.75, 1.25),
    (wl.F32, (24, 20, 5, 22, 16), (4, 3, 2, 1, 0), 2.0, -1.0),   # ... whole vectors, B read as well
    (wl.F64, (6, 7, 5, 9), (3, 1, 0, 2), 1.5, 0.0),              # ... on one side only
    (wl.F32, (96, 20, 31), (0, 2, 1), 1.5, 0.0),       # stride-1 index fixed: the row kernel's candidates
    (wl.F32, (85, 9, 13), (0, 2, 1), 2.0, 0.0),        # rows that are no multiple of the vector
])
def test_every_candidate_of_the_one_shot_families(dtype, sizes, perm, alpha, beta):
    n = int(np.prod(sizes))
    A = wl.uniform_tensor(dtype, n, 4100)
    B0 = wl.uniform_tensor(dtype, n, 4200)
    want = oracle.transpose(dtype, sizes, perm, alpha, beta, A, B0.copy(), 4)
    pure = (complex(alpha) == 1 and complex(beta) == 0)
    dev = torch.device("cuda:0")
    dA, dB0 = torch.from_numpy(A).to(dev), torch.from_numpy(B0).to(dev)
    stream = torch.cuda.current_stream().cuda_stream
    plan = ttc.ttc_plan_create(dtype, len(sizes), sizes, perm, alpha, beta)
    try:
        ran = 0
        for k in range(ttc.ttc_plan_candidate_count(plan)):
            ttc.ttc_plan_select_candidate(plan, k)
            info = ttc.ttc_plan_get_info(plan)
            if info["kernel_class"] not in (ttc.TTC_KERNEL_MICRO, ttc.TTC_KERNEL_ROWS):
                continue
            dB = dB0.clone()
            ttc.ttc_execute(plan, dA.data_ptr(), dB.data_ptr(), stream)
            torch.cuda.synchronize()
            d = ulp_distance(dB.cpu().numpy(), want)
            assert d <= (0 if pure else 1), (sizes, perm, k, d, info)
            ran += 1
        assert ran >= 4, (sizes, perm, ran)
    finally:
        ttc.ttc_plan_destroy(plan)


@pytest.mark.gpu
def test_random_problems_through_the_micro_tile_families():
    """Random 3-D to 6-D shapes with odd extents, every element type the micro-tile kernel takes, with and without
    an update of B: the best-ranked candidates over single and over merged indices against the oracle."""
    rng = np.random.default_rng(1603)
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    ran = {1: 0, 2: 0}
    for trial in range(36):
        ndim = int(rng.integers(3, 7))
        sizes, perm = wl.random_problem(rng, ndim, 400000, 26)
        dtype = (wl.F32, wl.F64, wl.C64)[trial % 3]
        alpha, beta = SCALARS[dtype][trial % len(SCALARS[dtype])]
        n = int(np.prod(sizes))
        A = wl.uniform_tensor(dtype, n, 5000 + trial)
        B0 = wl.uniform_tensor(dtype, n, 6000 + trial)
        want = oracle.transpose(dtype, sizes, perm, alpha, beta, A, B0.copy(), 4)
        pure = (complex(alpha) == 1 and complex(beta) == 0)
        dA, dB0 = torch.from_numpy(A).to(dev), torch.from_numpy(B0).to(dev)
        plan = ttc.ttc_plan_create(dtype, len(sizes), sizes, perm, alpha, beta)
        try:
            taken = {1: 0, 2: 0}
            for k in range(ttc.ttc_plan_candidate_count(plan)):
                ttc.ttc_plan_select_candidate(plan, k)
                info = ttc.ttc_plan_get_info(plan)
                if info["kernel_class"] != ttc.TTC_KERNEL_MICRO:
                    continue
                fam = 2 if info["merged"] else 1
                if taken[fam] >= 3:
                    continue
                taken[fam] += 1
                dB = dB0.clone()
                ttc.ttc_execute(plan, dA.data_ptr(), dB.data_ptr(), stream)
                torch.cuda.synchronize()
                d = ulp_distance(dB.cpu().numpy(), want)
                assert d <= (0 if pure else 1), (sizes, perm, alpha, beta, k, d, info)
                ran[fam] += 1
        finally:
            ttc.ttc_plan_destroy(plan)
    assert ran[1] >= 20 and ran[2] >= 20, ran
