"""Pins for the CPU oracle: what the paper and the mathematics fix, written out
independently of the oracle's own code.  None of these tests touches the GPU."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import F32, F64, C64, C128, F32_F64, F64_F32, C64_C128, C128_C64

REAL = {F32: np.float32, F64: np.float64, C64: np.float32, C128: np.float64}
COMPS = {F32: 1, F64: 1, C64: 2, C128: 2}


def prod(xs):
    n = 1
    for x in xs:
        n *= x
    return n


def rand(dtype, n, seed):
    return np.random.default_rng(seed).uniform(-1, 1, n * COMPS[dtype]).astype(REAL[dtype])


def run(dtype, sizes, perm, alpha, beta, A, B0=None, nthreads=1):
    B = np.full(prod(sizes) * COMPS[dtype], np.nan, REAL[dtype]) if B0 is None else B0.copy()
    return oracle.transpose(dtype, sizes, perm, alpha, beta, A, B, nthreads)


def ulp(x, real):
    return float(np.spacing(np.abs(real(x))))


def test_listing_address_map_golden_file():
    """tests/golden/listing_address_map_2x3x4.txt: the address map of the paper's Section 3.5 listing for
    permutation (i3,i2,i1), written by a script that evaluates the printed formula only."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "listing_address_map_2x3x4.txt")
    pairs = [tuple(int(x) for x in line.split()) for line in open(path) if not line.startswith("#")]
    assert len(pairs) == 24 and sorted(a for a, _ in pairs) == list(range(24))
    assert sorted(oracle.element_pairs((2, 3, 4), (2, 1, 0))) == sorted(pairs)
    A = np.arange(24, dtype=np.float32)
    B = run(F32, (2, 3, 4), (2, 1, 0), 1.0, 0.0, A)
    for off_a, off_b in pairs:
        assert B[off_b] == off_a


# -- pin 1: closed-form address map printed in the paper's parallel-code listing (Section 3.5):
#    permutation (i3,i2,i1) reads A[i1 + i2*lda1 + i3*lda2] and writes B[i1*ldb2 + i2*ldb1 + i3].
@pytest.mark.parametrize("sizes", [(2, 3, 4), (5, 1, 3), (7, 6, 5)])
def test_listing_address_map_reversal_3d(sizes):
    s0, s1, s2 = sizes
    lda1, lda2 = s0, s0 * s1          # dense A
    ldb1, ldb2 = s2, s2 * s1          # dense B with extents (s2, s1, s0)
    A = np.arange(prod(sizes), dtype=np.float32)
    B = run(F32, sizes, (2, 1, 0), 1.0, 0.0, A)
    for i3 in range(s2):
        for i2 in range(s1):
            for i1 in range(s0):
                assert B[i1 * ldb2 + i2 * ldb1 + i3] == A[i1 + i2 * lda1 + i3 * lda2]


# -- pin 2: the 2-D case with alpha=1, beta=0 is the ordinary matrix transpose (Section 1).
@pytest.mark.parametrize("m,n", [(1, 1), (3, 5), (8, 2), (17, 13)])
def test_2d_is_textbook_transpose(m, n):
    A = rand(F64, m * n, 1)
    B = run(F64, (m, n), (1, 0), 1.0, 0.0, A)
    for i in range(m):
        for j in range(n):
            assert B[j + i * n] == A[i + j * m]


# -- pin 3: the identity permutation is axpby on the flat arrays (Eq. 1 with Pi = id).
@pytest.mark.parametrize("dtype", [F32, F64])
def test_identity_is_axpby(dtype):
    sizes = (3, 4, 5)
    A, B0 = rand(dtype, 60, 2), rand(dtype, 60, 3)
    B = run(dtype, sizes, (0, 1, 2), 2.0, -1.0, A, B0)       # 2a - b is exact in one rounding
    want = (2.0 * A.astype(np.float64) - B0.astype(np.float64)).astype(REAL[dtype])
    assert np.array_equal(B, want)
    B = run(dtype, sizes, (0, 1, 2), 1.0, 0.0, A, B0)
    assert np.array_equal(B, A)


# -- pin 4: Pi followed by its inverse reproduces A bit for bit.
@pytest.mark.parametrize("seed", range(6))
def test_round_trip_with_inverse(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(2, 7))
    sizes = tuple(int(x) for x in rng.integers(1, 6, n))
    perm = tuple(int(x) for x in rng.permutation(n))
    inv = [0] * n
    for j, k in enumerate(perm):
        inv[k] = j
    A = rand(F32, prod(sizes), seed)
    B = run(F32, sizes, perm, 1.0, 0.0, A)
    sizes_b = tuple(sizes[perm[j]] for j in range(n))
    back = run(F32, sizes_b, tuple(inv), 1.0, 0.0, B)
    assert np.array_equal(back, A)


# -- pin 5: applying p then q equals applying the composed permutation once.
@pytest.mark.parametrize("seed", range(6))
def test_composition(seed):
    rng = np.random.default_rng(200 + seed)
    n = int(rng.integers(2, 6))
    sizes = tuple(int(x) for x in rng.integers(1, 6, n))
    p = tuple(int(x) for x in rng.permutation(n))
    q = tuple(int(x) for x in rng.permutation(n))
    A = rand(F64, prod(sizes), seed)
    B = run(F64, sizes, p, 1.0, 0.0, A)
    sizes_b = tuple(sizes[p[j]] for j in range(n))
    C = run(F64, sizes_b, q, 1.0, 0.0, B)
    # index j of C is index q[j] of B, which is index p[q[j]] of A
    pq = tuple(p[q[j]] for j in range(n))
    assert np.array_equal(C, run(F64, sizes, pq, 1.0, 0.0, A))


# -- pin 6: merged-index invariant, the paper's own example (Section 3, stage (1)):
#    Pi(i1,i2,i3) = (i2,i3,i1) is the 2-D transposition (i~2, i1) with size(i~2) = size(i2)*size(i3).
@pytest.mark.parametrize("sizes", [(2, 3, 4), (5, 2, 7), (1, 4, 3)])
def test_merge_example(sizes):
    s0, s1, s2 = sizes
    A, B0 = rand(F32, prod(sizes), 5), rand(F32, prod(sizes), 6)
    B3 = run(F32, sizes, (1, 2, 0), 1.5, 0.5, A, B0)
    B2 = run(F32, (s0, s1 * s2), (1, 0), 1.5, 0.5, A, B0)
    assert np.array_equal(B3, B2)


# -- pin 7: C walker vs the definition written out element by element, every permutation
#    of up to 4 indices on tiny extents (includes non-involutions, where perm and its
#    inverse differ).
@pytest.mark.parametrize("n", [1, 2, 3, 4])
def test_walker_vs_element_map_all_perms(n):
    extents = [1, 2, 3, 5]
    for perm in itertools.permutations(range(n)):
        for shift in range(2):
            sizes = tuple(extents[(k + shift + perm[0]) % 4] for k in range(n))
            A = np.arange(1, prod(sizes) + 1, dtype=np.float64)
            B = run(F64, sizes, perm, 1.0, 0.0, A)
            emap = oracle.element_map(sizes, perm)
            assert sorted(emap) == list(range(prod(sizes)))       # a bijection
            for off_a, off_b in enumerate(emap):
                assert B[off_b] == A[off_a], (sizes, perm, off_a)


def test_element_map_by_hand():
    # sizes (2,3), perm (1,0): A[i + 2j] -> B[j + 3i]
    assert oracle.element_map((2, 3), (1, 0)) == [0, 3, 1, 4, 2, 5]
    # sizes (2,2,2), perm (1,2,0): B index order (i1,i2,i0): off_b = i1 + 2*i2 + 4*i0
    assert oracle.element_map((2, 2, 2), (1, 2, 0)) == [0, 4, 1, 5, 2, 6, 3, 7]


# -- pin 8: numpy.transpose on Fortran-ordered arrays is an independent implementation of
#    the same definition (B.shape[j] = A.shape[perm[j]]).
@pytest.mark.parametrize("seed", range(8))
def test_matches_numpy_fortran_transpose(seed):
    rng = np.random.default_rng(300 + seed)
    n = int(rng.integers(2, 7))
    sizes = tuple(int(x) for x in rng.integers(1, 7, n))
    perm = tuple(int(x) for x in rng.permutation(n))
    A = rand(F32, prod(sizes), seed)
    B = run(F32, sizes, perm, 1.0, 0.0, A, nthreads=1 + seed % 3)
    want = np.transpose(A.reshape(sizes, order="F"), perm).reshape(-1, order="F")
    assert np.array_equal(B, want)


def test_complex_permutation_moves_pairs():
    sizes, perm = (3, 4, 2), (2, 0, 1)
    A = rand(C64, prod(sizes), 9)
    B = run(C64, sizes, perm, 1.0, 0.0, A)
    z = A.view(np.complex64)
    want = np.transpose(z.reshape(sizes, order="F"), perm).reshape(-1, order="F")
    assert np.array_equal(B.view(np.complex64), want)


# -- pin 9: the alpha/beta arithmetic against exact rational arithmetic.
@pytest.mark.parametrize("dtype,alpha,beta", [
    (F32, 1.5, 0.0), (F32, 0.75, 1.25), (F32, 2.0, -1.0), (F32, -0.3, 0.7),
    (F64, 0.75, 1.25), (F64, 1.5, 0.0), (F64, 1.0 / 3.0, -2.0 / 7.0),
    (C64, 0.5 + 0.5j, 1.0 + 0.0j), (C64, 0.3 - 0.2j, 0.0), (C64, -1.25 + 2j, 0.5 - 0.75j),
    (C128, 0.5 + 0.5j, 1.0 + 0.0j), (C128, 0.1 + 0.7j, -0.3 + 0.9j),
])
def test_alpha_beta_against_exact_rationals(dtype, alpha, beta):
    sizes, perm = (3, 2, 4), (2, 0, 1)
    real = REAL[dtype]
    A, B0 = rand(dtype, prod(sizes), 11), rand(dtype, prod(sizes), 12)
    B = run(dtype, sizes, perm, alpha, beta, A, B0)
    exact = oracle.exact_expected(dtype, sizes, perm, alpha, beta, A, B0)
    # error budget of the fixed evaluation order: every rounded intermediate contributes
    # half an ulp of its own magnitude; all magnitudes here are below 8.
    eps = float(np.finfo(real).eps)
    for got, want in zip(B, exact):
        err = abs(Fraction(float(got)) - want)
        if COMPS[dtype] == 1 and beta == 0:
            assert err <= Fraction(ulp(got, real)) / 2                 # one rounding
        elif COMPS[dtype] == 1:
            # t = round(beta*b); r = round(alpha*a + t)
            assert err <= Fraction(ulp(got, real)) / 2 + Fraction(eps) * 2
        else:
            assert err <= Fraction(eps) * 16


def test_exact_one_rounding_case_is_bit_exact():
    # alpha=2, beta=-1: 2a - b has one rounding under any evaluation order
    sizes, perm = (4, 3, 5), (1, 2, 0)
    A, B0 = rand(F32, 60, 21), rand(F32, 60, 22)
    B = run(F32, sizes, perm, 2.0, -1.0, A, B0)
    want_lin = (2.0 * A.astype(np.float64))
    emap = oracle.element_map(sizes, perm)
    for off_a, off_b in enumerate(emap):
        assert B[off_b] == np.float32(want_lin[off_a] - np.float64(B0[off_b]))


def test_beta_zero_never_reads_b():
    sizes, perm = (3, 5, 2), (1, 0, 2)
    A = rand(F32, 30, 31)
    for alpha in (1.0, 1.5):
        B = run(F32, sizes, perm, alpha, 0.0, A, np.full(30, np.nan, np.float32))
        assert not np.isnan(B).any()
    Bc = run(C64, sizes, perm, 0.5 + 0.5j, 0.0, rand(C64, 30, 32), np.full(60, np.nan, np.float32))
    assert not np.isnan(Bc).any()


def test_alpha_zero_is_not_special():
    A = np.array([np.nan, 1.0], dtype=np.float32)
    B = run(F32, (2,), (0,), 0.0, 0.0, A)
    assert np.isnan(B[0]) and B[1] == 0.0


def test_size_one_extents_change_nothing():
    A = rand(F64, 24, 41)
    B1 = run(F64, (2, 1, 3, 1, 4), (4, 1, 0, 3, 2), 1.0, 0.0, A)
    B2 = run(F64, (2, 3, 4), (2, 0, 1), 1.0, 0.0, A)
    assert np.array_equal(B1, B2)


def test_threads_give_identical_results():
    sizes, perm = (7, 5, 6, 3), (2, 0, 3, 1)
    A, B0 = rand(F32, prod(sizes), 51), rand(F32, prod(sizes), 52)
    ref = run(F32, sizes, perm, 0.75, 1.25, A, B0, nthreads=1)
    for t in (2, 3, 8):
        assert np.array_equal(ref, run(F32, sizes, perm, 0.75, 1.25, A, B0, nthreads=t))


def test_rejects_what_the_definition_does_not_cover():
    A = np.zeros(6, np.float32)
    for sizes, perm in [((2, 3), (0, 0)), ((2, 3), (0, 2))]:
        with pytest.raises(ValueError):
            oracle.transpose(F32, sizes, perm, 1.0, 0.0, A, np.zeros(6, np.float32))
    with pytest.raises(ValueError):
        oracle.transpose(F32, (2, 3), (1, 0), 1.0, 0.0, A, A)


# ======================================================================================
# Sub-tensors (paper Table 1, --lda / --ldb; Section 3: "a portion of larger tensors").
# ======================================================================================

def test_ld_pairs_by_hand():
    # sizes 2x2 inside A of leading dimension 3 and B of leading dimension 4, matrix transpose:
    # A offset i0 + 3*i1 goes to B offset i1 + 4*i0.
    assert oracle.element_pairs((2, 2), (1, 0), lda=(3, 2), ldb=(4, 2)) == [(0, 0), (1, 4), (3, 1), (4, 5)]
    assert oracle.strides((2, 5, 3), (4, 6, 3)) == [1, 4, 24]
    assert oracle.span((2, 5, 3), (4, 6, 3)) == 1 + 1 + 4 * 4 + 2 * 24


def test_ld_equal_to_size_is_the_dense_operation():
    sizes, perm = (5, 3, 4), (2, 0, 1)
    A, B0 = rand(F32, 60, 61), rand(F32, 60, 62)
    dense = run(F32, sizes, perm, 0.75, 1.25, A, B0)
    ld = oracle.transpose(F32, sizes, perm, 0.75, 1.25, A, B0.copy(), 1, lda=sizes, ldb=(4, 5, 3))
    assert np.array_equal(dense, ld)


def _random_ld_problem(seed, n=None):
    rng = np.random.default_rng(seed)
    n = n or int(rng.integers(2, 5))
    sizes = tuple(int(x) for x in rng.integers(1, 6, n))
    perm = tuple(int(x) for x in rng.permutation(n))
    lda = tuple(s + int(x) for s, x in zip(sizes, rng.integers(0, 3, n)))
    ldb = tuple(sizes[perm[j]] + int(x) for j, x in zip(range(n), rng.integers(0, 3, n)))
    return sizes, perm, lda, ldb


@pytest.mark.parametrize("seed", range(10))
@pytest.mark.parametrize("alpha,beta", [(1.0, 0.0), (2.0, -1.0)])
def test_subtensor_matches_numpy_slicing(seed, alpha, beta):
    # numpy does the addressing: the enclosing arrays are Fortran-ordered, the sub-tensors are slices of
    # them.  alpha=2, beta=-1 has a single rounding, so the values are fixed bit for bit too.
    sizes, perm, lda, ldb = _random_ld_problem(100 + seed)
    n = len(sizes)
    PA, PB0 = rand(F32, prod(lda), 200 + seed), rand(F32, prod(ldb), 300 + seed)
    PB = oracle.transpose(F32, sizes, perm, alpha, beta, PA, PB0.copy(), 1, lda=lda, ldb=ldb)
    want = PB0.reshape(ldb, order="F").copy(order="F")
    sub_a = PA.reshape(lda, order="F")[tuple(slice(0, s) for s in sizes)]
    sl_b = tuple(slice(0, sizes[perm[j]]) for j in range(n))
    moved = np.transpose(sub_a, perm).astype(np.float64)
    if beta == 0.0:
        want[sl_b] = moved.astype(np.float32)
    else:
        want[sl_b] = (2.0 * moved - want[sl_b].astype(np.float64)).astype(np.float32)
    assert np.array_equal(PB, want.reshape(-1, order="F"))      # inside AND outside the sub-tensor


@pytest.mark.parametrize("n", [1, 2, 3])
def test_walker_vs_strided_element_pairs(n):
    for seed in range(4):
        sizes, _, lda, _ = _random_ld_problem(400 + 10 * n + seed, n)
        for perm in itertools.permutations(range(n)):
            ldb = tuple(sizes[perm[j]] + (j + seed) % 3 for j in range(n))
            PA = np.arange(prod(lda), dtype=np.float64)             # value = offset in A
            PB = oracle.transpose(F64, sizes, perm, 1.0, 0.0, PA, np.full(prod(ldb), -1.0), 1, lda=lda, ldb=ldb)
            want = np.full(prod(ldb), -1.0)
            for off_a, off_b in oracle.element_pairs(sizes, perm, lda, ldb):
                want[off_b] = off_a
            assert np.array_equal(PB, want)


def test_merge_condition_with_leading_dimensions():
    # Footnote of Section 3, stage (1): indices m, m+1 may merge iff ld(m+1) = size(m) * ld(m), here
    # in both tensors.  A: 4 x 3 x 5 inside 6 x 3 x 5 (index 1 is not padded, so 1 and 2 merge);
    # B = (i1, i2, i0): 3 x 5 x 4 inside 3 x 7 x 4 (index i1 not padded).
    sizes, perm = (4, 3, 5), (1, 2, 0)
    lda, ldb = (6, 3, 5), (3, 7, 4)
    PA = rand(F64, prod(lda), 71)
    PB0 = rand(F64, prod(ldb), 72)
    unfused = oracle.transpose(F64, sizes, perm, 0.75, 1.25, PA, PB0.copy(), 1, lda=lda, ldb=ldb)
    # merged: A is 4 x 15 with leading dimension 6; B is 15 x 4 -- but B's i2 IS padded (7 > 5), so the
    # merge is illegal in B: the merged call must differ, the legal variant (ldb not padded) must agree.
    ldb_ok = (3, 5, 4)
    PB0s = rand(F64, prod(ldb_ok), 73)
    unfused_ok = oracle.transpose(F64, sizes, perm, 0.75, 1.25, PA, PB0s.copy(), 1, lda=lda, ldb=ldb_ok)
    fused_ok = oracle.transpose(F64, (4, 15), (1, 0), 0.75, 1.25, PA, PB0s.copy(), 1, lda=(6, 15), ldb=(15, 4))
    assert np.array_equal(unfused_ok, fused_ok)
    touched = sorted(b for _, b in oracle.element_pairs(sizes, perm, lda, ldb))
    touched_fused = sorted(b for _, b in oracle.element_pairs((4, 15), (1, 0), (6, 15), (15, 4)))
    assert touched != touched_fused and not np.array_equal(unfused[:60], PB0[:60])


def test_ld_smaller_than_size_is_rejected():
    with pytest.raises(ValueError):
        oracle.transpose(F32, (2, 3), (1, 0), 1.0, 0.0, np.zeros(6, np.float32), np.zeros(6, np.float32), 1,
                         lda=(1, 3), ldb=(3, 2))


# ======================================================================================
# Mixed precision (paper Table 1, --dataType sd / ds / cz / zc; Section 3).
# ======================================================================================

A_REAL = {F32_F64: np.float32, F64_F32: np.float64, C64_C128: np.float32, C128_C64: np.float64}
B_REAL = {F32_F64: np.float64, F64_F32: np.float32, C64_C128: np.float64, C128_C64: np.float32}
MCOMPS = {F32_F64: 1, F64_F32: 1, C64_C128: 2, C128_C64: 2}
WIDE = {F32_F64: F64, F64_F32: F64, C64_C128: C128, C128_C64: C128}


def mrand(real, n, seed):
    return np.random.default_rng(seed).uniform(-1, 1, n).astype(real)


@pytest.mark.parametrize("dtype", [F32_F64, F64_F32, C64_C128, C128_C64])
def test_mixed_pure_permutation_is_numpy_cast(dtype):
    # alpha=1, beta=0: the element is moved and converted; numpy's astype rounds to nearest even.
    sizes, perm = (3, 4, 2, 5), (2, 0, 3, 1)
    c = MCOMPS[dtype]
    A = mrand(A_REAL[dtype], prod(sizes) * c, 81)
    B = oracle.transpose(dtype, sizes, perm, 1.0, 0.0, A, np.full(prod(sizes) * c, np.nan, B_REAL[dtype]))
    if c == 1:
        want = np.transpose(A.reshape(sizes, order="F"), perm).reshape(-1, order="F").astype(B_REAL[dtype])
    else:
        z = A.reshape(-1, 2)
        zz = (z[:, 0] + 1j * z[:, 1]).reshape(sizes, order="F")
        w = np.transpose(zz, perm).reshape(-1, order="F")
        want = np.stack([w.real, w.imag], axis=1).reshape(-1).astype(B_REAL[dtype])
    assert np.array_equal(B, want)


@pytest.mark.parametrize("dtype,alpha,beta", [
    (F32_F64, 0.75, 1.25), (F32_F64, 1.0 / 3.0, 0.0), (F64_F32, 0.75, 1.25), (F64_F32, 1.0 / 3.0, 0.0),
    (C64_C128, 0.5 + 0.5j, 1.0 + 0.0j), (C128_C64, 0.1 + 0.7j, -0.3 + 0.9j), (C128_C64, 0.3 - 0.2j, 0.0),
])
def test_mixed_is_the_double_precision_operation_on_widened_data(dtype, alpha, beta):
    # The reading: widen (exact), compute as the double-precision operation does, round once to B's type.
    # The double-precision operation is pinned above; widening and rounding are numpy's.
    sizes, perm = (4, 3, 5), (1, 2, 0)
    c = MCOMPS[dtype]
    A = mrand(A_REAL[dtype], prod(sizes) * c, 91)
    B0 = mrand(B_REAL[dtype], prod(sizes) * c, 92)
    got = oracle.transpose(dtype, sizes, perm, alpha, beta, A, B0.copy())
    wide = oracle.transpose(WIDE[dtype], sizes, perm, alpha, beta, A.astype(np.float64), B0.astype(np.float64))
    assert np.array_equal(got, wide.astype(B_REAL[dtype]))


@pytest.mark.parametrize("dtype", [F32_F64, F64_F32])
def test_mixed_against_exact_rationals(dtype):
    sizes, perm = (3, 2, 4), (2, 0, 1)
    A, B0 = mrand(A_REAL[dtype], 24, 95), mrand(B_REAL[dtype], 24, 96)
    got = oracle.transpose(dtype, sizes, perm, 0.3, -0.7, A, B0.copy())
    exact = oracle.exact_expected(dtype, sizes, perm, 0.3, -0.7, A, B0)
    eps64 = float(np.finfo(np.float64).eps)
    for g, want in zip(got, exact):
        err = abs(Fraction(float(g)) - want)
        assert err <= Fraction(ulp(g, B_REAL[dtype])) / 2 + Fraction(eps64) * 4
