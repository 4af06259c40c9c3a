"""CPU oracle for B[Pi(i)] <- alpha*A[i] + beta*B[Pi(i)] (paper Eq. 1).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this module;
its callers are the tests, the smoke check and the cpu_baseline leg of the benchmark.
It shares no code with the HIP library and never imports it.

Two independent formulations live here:

* :func:`transpose` -- the plain C walker in ``ttc_oracle.c`` (B visited linearly,
  the loop order of the paper's reference routine, Section 4.2), loaded with ctypes.
* :func:`element_map` / :func:`exact_expected` -- a pure-Python element-by-element
  evaluation of the definition for tiny tensors: every linear offset of A is split
  into its multi-index by div/mod and sent to its place in B (Eq. 1), values in exact
  rational arithmetic.  It is what the C walker is pinned against.

Tensors are flat, column-major (leftmost index has stride 1; paper Section 1);
``perm[j]`` is the index of A that becomes index j of B.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from fractions import Fraction

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ttc_oracle.c")
_LIB = os.path.join(_HERE, "libttc_oracle.so")

F32, F64, C64, C128 = 0, 1, 2, 3
# A and B of different precision (paper Table 1, --dataType sd / ds / cz / zc): first letter A, second B
F32_F64, F64_F32, C64_C128, C128_C64 = 4, 5, 6, 7
_NP_A = {F32: np.float32, F64: np.float64, C64: np.float32, C128: np.float64,
         F32_F64: np.float32, F64_F32: np.float64, C64_C128: np.float32, C128_C64: np.float64}
_NP_B = {F32: np.float32, F64: np.float64, C64: np.float32, C128: np.float64,
         F32_F64: np.float64, F64_F32: np.float32, C64_C128: np.float64, C128_C64: np.float32}
# alpha, beta and the arithmetic: the data type, or double precision for the mixed types
_NP_REAL = {F32: np.float32, F64: np.float64, C64: np.float32, C128: np.float64,
            F32_F64: np.float64, F64_F32: np.float64, C64_C128: np.float64, C128_C64: np.float64}
_COMPONENTS = {F32: 1, F64: 1, C64: 2, C128: 2, F32_F64: 1, F64_F32: 1, C64_C128: 2, C128_C64: 2}


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (contraction off, OpenMP on)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.ttc_oracle_transpose.restype = ctypes.c_int
        _lib.ttc_oracle_transpose.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int),
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        _lib.ttc_oracle_transpose_ld.restype = ctypes.c_int
        _lib.ttc_oracle_transpose_ld.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int),
            ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int64),
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
    return _lib


def scalar_array(dtype: int, value) -> np.ndarray:
    """One scalar of `dtype` as a real numpy array (two reals for complex types)."""
    real = _NP_REAL[dtype]
    if _COMPONENTS[dtype] == 2:
        z = complex(value)
        return np.array([z.real, z.imag], dtype=real)
    return np.array([value], dtype=real)


def strides(extents, ld=None):
    """Column-major element strides: stride[0] = 1, stride[k] = stride[k-1] * ld[k-1] (ld = extents if None)."""
    ld = list(extents) if ld is None else list(ld)
    out, st = [], 1
    for k in range(len(extents)):
        out.append(st)
        st *= int(ld[k])
    return out


def span(extents, ld=None) -> int:
    """Number of elements from the first to the last element of the (sub-)tensor, inclusive."""
    return 1 + sum((int(e) - 1) * st for e, st in zip(extents, strides(extents, ld)))


def transpose(dtype: int, sizes, perm, alpha, beta, A: np.ndarray, B: np.ndarray,
              nthreads: int = 1, lda=None, ldb=None) -> np.ndarray:
    """Run the C walker in place on B and return B.

    A and B are flat C-contiguous numpy arrays of the real component type of their side
    (interleaved re/im for complex types).  Dense: length prod(sizes).  With lda / ldb
    (extents of the enclosing tensors, per index of A / of B) they hold at least the span
    of the sub-tensor, which starts at element 0; elements outside it are left alone.
    """
    lib = _load()
    n = len(sizes)
    comps = _COMPONENTS[dtype]
    if len(perm) != n or sorted(int(p) for p in perm) != list(range(n)):
        raise ValueError("perm is not a permutation of the indices")
    size_b = [int(sizes[perm[j]]) for j in range(n)]
    need_a = span([int(x) for x in sizes], lda)
    need_b = span(size_b, ldb)
    for name, arr, real, need in (("A", A, _NP_A[dtype], need_a), ("B", B, _NP_B[dtype], need_b)):
        if arr.dtype != real or not arr.flags.c_contiguous or arr.ndim != 1:
            raise ValueError(f"{name}: need a flat contiguous {real.__name__} array")
        if (lda is None and ldb is None and arr.size != need * comps) or arr.size < need * comps:
            raise ValueError(f"{name}: need {need * comps} values, got {arr.size}")
    if np.shares_memory(A, B):
        raise ValueError("A and B overlap")
    c_sizes = (ctypes.c_int64 * n)(*[int(x) for x in sizes])
    c_perm = (ctypes.c_int * n)(*[int(p) for p in perm])
    c_lda = (ctypes.c_int64 * n)(*[int(x) for x in lda]) if lda is not None else None
    c_ldb = (ctypes.c_int64 * n)(*[int(x) for x in ldb]) if ldb is not None else None
    a = scalar_array(dtype, alpha)
    b = scalar_array(dtype, beta)
    rc = lib.ttc_oracle_transpose_ld(dtype, n, c_sizes, c_perm, c_lda, c_ldb, a.ctypes.data, b.ctypes.data,
                                     A.ctypes.data, B.ctypes.data, int(nthreads))
    if rc != 0:
        raise ValueError(f"ttc_oracle_transpose_ld rejected its arguments (code {rc})")
    return B


# ----------------------------------------------------------------------------------
# Definition written out element by element (tiny tensors only).
# ----------------------------------------------------------------------------------

def element_pairs(sizes, perm, lda=None, ldb=None):
    """(offset in A, offset in B) of every element, in A's index order (Eq. 1).

    Pure Python: a counter over A's elements is split into the multi-index (i_0..i_{N-1}) by
    div/mod with i_0 fastest; B's j-th index is i_{perm[j]}; offsets are index times stride,
    strides from the leading dimensions (column-major, see :func:`strides`).
    """
    n = len(sizes)
    total = 1
    for s in sizes:
        total *= s
    size_b = [sizes[perm[j]] for j in range(n)]
    st_a, st_b = strides(sizes, lda), strides(size_b, ldb)
    out = []
    for count in range(total):
        rest, idx = count, []
        for k in range(n):
            idx.append(rest % sizes[k])
            rest //= sizes[k]
        off_a = sum(idx[k] * st_a[k] for k in range(n))
        off_b = sum(idx[perm[j]] * st_b[j] for j in range(n))
        out.append((off_a, off_b))
    return out


def element_map(sizes, perm):
    """Dense tensors: for every linear offset of A, the linear offset of B it is sent to."""
    return [off_b for _, off_b in element_pairs(sizes, perm)]


def exact_expected(dtype: int, sizes, perm, alpha, beta, A: np.ndarray, B0: np.ndarray, lda=None, ldb=None):
    """Exact value of alpha*A[i] + beta*B0[Pi(i)] at every B offset, as Fractions.

    Returns a list of length B0.size (components interleaved for complex types); positions
    outside a sub-tensor hold None.  With beta == 0 the old B does not enter (it is
    overwritten, never read).  alpha and beta are first rounded to the precision the
    operation takes them in.
    """
    comps = _COMPONENTS[dtype]
    pairs = element_pairs(sizes, perm, lda, ldb)
    fa = [Fraction(float(x)) for x in A]
    fb = [Fraction(float(x)) for x in B0]
    out = [None] * len(fb)
    if comps == 1:
        al, be = Fraction(float(_NP_REAL[dtype](alpha))), Fraction(float(_NP_REAL[dtype](beta)))
        for off_a, off_b in pairs:
            out[off_b] = al * fa[off_a] + (be * fb[off_b] if be != 0 else 0)
    else:
        a = scalar_array(dtype, alpha)
        b = scalar_array(dtype, beta)
        ar, ai = Fraction(float(a[0])), Fraction(float(a[1]))
        br, bi = Fraction(float(b[0])), Fraction(float(b[1]))
        beta_zero = (br == 0 and bi == 0)
        for off_a, off_b in pairs:
            xr, xi = fa[2 * off_a], fa[2 * off_a + 1]
            re, im = ar * xr - ai * xi, ar * xi + ai * xr
            if not beta_zero:
                yr, yi = fb[2 * off_b], fb[2 * off_b + 1]
                re += br * yr - bi * yi
                im += br * yi + bi * yr
            out[2 * off_b], out[2 * off_b + 1] = re, im
    return out
