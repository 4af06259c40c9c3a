"""Seeded synthetic inputs and the benchmark case table.

This module holds no arithmetic of the transposition itself: it only names the
workloads (shapes, permutations, scalars) and draws their values.  It is the one
module that both the HIP path's callers and the CPU oracle's callers may share.

The shapes follow the design rules of the paper's transposition benchmark
(Section 4.1): tensors of roughly 200 MiB, one shape with about equal extents, shapes
with irregular extents, the full index reversal and one permutation that keeps the
stride-1 index for a given dimensionality.  The paper's own 57-case list is not
reproduced; these cases stand in for it.

Values: uniform on [-1, 1) from numpy's default_rng with a fixed seed per tensor;
complex tensors are interleaved (re, im) pairs drawn as 2n reals.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Tuple

import numpy as np

F32, F64, C64, C128 = 0, 1, 2, 3
F32_F64, F64_F32, C64_C128, C128_C64 = 4, 5, 6, 7          # A's type, then B's (paper Table 1: sd ds cz zc)
DTYPE_NAME = {F32: "f32", F64: "f64", C64: "c64", C128: "c128",
              F32_F64: "f32f64", F64_F32: "f64f32", C64_C128: "c64c128", C128_C64: "c128c64"}
REAL_DTYPE = {F32: np.float32, F64: np.float64, C64: np.float32, C128: np.float64,          # of A
              F32_F64: np.float32, F64_F32: np.float64, C64_C128: np.float32, C128_C64: np.float64}
REAL_DTYPE_B = {F32: np.float32, F64: np.float64, C64: np.float32, C128: np.float64,
                F32_F64: np.float64, F64_F32: np.float32, C64_C128: np.float64, C128_C64: np.float32}
COMPONENTS = {F32: 1, F64: 1, C64: 2, C128: 2, F32_F64: 1, F64_F32: 1, C64_C128: 2, C128_C64: 2}
ELEM_BYTES = {F32: 4, F64: 8, C64: 8, C128: 16, F32_F64: 4, F64_F32: 8, C64_C128: 8, C128_C64: 16}        # of A
ELEM_BYTES_B = {F32: 4, F64: 8, C64: 8, C128: 16, F32_F64: 8, F64_F32: 4, C64_C128: 16, C128_C64: 8}

SEED_BASE = 16030229700


@dataclass(frozen=True)
class Case:
    """One (tensor, permutation, alpha, beta) benchmark case."""
    config: int                 # 1-based workload number
    dtype: int
    sizes: Tuple[int, ...]      # extents of A, index 0 has stride 1
    perm: Tuple[int, ...]       # perm[j] = index of A that becomes index j of B
    alpha: complex
    beta: complex

    @property
    def name(self) -> str:
        p = "".join(str(x) for x in self.perm)
        return f"cfg{self.config}-{DTYPE_NAME[self.dtype]}-p{p}-a{self.alpha:g}-b{self.beta:g}"

    @property
    def elements(self) -> int:
        n = 1
        for s in self.sizes:
            n *= s
        return n

    @property
    def tensor_bytes(self) -> int:
        return self.elements * ELEM_BYTES[self.dtype]

    @property
    def beta_is_zero(self) -> bool:
        return complex(self.beta) == 0

    @property
    def traffic_bytes(self) -> int:
        """Bytes the method must move: read A, write B, and read B when beta != 0
        (the factor 3 of the paper's bandwidth formula, Eq. 2)."""
        return (2 if self.beta_is_zero else 3) * self.tensor_bytes


def _cases():
    out = []
    out.append(Case(1, F32, (1024, 1024), (1, 0), 1.0, 0.0))
    for p in ((2, 1, 0), (1, 0, 2), (0, 2, 1)):
        out.append(Case(2, F32, (384, 384, 384), p, 1.5, 0.0))
    for p in ((3, 2, 1, 0), (1, 0, 3, 2), (2, 3, 0, 1)):
        out.append(Case(3, F64, (72, 72, 72, 72), p, 0.75, 1.25))
    for p in ((5, 3, 1, 0, 4, 2), (1, 0, 2, 3, 5, 4), (5, 4, 3, 2, 1, 0)):
        for al, be in ((1.0, 0.0), (2.0, -1.0)):
            out.append(Case(4, F32, (24, 20, 16, 18, 22, 17), p, al, be))
    for p in ((4, 1, 3, 0, 2), (2, 0, 4, 3, 1)):
        out.append(Case(5, C64, (8, 64, 48, 40, 80), p, 0.5 + 0.5j, 1.0 + 0.0j))
    return tuple(out)


CASES = _cases()          # the 15 cases the headline median is taken over


def uniform_tensor(dtype: int, elements: int, seed: int, side: str = "a") -> np.ndarray:
    """Flat array of the real component type of A (side "a") or of B (side "b"), uniform on [-1, 1)."""
    n = elements * COMPONENTS[dtype]
    rng = np.random.default_rng(seed)
    real = REAL_DTYPE[dtype] if side == "a" else REAL_DTYPE_B[dtype]
    return rng.uniform(-1.0, 1.0, n).astype(real, copy=False)


def case_inputs(case: Case):
    """(A, B0) for a benchmark case: A from seed base+10*config, B0 from the next seed."""
    a = uniform_tensor(case.dtype, case.elements, SEED_BASE + 10 * case.config + 0)
    b = uniform_tensor(case.dtype, case.elements, SEED_BASE + 10 * case.config + 1)
    return a, b


def random_problem(rng: np.random.Generator, ndim: int, max_elements: int, max_extent: int = 40):
    """A random (sizes, perm) with at most max_elements elements, for parity sweeps."""
    while True:
        sizes = tuple(int(x) for x in rng.integers(1, max_extent + 1, ndim))
        n = 1
        for s in sizes:
            n *= s
        if n <= max_elements:
            break
    perm = tuple(int(x) for x in rng.permutation(ndim))
    return sizes, perm
