"""ctypes binding of libttc.so: the same names as the C ABI in include/ttc.h, argument
marshalling only.  Every step of the transposition runs inside the library's kernels; there
is no Python or CPU fallback -- if the library is missing, loading fails loudly."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libttc.so")

TTC_MAX_DIM = 6
TTC_F32, TTC_F64, TTC_C64, TTC_C128 = 0, 1, 2, 3
TTC_F32_F64, TTC_F64_F32, TTC_C64_C128, TTC_C128_C64 = 4, 5, 6, 7      # A's type, then B's
TTC_OK = 0
(TTC_ERR_INVALID_VALUE, TTC_ERR_INVALID_PERM, TTC_ERR_UNSUPPORTED_DTYPE, TTC_ERR_NULL_POINTER,
 TTC_ERR_ALIAS, TTC_ERR_OVERFLOW, TTC_ERR_HIP, TTC_ERR_ALLOC, TTC_ERR_MISALIGNED, TTC_ERR_INTERNAL,
 TTC_ERR_NOT_FOUND, TTC_ERR_IO) = range(1, 13)
TTC_KERNEL_DIRECT, TTC_KERNEL_LDS, TTC_KERNEL_ROWS, TTC_KERNEL_MICRO = 0, 1, 2, 3
TTC_EPI_COPY, TTC_EPI_SCALE, TTC_EPI_AXPBY = 0, 1, 2

EXPORTS = (
    "ttc_plan_create", "ttc_plan_create_ex", "ttc_execute", "ttc_plan_destroy", "ttc_last_status", "ttc_status_string",
    "ttc_plan_get_info", "ttc_plan_candidate_count", "ttc_plan_select_candidate", "ttc_plan_tune",
    "ttc_plan_tune_pairs", "ttc_time_execute", "ttc_time_ceiling", "ttc_debug_emulate_map",
    "ttc_plan_cache_store", "ttc_plan_cache_lookup", "ttc_plan_set_streaming", "ttc_plan_set_tile_mapping",
)


class ttc_plan_info_t(ctypes.Structure):
    _fields_ = [
        ("dtype", ctypes.c_int), ("ndim", ctypes.c_int),
        ("sizes", ctypes.c_int64 * TTC_MAX_DIM), ("perm", ctypes.c_int * TTC_MAX_DIM),
        ("stride1_fixed", ctypes.c_int), ("kernel_class", ctypes.c_int), ("epilogue", ctypes.c_int),
        ("tile", ctypes.c_int * TTC_MAX_DIM), ("digits_a", ctypes.c_int), ("digits_b", ctypes.c_int),
        ("digit_tile_a", ctypes.c_int * 4), ("digit_lane_a", ctypes.c_int * 4),
        ("digit_tile_b", ctypes.c_int * 4), ("digit_lane_b", ctypes.c_int * 4),
        ("tile_order", ctypes.c_int * TTC_MAX_DIM),
        ("lds_stride", ctypes.c_int * TTC_MAX_DIM),
        ("vec_a", ctypes.c_int), ("vec_b", ctypes.c_int), ("partial_a", ctypes.c_int), ("partial_b", ctypes.c_int),
        ("threads", ctypes.c_int), ("wg_per_cu", ctypes.c_int),
        ("xcd_remap", ctypes.c_int), ("lds_bytes", ctypes.c_int), ("lds_buffers", ctypes.c_int),
        ("nt_a", ctypes.c_int), ("nt_b", ctypes.c_int),
        ("lds_conflict_a", ctypes.c_int), ("lds_conflict_b", ctypes.c_int),
        ("run_bytes_a", ctypes.c_int), ("run_bytes_b", ctypes.c_int), ("seg_bytes_a", ctypes.c_int),
        ("seg_bytes_b", ctypes.c_int), ("align_a", ctypes.c_int), ("align_b", ctypes.c_int),
        ("num_tiles", ctypes.c_int64), ("elements", ctypes.c_int64), ("bytes_moved", ctypes.c_int64),
        ("span_a", ctypes.c_int64), ("span_b", ctypes.c_int64),
        ("stride_a", ctypes.c_int64 * TTC_MAX_DIM), ("stride_b", ctypes.c_int64 * TTC_MAX_DIM),
        ("candidate_index", ctypes.c_int), ("candidate_count", ctypes.c_int), ("tuned_ms", ctypes.c_float), ("heuristic_cost", ctypes.c_double),
        ("unroll", ctypes.c_int), ("merged", ctypes.c_int),
    ]

    def as_dict(self) -> dict:
        n = self.ndim
        out = {}
        for name, _ in self._fields_:
            v = getattr(self, name)
            if name.startswith("digit_"):
                out[name] = list(v)[:(self.digits_a if name.endswith("_a") else self.digits_b)]
            else:
                out[name] = list(v)[:n] if hasattr(v, "__len__") else v
        return out


class TtcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {ttc_status_string(status)} (status {status})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load libttc.so (built by paper_1603_02297_amd.build).  No fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_1603_02297_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i, i64p, ip = ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int)
        L.ttc_plan_create.restype = vp
        L.ttc_plan_create.argtypes = [i, i, i64p, ip, vp, vp]
        L.ttc_plan_create_ex.restype = vp
        L.ttc_plan_create_ex.argtypes = [i, i, i64p, ip, i64p, i64p, vp, vp]
        L.ttc_execute.restype = i
        L.ttc_execute.argtypes = [vp, vp, vp, vp]
        L.ttc_plan_destroy.restype = i
        L.ttc_plan_destroy.argtypes = [vp]
        L.ttc_last_status.restype = i
        L.ttc_last_status.argtypes = []
        L.ttc_status_string.restype = ctypes.c_char_p
        L.ttc_status_string.argtypes = [i]
        L.ttc_plan_get_info.restype = i
        L.ttc_plan_get_info.argtypes = [vp, ctypes.POINTER(ttc_plan_info_t)]
        L.ttc_plan_candidate_count.restype = i
        L.ttc_plan_candidate_count.argtypes = [vp]
        L.ttc_plan_select_candidate.restype = i
        L.ttc_plan_select_candidate.argtypes = [vp, i]
        L.ttc_plan_tune.restype = i
        L.ttc_plan_tune.argtypes = [vp, vp, vp, vp, i]
        pvp = ctypes.POINTER(ctypes.c_void_p)
        L.ttc_plan_tune_pairs.restype = i
        L.ttc_plan_tune_pairs.argtypes = [vp, i, pvp, pvp, vp, i]
        L.ttc_time_execute.restype = i
        L.ttc_time_execute.argtypes = [vp, i, pvp, pvp, vp, i, i, ctypes.POINTER(ctypes.c_float)]
        L.ttc_time_ceiling.restype = i
        L.ttc_time_ceiling.argtypes = [i, ctypes.c_int64, i, pvp, pvp, vp, i, i, ctypes.POINTER(ctypes.c_float)]
        L.ttc_plan_set_streaming.restype = i
        L.ttc_plan_set_streaming.argtypes = [vp, i, i]
        L.ttc_plan_set_tile_mapping.restype = i
        L.ttc_plan_set_tile_mapping.argtypes = [vp, i]
        L.ttc_plan_cache_store.restype = i
        L.ttc_plan_cache_store.argtypes = [vp, ctypes.c_char_p]
        L.ttc_plan_cache_lookup.restype = i
        L.ttc_plan_cache_lookup.argtypes = [vp, ctypes.c_char_p]
        L.ttc_debug_emulate_map.restype = i
        L.ttc_debug_emulate_map.argtypes = [vp, i64p]
        _lib = L
    return _lib


def _scalar(dtype: int, value):
    """Host scalar of `dtype` as a ctypes object, or None for the library default."""
    if value is None:
        return None
    if dtype == TTC_F32:
        return ctypes.c_float(float(value))
    if dtype in (TTC_F64, TTC_F32_F64, TTC_F64_F32):
        return ctypes.c_double(float(value))
    z = complex(value)
    if dtype == TTC_C64:
        return (ctypes.c_float * 2)(z.real, z.imag)
    return (ctypes.c_double * 2)(z.real, z.imag)


def _ref(obj):
    return None if obj is None else ctypes.cast(ctypes.byref(obj), ctypes.c_void_p)


def ttc_status_string(status: int) -> str:
    return lib().ttc_status_string(int(status)).decode()


def ttc_last_status() -> int:
    return lib().ttc_last_status()


def ttc_plan_create(dtype: int, ndim: int, sizes: Sequence[int], perm: Sequence[int],
                    alpha=None, beta=None) -> int:
    """Returns the plan handle (an integer address).  Raises TtcError when the library refuses."""
    c_sizes = (ctypes.c_int64 * max(len(sizes), 1))(*[int(s) for s in sizes])
    c_perm = (ctypes.c_int * max(len(perm), 1))(*[int(p) for p in perm])
    a, b = _scalar(dtype, alpha), _scalar(dtype, beta)
    h = lib().ttc_plan_create(int(dtype), int(ndim), c_sizes, c_perm, _ref(a), _ref(b))
    if not h:
        raise TtcError(ttc_last_status(), "ttc_plan_create")
    return h


def ttc_plan_create_ex(dtype: int, ndim: int, sizes: Sequence[int], perm: Sequence[int],
                       lda: Optional[Sequence[int]] = None, ldb: Optional[Sequence[int]] = None,
                       alpha=None, beta=None) -> int:
    """Plan for sub-tensors (leading dimensions per index of A / of B) and for every data type."""
    c_sizes = (ctypes.c_int64 * max(len(sizes), 1))(*[int(s) for s in sizes])
    c_perm = (ctypes.c_int * max(len(perm), 1))(*[int(p) for p in perm])
    c_lda = None if lda is None else (ctypes.c_int64 * max(len(lda), 1))(*[int(x) for x in lda])
    c_ldb = None if ldb is None else (ctypes.c_int64 * max(len(ldb), 1))(*[int(x) for x in ldb])
    a, b = _scalar(dtype, alpha), _scalar(dtype, beta)
    h = lib().ttc_plan_create_ex(int(dtype), int(ndim), c_sizes, c_perm, c_lda, c_ldb, _ref(a), _ref(b))
    if not h:
        raise TtcError(ttc_last_status(), "ttc_plan_create_ex")
    return h


def ttc_execute(plan: int, A: int, B: int, stream: Optional[int] = None) -> None:
    """A, B: device addresses (tensor.data_ptr()); stream: hipStream_t as an integer or None."""
    st = lib().ttc_execute(plan, A, B, stream or None)
    if st != TTC_OK:
        raise TtcError(st, "ttc_execute")


def ttc_plan_destroy(plan: Optional[int]) -> None:
    lib().ttc_plan_destroy(plan)


def ttc_plan_get_info(plan: int) -> dict:
    info = ttc_plan_info_t()
    st = lib().ttc_plan_get_info(plan, ctypes.byref(info))
    if st != TTC_OK:
        raise TtcError(st, "ttc_plan_get_info")
    return info.as_dict()


def ttc_plan_candidate_count(plan: int) -> int:
    n = lib().ttc_plan_candidate_count(plan)
    if n < 0:
        raise TtcError(-n, "ttc_plan_candidate_count")
    return n


def ttc_plan_select_candidate(plan: int, index: int) -> None:
    st = lib().ttc_plan_select_candidate(plan, int(index))
    if st != TTC_OK:
        raise TtcError(st, "ttc_plan_select_candidate")


def ttc_plan_tune(plan: int, A: int, B: int, stream: Optional[int] = None, max_candidates: int = 0) -> None:
    st = lib().ttc_plan_tune(plan, A, B, stream or None, int(max_candidates))
    if st != TTC_OK:
        raise TtcError(st, "ttc_plan_tune")


def ttc_plan_tune_pairs(plan: int, A_list: Sequence[int], B_list: Sequence[int], stream: Optional[int] = None,
                        max_candidates: int = 0) -> None:
    st = lib().ttc_plan_tune_pairs(plan, len(A_list), _ptr_array(A_list), _ptr_array(B_list), stream or None,
                                   int(max_candidates))
    if st != TTC_OK:
        raise TtcError(st, "ttc_plan_tune_pairs")


def _ptr_array(ptrs: Sequence[int]):
    return (ctypes.c_void_p * len(ptrs))(*[int(p) for p in ptrs])


def ttc_time_execute(plan: int, A_list: Sequence[int], B_list: Sequence[int], stream: Optional[int] = None,
                     warmup: int = 2, iters: int = 10) -> float:
    """Mean milliseconds per launch over `iters` launches, buffer pairs rotating."""
    ms = ctypes.c_float(0)
    st = lib().ttc_time_execute(plan, len(A_list), _ptr_array(A_list), _ptr_array(B_list), stream or None,
                                int(warmup), int(iters), ctypes.byref(ms))
    if st != TTC_OK:
        raise TtcError(st, "ttc_time_execute")
    return ms.value


def ttc_time_ceiling(kind: int, nbytes: int, src_list: Sequence[int], dst_list: Sequence[int],
                     stream: Optional[int] = None, warmup: int = 2, iters: int = 10) -> float:
    ms = ctypes.c_float(0)
    st = lib().ttc_time_ceiling(int(kind), int(nbytes), len(src_list), _ptr_array(src_list), _ptr_array(dst_list),
                                stream or None, int(warmup), int(iters), ctypes.byref(ms))
    if st != TTC_OK:
        raise TtcError(st, "ttc_time_ceiling")
    return ms.value


def ttc_plan_set_tile_mapping(plan: int, mode: int = -1) -> None:
    """How the selected candidate deals its tiles to the XCDs: 0 round robin, 1 one range each, 2..10 chunks of 2**mode, -1 default."""
    st = lib().ttc_plan_set_tile_mapping(plan, int(mode))
    if st != TTC_OK:
        raise TtcError(st, "ttc_plan_set_tile_mapping")


def ttc_plan_set_streaming(plan: int, stream_a: int = -1, stream_b: int = -1) -> None:
    """Non-temporal accesses of the selected candidate: 1 on, 0 off, -1 the planner's rule."""
    st = lib().ttc_plan_set_streaming(plan, int(stream_a), int(stream_b))
    if st != TTC_OK:
        raise TtcError(st, "ttc_plan_set_streaming")


def ttc_plan_cache_store(plan: int, path: str) -> None:
    st = lib().ttc_plan_cache_store(plan, os.fsencode(path))
    if st != TTC_OK:
        raise TtcError(st, "ttc_plan_cache_store")


def ttc_plan_cache_lookup(plan: int, path: str) -> bool:
    """True if the store held a usable entry (now selected), False if it did not."""
    st = lib().ttc_plan_cache_lookup(plan, os.fsencode(path))
    if st == TTC_OK:
        return True
    if st == TTC_ERR_NOT_FOUND:
        return False
    raise TtcError(st, "ttc_plan_cache_lookup")


def ttc_debug_emulate_map(plan: int, elements: Optional[int] = None):
    """Host replay of the selected candidate: array b_from_a of span_b entries (see ttc.h)."""
    span = ttc_plan_get_info(plan)["span_b"]
    if elements is not None and int(elements) < span:
        raise ValueError("b_from_a needs span_b entries")
    buf = (ctypes.c_int64 * max(int(span), 1))()
    st = lib().ttc_debug_emulate_map(plan, buf)
    if st != TTC_OK:
        raise TtcError(st, "ttc_debug_emulate_map")
    return buf
