"""The C-ABI library loads without a GPU and exports every function include/ttc.h and include/ttc_aux.h declare."""
import ctypes
import os
import re

import paper_1603_02297_amd as ttc
from paper_1603_02297_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ttc.h")).read() + open(os.path.join(ROOT, "include", "ttc_aux.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ttc_[a-z_0-9]+)\s*\(", text)))


def test_header_functions_are_exported():
    names = declared_functions()
    assert "ttc_plan_create" in names and "ttc_execute" in names and "ttc_plan_destroy" in names
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"libttc.so does not export {n}"


def test_binding_covers_the_header():
    assert sorted(binding.EXPORTS) == declared_functions()
    for n in binding.EXPORTS:
        assert callable(getattr(ttc, n))


def test_status_strings():
    assert ttc.ttc_status_string(0) == "ok"
    for st in range(1, 13):
        assert ttc.ttc_status_string(st) not in ("ok", "unknown status")
    assert ttc.ttc_status_string(99) == "unknown status"


def test_info_struct_layout_matches_header():
    # a field the C side fills last must come back intact: catches any drift between the
    # ctypes structure and ttc_plan_info_t
    p = ttc.ttc_plan_create(ttc.TTC_F32, 3, (6, 5, 4), (2, 0, 1), 1.0, 0.0)
    info = ttc.ttc_plan_get_info(p)
    assert info["elements"] == 120 and info["bytes_moved"] == 2 * 120 * 4
    assert info["candidate_count"] == 1 and info["candidate_index"] == 0      # only the heuristic's choice is laid out yet
    assert info["heuristic_cost"] > 0
    n = ttc.ttc_plan_candidate_count(p)                                        # builds the ranked list
    again = ttc.ttc_plan_get_info(p)
    assert n > 1 and again["candidate_count"] == n and again["candidate_index"] == 0
    assert {k: v for k, v in again.items() if k != "candidate_count"} == {k: v for k, v in info.items() if k != "candidate_count"}
    ttc.ttc_plan_destroy(p)
