"""Host-side checks of the study helpers (no GPU): the benchmark's permutations and shapes, the rule by which the
search fills its places (mirrored from the library), and the feature functions the ranking models are fitted with."""
import numpy as np
import pytest

import paper_1603_02297_amd as ttc
from paper_1603_02297_amd import studies as st


def test_benchmark_has_57_cases_without_mergeable_indices():
    perms = st.benchmark_permutations()
    assert len(perms) == 19 and len(perms) * 3 == 57
    for perm, cls in perms:
        assert sorted(perm) == list(range(len(perm)))
        assert not st.mergeable(perm)
        assert cls in ("stride-1", "inverse", "general")
        assert (perm[0] == 0) == (cls == "stride-1")
    for n in range(2, 7):
        for cfg in (0, 1, 2):
            sizes = st.shape_for(n, cfg)
            assert len(sizes) == n and 150e6 < 4 * np.prod(sizes) < 260e6


def test_search_set_keeps_places_for_both_micro_tile_families():
    fam = [0] * 300
    for i in (5, 150, 210):
        fam[i] = 1
    for i in (220, 230, 280):
        fam[i] = 2
    assert st.search_set(fam, 1) == [0]
    assert st.search_set(fam, 10) == [0, 1, 2, 3, 4, 5, 6, 150, 220, 230]      # two places per family, candidate 5 was in anyway
    chosen = st.search_set(fam, 100)
    assert len(set(chosen)) == 100 and {150, 210, 220, 230, 280} <= set(chosen)
    assert st.search_set(fam, 400) == list(range(300))


def test_micro_tile_features_mirror_the_library_model():
    """micro_cost() of the library = exp(offset + sum of the fitted weights times these features)."""
    weights = {"A<128": 0.05, "B<128": 0.012, "A>1K": -0.01, "B>1K": -0.03, "pad": 0.11, "unA*A<512": 0.028,
               "unB*B<512": 0.072, "t128": 0.04, "t64": 0.068, "ordNotB": 0.054, "blocks": 0.009, "lds": 0.114,
               "mergeA": 0.006, "mergeB": 0.011, "idle": 0.27}
    p = ttc.ttc_plan_create(ttc.TTC_F32, 5, (512, 20, 9, 22, 768), (4, 3, 2, 1, 0), 1.0, 0.0)   # large enough that no small-problem term applies
    seen = 0
    for k in range(ttc.ttc_plan_candidate_count(p)):
        ttc.ttc_plan_select_candidate(p, k)
        info = ttc.ttc_plan_get_info(p)
        if info["kernel_class"] != ttc.TTC_KERNEL_MICRO:
            continue
        seen += 1
        assert st.micro_family(info) == (2 if info["merged"] else 1)
        f = st.fit_micro_features(info)
        model = np.exp(-0.22 + sum(weights[q] * v for q, v in f.items() if q in weights))
        assert model == pytest.approx(info["heuristic_cost"], rel=1e-12), (k, info["tile"], f)
    assert seen >= 20
    ttc.ttc_plan_destroy(p)
