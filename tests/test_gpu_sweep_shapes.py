"""The shapes of the 57-case benchmark study (paper_1603_02297_amd/studies.py sweep, built by the rules of
the paper's Section 4.1) against the CPU oracle, at the size the study times them: the study itself only
times, and this is where its results are checked.  Values are drawn on the host from fixed seeds."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
import paper_1603_02297_amd as ttc
from paper_1603_02297_amd import studies
from paper_1603_02297_amd import workloads as wl

pytestmark = pytest.mark.gpu

PERMS = studies.benchmark_permutations()
# every permutation on the equal-extent shape; the class representatives of each dimension also on the two
# shapes whose extents grow or shrink by a factor of 6
CASES = [(perm, cls, 0) for perm, cls in PERMS]
for _n in (3, 6):
    for _cls in ("inverse", "stride-1", "general"):
        _perm = next(p for p, c in PERMS if len(p) == _n and c == _cls)
        CASES += [(_perm, _cls, 1), (_perm, _cls, 2)]


def run(sizes, perm, A, B0, tune):
    dev = torch.device("cuda:0")
    dA, dB = torch.from_numpy(A).to(dev), torch.from_numpy(B0).to(dev)
    stream = torch.cuda.current_stream().cuda_stream
    plan = ttc.ttc_plan_create(wl.F32, len(sizes), sizes, perm, 1.0, 0.0)
    try:
        if tune:
            scratch = torch.empty_like(dB)
            ttc.ttc_plan_tune(plan, dA.data_ptr(), scratch.data_ptr(), stream, 40)
        ttc.ttc_execute(plan, dA.data_ptr(), dB.data_ptr(), stream)
        torch.cuda.synchronize()
        info = ttc.ttc_plan_get_info(plan)
    finally:
        ttc.ttc_plan_destroy(plan)
    return dB.cpu().numpy(), info


@pytest.mark.parametrize("perm,cls,cfg", CASES, ids=[f"{len(p)}d-{c}-cfg{g}-p{''.join(map(str, p))}" for p, c, g in CASES])
def test_sweep_shape_matches_the_oracle(perm, cls, cfg):
    sizes = studies.shape_for(len(perm), cfg)
    n = int(np.prod(sizes))
    A = wl.uniform_tensor(wl.F32, n, 5700 + 10 * len(perm) + cfg)
    B0 = wl.uniform_tensor(wl.F32, n, 5800 + 10 * len(perm) + cfg)
    want = oracle.transpose(wl.F32, sizes, perm, 1.0, 0.0, A, B0.copy(), 16)
    got, info = run(sizes, perm, A, B0, tune=False)
    assert np.array_equal(got, want), (sizes, perm, "heuristic", info)
    if cfg == 0 and cls != "general":            # the searched plan too, for the representatives
        got, info = run(sizes, perm, A, B0, tune=True)
        assert np.array_equal(got, want), (sizes, perm, "searched", info)
