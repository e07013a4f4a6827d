"""GPU parity of fg_oc_helper (Algorithm 3) against its CPU oracle: bit-exact index matrices."""
import numpy as np
import pytest
import torch

import oracle
from paper_2511_10442_amd import binding as B
from paper_2511_10442_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_gpu(asso, uq, uqrs, rs, n_maxuq, n_maxrs, calc, rot, workspace="auto"):
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    M, Mn = B.fg_oc_helper(t(asso), t(uq), t(uqrs), t(rs), n_maxuq, n_maxrs, calc, rot, workspace=workspace)
    torch.cuda.synchronize()
    return M.cpu().numpy(), None if Mn is None else Mn.cpu().numpy()


@pytest.mark.parametrize("rot", [1, 7, 64, 256])
@pytest.mark.parametrize("sizes,objs", [([50], 5), ([0, 333, 7, 1200, 1], 70), ([3000, 2000], 300)])
def test_matches_oracle(sizes, objs, rot):
    asso, uq, uqrs, rs, n_maxuq, n_maxrs = W.oc_association(sizes, objs, 0.2, seed=objs + len(sizes))
    for cap_uq, cap_rs, calc in [(n_maxuq, n_maxrs, True), (max(1, n_maxuq // 3), n_maxrs, True),
                                 (n_maxuq + 5, max(1, n_maxrs // 2), True), (n_maxuq, n_maxrs, False)]:
        oM, oMn = oracle.oc_helper(asso, uq, uqrs, rs, cap_uq, cap_rs, calc, rot)
        for ws in ("auto", None):            # chunked kernels, then the single-kernel form
            M, Mn = run_gpu(asso, uq, uqrs, rs, cap_uq, cap_rs, calc, rot, ws)
            assert np.array_equal(M, oM)
            assert (Mn is None and oMn is None) or np.array_equal(Mn, oMn)


def test_detector_sized_batch():
    """10 row splits of 100,000 hits with 200 object candidates each (the shape of configuration 3)."""
    sizes = [100_000] * 10
    asso, uq, uqrs, rs, n_maxuq, n_maxrs = W.oc_association(sizes, 200, 0.1, seed=33)
    M, Mn = run_gpu(asso, uq, uqrs, rs, n_maxuq, n_maxrs, True, 256)
    oM, oMn = oracle.oc_helper(asso, uq, uqrs, rs, n_maxuq, n_maxrs, True, 256)
    assert np.array_equal(M, oM) and np.array_equal(Mn, oMn)
