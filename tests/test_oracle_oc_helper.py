"""Pins for the Algorithm 3 oracle (object-condensation index matrices), no GPU: a numpy
re-statement on small inputs, a hand-worked case, and set / order invariants."""
import numpy as np
import pytest

import oracle
from paper_2511_10442_amd import workloads as W


def numpy_oc_helper(asso, unique_idx, unique_rs, rs, n_maxuq, n_maxrs, rot_block):
    n_unique = len(unique_idx)
    M = np.full((n_maxuq, n_unique), -1, dtype=np.int32)
    Mn = np.full((n_maxrs, n_unique), -1, dtype=np.int32)
    for k in range(n_unique):
        start, end = int(rs[unique_rs[k]]), int(rs[unique_rs[k] + 1])
        end = min(end, len(asso), start + n_maxrs)
        window = np.arange(start, end)
        tid = k % rot_block
        if 0 < tid < len(window):
            window = np.roll(window, -tid)                 # start tid vertices in, wrap round
        member = asso[window] == unique_idx[k]
        mem = window[member][:n_maxuq]
        non = window[~member][:n_maxrs]
        M[:len(mem), k] = mem
        Mn[:len(non), k] = non
    return M, Mn


@pytest.mark.parametrize("rot_block", [1, 4, 256])
@pytest.mark.parametrize("sizes,objs", [([50], 5), ([0, 33, 7, 120], 6), ([300, 1, 2], 40)])
def test_matches_numpy_restatement(sizes, objs, rot_block):
    asso, uq, uqrs, rs, n_maxuq, n_maxrs = W.oc_association(sizes, objs, 0.2, seed=len(sizes) + objs)
    for cap_uq, cap_rs in [(n_maxuq, n_maxrs), (max(1, n_maxuq // 2), n_maxrs), (n_maxuq + 3, max(1, n_maxrs // 3))]:
        M, Mn = oracle.oc_helper(asso, uq, uqrs, rs, cap_uq, cap_rs, True, rot_block)
        M2, Mn2 = numpy_oc_helper(asso, uq, uqrs, rs, cap_uq, cap_rs, rot_block)
        assert np.array_equal(M, M2) and np.array_equal(Mn, Mn2)
    M3, none = oracle.oc_helper(asso, uq, uqrs, rs, n_maxuq, n_maxrs, False, rot_block)
    assert none is None and np.array_equal(M3, numpy_oc_helper(asso, uq, uqrs, rs, n_maxuq, n_maxrs, rot_block)[0])


def test_by_hand():
    # split 0 = vertices 0..4, split 1 = vertices 5..7; objects: vertex 1 (split 0), vertex 3 (split 0), vertex 6 (split 1)
    asso = np.array([1, 1, 3, 3, -1, 6, 6, -1], dtype=np.int32)
    uq = np.array([1, 3, 6], dtype=np.int32)
    uqrs = np.array([0, 0, 1], dtype=np.int32)
    rs = np.array([0, 5, 8], dtype=np.int32)
    M, Mn = oracle.oc_helper(asso, uq, uqrs, rs, 3, 5, True, 1)
    assert M.T.tolist() == [[0, 1, -1], [2, 3, -1], [5, 6, -1]]
    assert Mn.T.tolist() == [[2, 3, 4, -1, -1], [0, 1, 4, -1, -1], [7, -1, -1, -1, -1]]
    # with a rotation block of 4 object k starts k vertices into its window and wraps round:
    #   k=1 walks 1,2,3,4,0: members 2,3, non-members 1,4,0;  k=2 walks 7,5,6: members 5,6, non-member 7
    M, Mn = oracle.oc_helper(asso, uq, uqrs, rs, 3, 5, True, 4)
    assert M.T.tolist() == [[0, 1, -1], [2, 3, -1], [5, 6, -1]]
    assert Mn.T.tolist() == [[2, 3, 4, -1, -1], [1, 4, 0, -1, -1], [7, -1, -1, -1, -1]]
    # capacity 1 keeps the first member of the walk; for an object whose walk starts past a member that is a later vertex
    asso2 = np.array([1, 1, 1, 1, 1], dtype=np.int32)
    M, _ = oracle.oc_helper(asso2, np.array([1, 1, 1], dtype=np.int32), np.zeros(3, dtype=np.int32),
                            np.array([0, 5], dtype=np.int32), 2, 5, False, 8)
    assert M.T.tolist() == [[0, 1], [1, 2], [2, 3]]


def test_invariants_at_size():
    sizes = [4000, 2500, 0, 6000]
    asso, uq, uqrs, rs, n_maxuq, n_maxrs = W.oc_association(sizes, 60, 0.15, seed=9)
    M, Mn = oracle.oc_helper(asso, uq, uqrs, rs, n_maxuq, n_maxrs, True, 256)
    for k in range(len(uq)):
        b, e = int(rs[uqrs[k]]), int(rs[uqrs[k] + 1])
        mem = M[:, k][M[:, k] >= 0]
        non = Mn[:, k][Mn[:, k] >= 0]
        assert set(mem.tolist()) == set((np.nonzero(asso[b:e] == uq[k])[0] + b).tolist())      # exactly the members
        assert len(mem) + len(non) == e - b and not set(mem.tolist()) & set(non.tolist())       # a partition of the split
        assert np.all(M[len(mem):, k] == -1) and np.all(Mn[len(non):, k] == -1)                 # padded after the entries
        both = np.concatenate([mem, non])
        assert np.sum(np.diff(np.sort(both)) != 1) == 0                                         # every vertex once
        for arr in (mem, non):                                                                  # a rotation of ascending order
            assert np.sum(np.diff(arr) < 0) <= 1
