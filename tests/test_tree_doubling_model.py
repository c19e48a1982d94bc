"""Host model of the pointer-doubling recurrence the HIP path uses for trees deeper than 32 levels (Sec. III-A: tree
position IDs and attention mask of a segment): A'[i] = A[i] | A[J[i]], D'[i] = D[i] + D[J[i]], J'[i] = J[J[i]], every
round reading the previous round's arrays only.  Checked against the oracle's ancestor sets and against a plain walk.
Also pins the deep-tree generator (deep, not a chain, topological).  CPU only."""
import numpy as np
import pytest

from oracle import oracle
from paper_2507_02620_amd import synth
from tests.helpers import ancestors_by_walking


def doubling(parent):
    T = len(parent)
    A = np.eye(T, dtype=bool)
    J = np.asarray(parent, dtype=np.int64).copy()
    D = (J >= 0).astype(np.int64)
    span = 1
    while span < T:
        live = J >= 0
        Jc = np.where(live, J, 0)
        A2 = A | (A[Jc] & live[:, None])
        D2 = D + np.where(live, D[Jc], 0)
        J2 = np.where(live, J[Jc], -1)
        A, D, J = A2, D2, J2
        span <<= 1
    assert (J < 0).all()
    return A, D


@pytest.mark.parametrize("spine", [1, 40, 200, 900, 1024])
def test_doubling_equals_ancestor_closure(spine):
    tree = synth.spine_tree(1024, spine, 32000, 3)
    assert (tree.parent[1:] < np.arange(1, 1024)).all() and tree.parent[0] == -1
    A, D = doubling(tree.parent)
    assert (A == ancestors_by_walking(tree.parent)).all()
    anc, depth = oracle.tree_ancestors(tree.parent)
    bits = (anc[:, :, None] >> np.arange(64, dtype=np.uint64)[None, None, :]) & np.uint64(1)
    assert (bits.reshape(1024, -1)[:, :1024].astype(bool) == A).all()
    assert (D == depth).all() and (D == tree.depth).all()


def test_spine_trees_are_deep_and_not_chains():
    for spine in (40, 200, 900):
        tree = synth.spine_tree(1024, spine, 32000, 3)
        assert tree.depth.max() >= spine - 1 and tree.depth.max() > 32
        assert not all(tree.parent[i] == i - 1 for i in range(tree.size))
        assert (np.diff(tree.score) <= 0).all()          # descending cumulative score (Eq. 1)
