"""Pins for acceptance, continuous condition, retain set, remap (Sec. III-C).  CPU only."""
import itertools
import os

import numpy as np
import pytest

from oracle import oracle
from paper_2507_02620_amd import synth
from tests.textbook import path_to

GOLD = os.path.join(os.path.dirname(__file__), "golden", "fig3_pruning.txt")


def read_fig3():
    vals = {}
    for line in open(GOLD):
        if line.startswith("#") or "=" not in line:
            continue
        k, v = line.split("=")
        vals[k.strip()] = [int(t) for t in v.split()]
    return vals


def test_pruning_figure_index_sets():
    g = read_fig3()
    parent = np.array(g["parent"], dtype=np.int32)
    token = np.array([10, 11, 12, 13, 14, 15, 16, 17], dtype=np.int32)
    n_ver = 3                                   # nodes 0..2 verified so far
    amax = np.array([11, 13, 99], dtype=np.int32)  # root predicts node 1's token, node 1 predicts node 3's token
    res, retain = oracle.accept(amax, token, parent, n_ver)
    assert retain[: res.n_acc].tolist() == g["I_acc"]
    assert retain[res.n_acc:].tolist() == g["I_draft"]
    assert res.as_tuple() == (2, 13, 3, 1, 5, 0)
    npar, ntok = oracle.tree_remap(parent, token, retain, res.n_acc)
    assert npar.tolist() == [-1, 0, 0] and ntok.tolist() == [13, 16, 17]
    # mask pruning rule of the caption: keep entries whose row and column are both in I_draft
    anc, _ = oracle.tree_ancestors(parent)
    full = np.array([[(int(anc[i, 0]) >> j) & 1 for j in range(8)] for i in range(8)])
    sub = full[np.ix_(g["I_draft"], g["I_draft"])]
    anc2, _ = oracle.tree_ancestors(npar)
    new = np.array([[(int(anc2[i, 0]) >> j) & 1 for j in range(3)] for i in range(3)])
    assert (sub == new).all()


def greedy_walk(amax, token, parent, n_ver):
    """Independent statement of greedy tree acceptance when sibling tokens are distinct: walk from the root."""
    T = len(parent)
    cur, acc = 0, [0]
    while True:
        nxt = [c for c in range(T) if parent[c] == cur and token[c] == amax[cur]]
        if not nxt:
            return acc, int(amax[cur]), -1
        c = nxt[0]
        if c >= n_ver:
            return acc, int(amax[cur]), c
        cur = c
        acc.append(c)


def brute_force(amax, token, parent, n_ver):
    """Enumerate every root-to-node path; a path is accepted iff every edge matches and every node is verified."""
    T = len(parent)
    best = [0]
    for i in range(n_ver):
        p = path_to(parent, i)
        if p[0] != 0 or any(q >= n_ver for q in p):
            continue
        if all(token[b] == amax[a] for a, b in zip(p[:-1], p[1:])) and len(p) > len(best):
            best = p
    return best


@pytest.mark.parametrize("seed", range(12))
def test_accept_equals_greedy_walk_and_brute_force(seed):
    rng = np.random.default_rng(seed)
    T = int(rng.integers(2, 40))
    vocab = 6
    tree = synth.random_tree(T, 6, 3, vocab, seed)
    n_ver = int(rng.integers(1, T + 1))
    # amax drawn from a tiny vocabulary so that matches are frequent
    amax = rng.integers(0, vocab, n_ver).astype(np.int32)
    res, retain = oracle.accept(amax, tree.token, tree.parent, n_ver)
    acc, x_new, n_new = greedy_walk(amax, tree.token, tree.parent, n_ver)
    assert retain[: res.n_acc].tolist() == acc == brute_force(amax, tree.token, tree.parent, n_ver)
    assert (res.x_new, res.n_new, res.continuous) == (x_new, n_new, int(n_new >= 0))
    # I_pr = n_new and all descendants, ascending
    if n_new >= 0:
        sub = [i for i in range(T) if n_new in path_to(tree.parent, i)]
        assert retain[res.n_acc:].tolist() == sub
        assert n_new >= n_ver and res.n_pr_verified == 0
    else:
        assert res.n_retain == res.n_acc
    assert (np.diff(retain) > 0).all()


def test_edge_cases():
    parent = np.array([-1, 0, 0, 1], dtype=np.int32)
    token = np.array([5, 6, 7, 8], dtype=np.int32)
    # nothing verified: no-op, everything retained, context not updated
    res, retain = oracle.accept([], token, parent, 0)
    assert res.as_tuple() == (0, -1, 0, 1, 4, 0) and retain.tolist() == [0, 1, 2, 3]
    # no child matches: only the root is accepted, round ends
    res, retain = oracle.accept([9, 9, 9, 9], token, parent, 4)
    assert res.as_tuple() == (1, 9, -1, 0, 1, 0) and retain.tolist() == [0]
    # full-depth acceptance of a verified chain; bonus token matches nothing
    res, retain = oracle.accept([6, 8, 0, 3], token, parent, 4)
    assert res.as_tuple() == (3, 3, -1, 0, 3, 0) and retain.tolist() == [0, 1, 3]
    # matching child not verified yet: continuous, n_new >= n_ver
    res, retain = oracle.accept([6, 8], token, parent, 2)
    assert res.as_tuple() == (2, 8, 3, 1, 3, 0) and retain.tolist() == [0, 1, 3]
    # a second root is never accepted nor retained
    parent2 = np.array([-1, -1, 1], dtype=np.int32)
    res, retain = oracle.accept([7, 7, 7], np.array([5, 7, 7], dtype=np.int32), parent2, 3)
    assert res.as_tuple() == (1, 7, -1, 0, 1, 0)
    # equal-depth duplicates (siblings with the same token): lowest S index wins
    parent3 = np.array([-1, 0, 0], dtype=np.int32)
    res, retain = oracle.accept([4, 1, 2], np.array([0, 4, 4], dtype=np.int32), parent3, 3)
    assert retain.tolist() == [0, 1] and res.x_new == 1
    with pytest.raises(oracle.OracleError):
        oracle.accept([1], token, np.array([-1, 2, 0, 0], dtype=np.int32), 1)


def test_l_glo_state_machine_over_many_steps():
    """l_glo grows by |S_acc| per step; retained draft keeps its order; verified nodes stay a prefix."""
    rng = np.random.default_rng(0)
    l_glo = 100
    tree = synth.random_tree(40, 6, 3, 50, 3)
    parent, token = tree.parent, tree.token
    n_ver = 0
    for step in range(30):
        T = len(parent)
        n_ver = min(T, n_ver + 8)
        amax = rng.integers(0, 50, n_ver).astype(np.int32)
        t = synth.Tree(parent, token, np.zeros(T), synth._depths(parent))
        for row, tok in synth.resolve_plants(synth.plant_path(t, n_ver, 0, step), t, 50):
            amax[row] = tok
        res, retain = oracle.accept(amax, token, parent, n_ver)
        assert res.n_acc >= 1
        l_glo += res.n_acc
        parent, token = oracle.tree_remap(parent, token, retain, res.n_acc)
        n_ver = res.n_pr_verified
        if len(parent) == 0:
            nt = synth.random_tree(40, 6, 3, 50, 3, stream=step + 1)
            parent, token, n_ver = nt.parent, nt.token, 0
        assert parent[0] == -1 and all(parent[i] < i for i in range(len(parent)))
    assert l_glo > 130
