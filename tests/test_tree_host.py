"""Draft-stage tree bookkeeping (host C++ in the library) against the path-based oracle and against the properties the
paper states for it (Sec. III-B, III-C, III-D).  CPU only."""
import time

import numpy as np
import pytest

from oracle import oracle, tree_oracle
from paper_2507_02620_amd import synth


def _fs():
    from paper_2507_02620_amd import flowspec as fs
    return fs


def _random_base(n, vocab, seed, depth=8, branch=4):
    """A base tree in generation order (not score order) with per-node confidences."""
    rng = np.random.default_rng(seed)
    parent = np.full(n, -1, dtype=np.int32)
    dep = np.zeros(n, dtype=np.int32)
    nch = np.zeros(n, dtype=np.int32)
    for i in range(1, n):
        ok = [j for j in range(i) if dep[j] < depth and nch[j] < branch] or [0]
        parent[i] = ok[int(rng.integers(0, len(ok)))]
        dep[i] = dep[parent[i]] + 1
        nch[parent[i]] += 1
    token = np.zeros(n, dtype=np.int32)
    used = {}
    for i in range(n):
        s = used.setdefault(int(parent[i]), set())
        t = int(rng.integers(0, vocab))
        while t in s and len(s) < vocab:
            t = int(rng.integers(0, vocab))
        s.add(t)
        token[i] = t
    conf = rng.random(n).astype(np.float32)
    conf[0] = 1.0
    return parent, token, conf


# ---- oracle pins ----------------------------------------------------------------------------------------------------

def test_oracle_cumulative_score_is_the_path_product_and_parents_outrank_children():
    parent, token, conf = _random_base(200, 50, 0)
    cu = tree_oracle.cumulative_scores(parent, conf)
    # closed form on a chain: product of the first k confidences
    chain = np.arange(-1, 9, dtype=np.int32)
    c = np.array([1, .5, .5, .25, 1, .5, 2 ** -3, .5, .5, .5], dtype=np.float32)
    assert tree_oracle.cumulative_scores(chain, c) == [float(np.prod(c[1:k + 1])) for k in range(10)]
    for i in range(1, 200):
        assert cu[i] <= cu[parent[i]]                      # Sec. III-B: a node outranks its children
    par, tok, sc, order = tree_oracle.segment(parent, token, conf, 80)
    assert all(par[j] < j for j in range(1, 80)) and par[0] == -1   # selected nodes form a connected tree, S is topological
    assert all(sc[j] >= sc[j + 1] for j in range(79))
    assert min(sc) >= max(cu[b] for b in range(200) if b not in set(order))  # they are the top-L0


def test_oracle_merge_is_the_union_of_paths():
    pp, tp, _ = _random_base(30, 4, 1, depth=5)
    pn, tn, _ = _random_base(40, 4, 2, depth=6)
    tn[0] = tp[0]
    par, tok, app, mp = tree_oracle.merge(pp, tp, pn, tn)
    paths = lambda p, t: {tree_oracle.path_tokens(p, t, i) for i in range(len(p))}
    assert paths(par, tok) == paths(pp, tp) | paths(pn, tn)                 # N_new = paths of T_new not in P_pr
    assert par[:30] == pp.tolist() and tok[:30] == tp.tolist()              # S_pr untouched, S_app appended behind it
    new_paths = [tree_oracle.path_tokens(par, tok, i) for i in range(30, len(par))]
    assert len(set(new_paths)) == len(new_paths) and not (set(new_paths) & paths(pp, tp))
    assert app == sorted(app)                                               # S_app keeps T_new's (score) order
    assert all(par[i] < i for i in range(1, len(par)))


# ---- library vs oracle ----------------------------------------------------------------------------------------------

@pytest.mark.parametrize("seed", range(8))
def test_segment_matches_oracle(seed):
    fs = _fs()
    rng = np.random.default_rng(seed)
    n = int(rng.choice([1, 2, 17, 80, 300, 1000]))
    L0 = int(rng.choice([1, 16, 80, 2000]))
    parent, token, conf = _random_base(n, 100, seed)
    if seed % 2:
        conf[rng.integers(1, max(n, 2), size=max(n // 5, 1)) % n] = 1.0      # exact ties between parent and child
        conf[0] = 1.0
    par, tok, sc, bi = fs.tree_segment(parent, token, conf, L0)
    o_par, o_tok, o_sc, o_order = tree_oracle.segment(parent, token, conf, L0)
    assert par.tolist() == o_par and tok.tolist() == o_tok and bi.tolist() == o_order
    assert sc.tolist() == o_sc                                               # same products in the same order: bit-exact


def test_segment_reproduces_the_generator_and_the_paper_sizes():
    """L0 = 80, L_max = 16 (the paper's setting): 5 segments; the result is what synth.random_tree builds the same way."""
    fs = _fs()
    parent, token, conf = _random_base(400, 32000, 3)
    par, tok, sc, bi = fs.tree_segment(parent, token, conf, 80)
    assert len(par) == 80 and len(synth.segments(80, 16)) == 5
    anc, depth = oracle.tree_ancestors(par)                                  # valid input for the verification stage
    assert depth.max() >= 2


@pytest.mark.parametrize("seed", range(10))
def test_prune_and_merge_match_oracle(seed):
    fs = _fs()
    rng = np.random.default_rng(100 + seed)
    vocab = int(rng.choice([3, 6, 50]))
    tree = synth.random_tree(int(rng.integers(2, 90)), 6, 3, vocab, seed)
    n_ver = int(rng.integers(1, tree.size + 1))
    amax = rng.integers(0, vocab, n_ver).astype(np.int32)
    for r, t in synth.resolve_plants(synth.plant_path(tree, n_ver, seed, 0, 0.0, 2.0), tree, vocab):
        amax[r] = t
    res, retain = oracle.accept(amax, tree.token, tree.parent, n_ver)
    ppr, tpr = fs.tree_prune(tree.parent, tree.token, retain, res.n_acc)
    o_ppr, o_tpr = oracle.tree_remap(tree.parent, tree.token, retain, res.n_acc)
    assert ppr.tolist() == o_ppr.tolist() and tpr.tolist() == o_tpr.tolist()
    # a new tree drafted from the new context, same root token (or any root when the round ended)
    new = synth.random_tree(int(rng.integers(1, 70)), 7, 3, vocab, seed, stream=5)
    tnew = new.token.copy()
    if len(tpr):
        tnew[0] = tpr[0]
    for limit in (-1, 0, 5):
        par, tok, app, mp = fs.tree_merge(ppr, tpr, new.parent, tnew, limit=limit)
        o = tree_oracle.merge(ppr, tpr, new.parent, tnew, limit)
        assert par.tolist() == o[0] and tok.tolist() == o[1] and app.tolist() == o[2] and mp.tolist() == o[3]
        assert limit < 0 or len(app) <= limit
        assert len(par) == 0 or (par[0] == -1 and all(par[i] < i for i in range(1, len(par))))


def test_error_codes():
    fs = _fs()
    with pytest.raises(fs.FlowSpecError) as e:
        fs.tree_segment([-1, 2, 0], [1, 2, 3], [1, .5, .5], 3)
    assert e.value.code == fs.FS_ETOPO
    with pytest.raises(fs.FlowSpecError) as e:
        fs.tree_merge([-1, 0], [7, 1], [-1, 0], [8, 1])                     # root tokens differ
    assert e.value.code == fs.FS_EINVAL
    with pytest.raises(fs.FlowSpecError) as e:
        fs.tree_merge([-1, 0], [7, 1], [-1, 0, 1], [7, 2, 3], max_out=3)
    assert e.value.code == fs.FS_ECAP
    with pytest.raises(fs.FlowSpecError) as e:
        fs.tree_prune([-1, 0, 0], [1, 2, 3], [2, 1], 0)
    assert e.value.code == fs.FS_EINVAL


def test_timing_at_the_papers_tree_sizes(capsys):
    """Prints the host cost per call at L0 = 80 / L_exp = 64 so that it can be quoted beside the GPU numbers (no time limit
    is asserted: the box may be busy)."""
    fs = _fs()
    parent, token, conf = _random_base(400, 32000, 9)
    t0 = time.perf_counter()
    for _ in range(200):
        par, tok, sc, bi = fs.tree_segment(parent, token, conf, 80)
    t_seg = (time.perf_counter() - t0) / 200
    new = synth.random_tree(64, 5, 4, 32000, 9)
    tnew = new.token.copy(); tnew[0] = tok[0]
    t0 = time.perf_counter()
    for _ in range(200):
        fs.tree_merge(par, tok, new.parent, tnew)
    t_mrg = (time.perf_counter() - t0) / 200
    print(f"fs_tree_segment(400 -> 80): {t_seg * 1e6:.1f} us; fs_tree_merge(80 + 64): {t_mrg * 1e6:.1f} us (incl. ctypes marshalling)")
    assert t_seg > 0 and t_mrg > 0
