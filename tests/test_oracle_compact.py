"""Pins for KV-cache pruning (I_incache), segment pruning (I_local) and continuity after a prune.  CPU only."""
import numpy as np
import pytest

from oracle import oracle
from paper_2507_02620_amd import synth
from tests.helpers import TINY, make_oracle_stage, verify_whole_tree


def test_incache_and_local_sets_by_hand():
    # retain (S indices) = {0,1,3,6,7}, l_glo = 10; the stage has cached 5 draft tokens (l_cache = 15) and
    # holds an in-flight segment of S indices 5..7 (l_s = 3).
    # Global positions: I_retain + l_glo = {10,11,13,16,17}; I_incache = those < 15 = {10,11,13};
    # I_local = {i - l_cache : l_cache <= i < l_cache + l_s} = {16-15, 17-15} = {1, 2}.
    retain = np.array([0, 1, 3, 6, 7], dtype=np.int32)
    cache = np.arange(1 * 2 * 1 * 20 * 2, dtype=np.float32).reshape(1, 2, 1, 20, 2)
    before = cache.copy()
    lg, lc = oracle.kv_compact(cache, 10, 15, retain, 2)
    assert (lg, lc) == (12, 13)
    assert np.array_equal(cache[..., :10, :], before[..., :10, :])            # context untouched
    assert np.array_equal(cache[..., 10:13, :], before[..., [10, 11, 13], :])  # gathered in order
    seg = np.arange(3 * 4, dtype=np.int16).reshape(3, 4)
    assert np.array_equal(oracle.seg_prune(seg, 15 - 10, retain), seg[[1, 2]])
    # a stage whose segment lies entirely among pruned indices ends up empty
    assert oracle.seg_prune(seg, 5, np.array([0, 1], dtype=np.int32)).shape[0] == 0


@pytest.mark.parametrize("dtype", [np.uint16, np.float32, np.float64])
def test_compact_random_against_fancy_indexing(dtype):
    rng = np.random.default_rng(5)
    for trial in range(20):
        L, H, cap, hd = 3, 2, 64, 4
        l_glo = int(rng.integers(0, 20))
        n_draft = int(rng.integers(0, 40))
        l_cache = l_glo + n_draft
        T = n_draft + int(rng.integers(0, 5))
        k = int(rng.integers(0, T + 1))
        retain = np.sort(rng.choice(T, size=k, replace=False)).astype(np.int32) if T > 0 else np.zeros(0, np.int32)
        n_acc = int(rng.integers(0, k + 1))
        cache = rng.integers(0, 60000, (L, 2, H, cap, hd)).astype(dtype)
        before = cache.copy()
        lg, lc = oracle.kv_compact(cache, l_glo, l_cache, retain, n_acc)
        inc = retain[retain + l_glo < l_cache]
        assert (lg, lc) == (l_glo + n_acc, l_glo + len(inc))
        assert np.array_equal(cache[:, :, :, :l_glo], before[:, :, :, :l_glo])
        assert np.array_equal(cache[:, :, :, l_glo:lc], before[:, :, :, l_glo + inc])
    # identity retain set: idempotent
    cache = rng.integers(0, 100, (1, 2, 1, 16, 2)).astype(dtype)
    before = cache.copy()
    oracle.kv_compact(cache, 4, 10, np.arange(6, dtype=np.int32), 0)
    assert np.array_equal(cache, before)


@pytest.mark.parametrize("seed", [20, 22, 27])
def test_compacted_kv_equals_accepted_path_kv_and_round_continues(seed):
    """After accept + compact, the draft region holds exactly the K/V that verifying only the kept nodes would
    have produced, and verifying the rest of the pruned tree gives the rows the unpruned tree would have given."""
    cfg = TINY
    tree = synth.random_tree(12, 5, 3, 64, seed)
    hid = synth.hidden(cfg, 12, 0, seed)
    # reference: the whole tree in one go
    full, *_ = make_oracle_stage(cfg, seed)
    out_full = verify_whole_tree(full, cfg, tree.parent, hid, 12)
    # an earlier stage has processed 8 nodes when the retain set arrives
    st, *_ = make_oracle_stage(cfg, seed)
    n_done = 8
    verify_whole_tree(st, cfg, tree.parent[:n_done], hid[:n_done], 4)
    # pick a depth-1 child of the root as n_new by planting
    child = next(i for i in range(1, 12) if tree.parent[i] == 0)
    amax = np.array([tree.token[child]], dtype=np.int32)
    res, retain = oracle.accept(amax, tree.token, tree.parent, 1)
    assert res.n_new == child and res.n_acc == 1
    lg, lc = oracle.kv_compact(st.kv, cfg.l_glo, cfg.l_glo + n_done, retain, res.n_acc)
    assert lg == cfg.l_glo + 1
    kept = retain[retain < n_done]
    assert lc == cfg.l_glo + len(kept)
    # cached K/V of kept nodes equal the reference run's K/V of the same nodes (positions are unchanged by pruning)
    assert np.array_equal(st.kv[:, :, :, cfg.l_glo:lc], full.kv[:, :, :, cfg.l_glo + kept])
    # continue on the pruned tree: remaining nodes of S_pr, new indices and new l_glo
    npar, _ = oracle.tree_remap(tree.parent, tree.token, retain, res.n_acc)
    pr = retain[res.n_acc:]
    done_pr = int((pr < n_done).sum())
    rest = pr[done_pr:]
    assert len(rest) > 0 and len(kept) < n_done
    out = st.verify(lg, lc, hid[rest], done_pr, npar)
    np.testing.assert_allclose(out, out_full[rest], rtol=1e-12, atol=1e-13)
