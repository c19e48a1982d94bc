"""Shared test plumbing: tiny configs and oracle stages built from the seeded generators."""
import numpy as np

from oracle import oracle
from paper_2507_02620_amd import synth

TINY = synth.StageConfig("tiny", "f32", 2, 32, 4, 2, 8, 48, 64, 5, 12, 4, 5, 0)


def make_oracle_stage(cfg, seed=0, capacity=None, head=False, bf16_bits=False, n_layers=None):
    nl = cfg.n_layers if n_layers is None else n_layers
    cfg = cfg.with_(n_layers=nl)
    layers = [synth.layer_weights(cfg, l, seed) for l in range(nl)]
    fn, lm = synth.head_weights(cfg, seed) if head else (None, None)
    if bf16_bits:
        conv = lambda a: None if a is None else synth.f32_to_bf16_bits(a)
        st = oracle.Stage(cfg, [{k: conv(v) for k, v in lw.items()} for lw in layers], conv(fn), conv(lm), capacity, bf16_bits=True)
    else:
        st = oracle.Stage(cfg, layers, fn, lm, capacity)
    prefix = [synth.prefix_kv(cfg, l, st.cap, seed) for l in range(nl)]
    for l in range(nl):
        st.load_prefix(l, prefix[l])
    return st, layers, prefix, (fn, lm)


def verify_whole_tree(st, cfg, tree_parent, hid, seg_len, l_glo=None):
    """Run the oracle over S in consecutive segments; returns all output rows."""
    l_glo = cfg.l_glo if l_glo is None else l_glo
    T = len(tree_parent)
    out = np.zeros((T, cfg.d_model))
    for off, n in synth.segments(T, seg_len):
        out[off:off + n] = st.verify(l_glo, l_glo + off, hid[off:off + n], off, tree_parent[: off + n])
    return out


def ancestors_by_walking(parent):
    """Reflexive-transitive ancestor closure, one node at a time (independent of the oracle's recurrence)."""
    T = len(parent)
    m = np.zeros((T, T), dtype=bool)
    for i in range(T):
        j = i
        while j >= 0:
            m[i, j] = True
            j = int(parent[j])
    return m


def reparent_same_depth(parent, seed=0):
    """A tree with the same depths (hence the same positions) but other ancestors: every node that has a choice moves under
    another earlier node of its parent's depth.  Returns (new parent array, number of nodes moved).  Used to show that a
    comparison would notice a wrong ancestor mask."""
    parent = np.asarray(parent, dtype=np.int32)
    depth = synth._depths(parent)
    rng = np.random.default_rng(seed)
    out = parent.copy()
    moved = 0
    for i in range(1, len(parent)):
        if parent[i] < 0:
            continue
        cands = [j for j in range(i) if depth[j] == depth[parent[i]] and j != parent[i]]
        if cands:
            out[i] = cands[int(rng.integers(0, len(cands)))]
            moved += 1
    assert (synth._depths(out) == depth).all()
    return out, moved
