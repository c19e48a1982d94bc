"""Pins for the oracle's forward (tree mask, positions, decoder layers).  CPU only."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import oracle
from paper_2507_02620_amd import synth
from tests import textbook
from tests.helpers import TINY, ancestors_by_walking, make_oracle_stage, verify_whole_tree


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_mask_is_ancestor_closure(seed):
    tree = synth.random_tree(100, 9, 3, 50, seed)
    anc, depth = oracle.tree_ancestors(tree.parent)
    walk = ancestors_by_walking(tree.parent)
    bits = np.zeros_like(walk)
    for i in range(tree.size):
        for j in range(tree.size):
            bits[i, j] = (int(anc[i, j // 64]) >> (j % 64)) & 1
    assert (bits == walk).all()
    assert (np.triu(bits, 1) == 0).all()                      # S is a topological order: lower triangular
    assert (bits.sum(1) == depth + 1).all()                   # popcount = depth + 1
    assert (depth == tree.depth).all()


def test_bad_topology_is_rejected():
    with pytest.raises(oracle.OracleError):
        oracle.tree_ancestors([-1, 0, 2])
    with pytest.raises(oracle.OracleError):
        oracle.tree_ancestors([-1, -2])


def test_rmsnorm_library_and_closed_form():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(40)
    g = (1 + 0.1 * rng.standard_normal(40)).astype(np.float32)
    ref = F.rms_norm(torch.tensor(x), (40,), torch.tensor(g, dtype=torch.float64), 1e-5).numpy()
    np.testing.assert_allclose(oracle.rmsnorm(x, g, 1e-5), ref, rtol=1e-13, atol=0)
    # constant vector c: x / sqrt(c^2 + eps) * g
    c = 3.0
    out = oracle.rmsnorm(np.full(8, c), np.arange(1, 9, dtype=np.float32), 1e-6)
    np.testing.assert_allclose(out, c / np.sqrt(c * c + 1e-6) * np.arange(1, 9), rtol=1e-14)


def test_rope_closed_forms():
    rng = np.random.default_rng(1)
    hd, theta = 16, 1e4
    q, k = rng.standard_normal(hd), rng.standard_normal(hd)
    np.testing.assert_allclose(oracle.rope(q, 0, theta), q, atol=0)                      # position 0: identity
    np.testing.assert_allclose(np.linalg.norm(oracle.rope(q, 37, theta)), np.linalg.norm(q), rtol=1e-13)
    # relative-position property: <R_m q, R_n k> depends on m - n only
    a = oracle.rope(q, 1037, theta) @ oracle.rope(k, 1030, theta)
    b = oracle.rope(q, 7, theta) @ oracle.rope(k, 0, theta)
    np.testing.assert_allclose(a, b, rtol=1e-10)
    # complex-multiplication form, pairing t with t + hd/2
    np.testing.assert_allclose(oracle.rope(q, 11, theta), textbook.rope_complex(torch.tensor(q), 11, theta).numpy(), rtol=1e-12, atol=1e-14)
    # first pair rotates by exactly pos radians (frequency theta^0 = 1); the sign convention is counter-clockwise
    v = np.zeros(hd)
    v[0] = 1.0
    r = oracle.rope(v, 0.5, theta)
    np.testing.assert_allclose([r[0], r[hd // 2]], [np.cos(0.5), np.sin(0.5)], rtol=1e-14)
    # last pair uses frequency theta^(-(hd-2)/hd)
    v = np.zeros(hd)
    v[hd // 2 - 1] = 1.0
    r = oracle.rope(v, 3.0, theta)
    ang = 3.0 * theta ** (-(hd - 2) / hd)
    np.testing.assert_allclose([r[hd // 2 - 1], r[hd - 1]], [np.cos(ang), np.sin(ang)], rtol=1e-13)


@pytest.mark.parametrize("seed,seg_len", [(0, 4), (1, 5), (2, 12), (3, 1)])
def test_tree_rows_equal_per_path_sequential_decoding(seed, seg_len):
    """The brute-force pin: every node's output row == ordinary causal decoding of its root-to-node path."""
    cfg = TINY
    tree = synth.random_tree(cfg.tree_size, cfg.max_depth, 3, cfg.vocab, seed)
    st, layers, prefix, _ = make_oracle_stage(cfg, seed)
    hid = synth.hidden(cfg, tree.size, 0, seed)
    out = verify_whole_tree(st, cfg, tree.parent, hid, seg_len)
    pre = [p[:, :, : cfg.l_glo, :] for p in prefix]
    for i in range(tree.size):
        path = textbook.path_to(tree.parent, i)
        ref, dec = textbook.decode_path(cfg, layers, pre, hid[path], cfg.l_glo)
        np.testing.assert_allclose(out[i], ref[-1], rtol=1e-9, atol=1e-11)
        # cached K/V of the node (slot l_glo + i) equals what sequential decoding cached for it
        for l in range(cfg.n_layers):
            np.testing.assert_allclose(st.kv[l, 0, :, cfg.l_glo + i, :], dec.k[l][:, -1, :].numpy(), rtol=1e-9, atol=1e-11)
            np.testing.assert_allclose(st.kv[l, 1, :, cfg.l_glo + i, :], dec.v[l][:, -1, :].numpy(), rtol=1e-9, atol=1e-11)


def test_forest_and_literal_c1_tree():
    """Several roots (parent -1 for i > 0): such a node sees the context and itself only."""
    cfg = synth.CONFIGS["C1"].with_(d_model=64, n_q_heads=2, n_kv_heads=2, head_dim=32, d_ffn=80, l_glo=9)
    tree = synth.config_tree(cfg, 5)
    assert (tree.parent[1:] == -1).any()
    st, layers, prefix, _ = make_oracle_stage(cfg, 5)
    hid = synth.hidden(cfg, tree.size, 0, 5)
    out = verify_whole_tree(st, cfg, tree.parent, hid, 16)
    pre = [p[:, :, : cfg.l_glo, :] for p in prefix]
    for i in range(tree.size):
        path = textbook.path_to(tree.parent, i)
        ref, _ = textbook.decode_path(cfg, layers, pre, hid[path], cfg.l_glo)
        np.testing.assert_allclose(out[i], ref[-1], rtol=1e-9, atol=1e-11)


def test_chain_tree_is_causal_prefill_and_empty_prefix():
    """parent[i] = i-1 reduces to chunked prefill with a causal mask; l_glo = 0 means no context."""
    cfg = TINY.with_(l_glo=0, n_layers=1)
    T = 9
    parent = np.arange(-1, T - 1, dtype=np.int32)
    st, layers, prefix, _ = make_oracle_stage(cfg, 3)
    hid = synth.hidden(cfg, T, 0, 3)
    out = verify_whole_tree(st, cfg, parent, hid, 4)
    # library-routine reference: one batched causal pass
    w = {k: (None if v is None else torch.tensor(v, dtype=torch.float64)) for k, v in layers[0].items()}
    x = torch.tensor(hid, dtype=torch.float64)
    n = F.rms_norm(x, (cfg.d_model,), w["rms_attn"], cfg.rms_eps)
    q = F.linear(n, w["wq"]).view(T, cfg.n_q_heads, cfg.head_dim)
    k = F.linear(n, w["wk"]).view(T, cfg.n_kv_heads, cfg.head_dim)
    v = F.linear(n, w["wv"]).view(T, cfg.n_kv_heads, cfg.head_dim)
    q = torch.stack([textbook.rope_complex(q[t], t, cfg.rope_theta) for t in range(T)])
    k = torch.stack([textbook.rope_complex(k[t], t, cfg.rope_theta) for t in range(T)])
    G = cfg.n_q_heads // cfg.n_kv_heads
    o = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1).repeat_interleave(G, 0),
                                       v.transpose(0, 1).repeat_interleave(G, 0), is_causal=True)
    x = x + F.linear(o.transpose(0, 1).reshape(T, -1), w["wo"])
    n = F.rms_norm(x, (cfg.d_model,), w["rms_ffn"], cfg.rms_eps)
    x = x + F.linear(F.silu(F.linear(n, w["w_gate"])) * F.linear(n, w["w_up"]), w["w_down"])
    np.testing.assert_allclose(out, x.numpy(), rtol=1e-9, atol=1e-11)


def test_star_forest_is_single_token_decode():
    cfg = TINY
    T = 6
    parent = np.full(T, -1, dtype=np.int32)
    st, layers, prefix, _ = make_oracle_stage(cfg, 4)
    hid = synth.hidden(cfg, T, 0, 4)
    out = verify_whole_tree(st, cfg, parent, hid, 6)
    pre = [p[:, :, : cfg.l_glo, :] for p in prefix]
    for i in range(T):
        ref, _ = textbook.decode_path(cfg, layers, pre, hid[[i]], cfg.l_glo)
        np.testing.assert_allclose(out[i], ref[0], rtol=1e-9, atol=1e-11)


def test_segment_invariance_is_bitwise():
    cfg = TINY
    tree = synth.random_tree(12, 5, 3, 64, 7)
    hid = synth.hidden(cfg, 12, 0, 7)
    outs, caches = [], []
    for seg in (1, 4, 5, 12):
        st, *_ = make_oracle_stage(cfg, 7)
        outs.append(verify_whole_tree(st, cfg, tree.parent, hid, seg))
        caches.append(st.kv.copy())
    for o, c in zip(outs[1:], caches[1:]):
        assert np.array_equal(o, outs[0])
        assert np.array_equal(c, caches[0])


def test_single_visible_slot_returns_its_value():
    """No context and a root: softmax over one slot is 1, so attention returns V of that slot, whatever Q and K are."""
    cfg = TINY.with_(l_glo=0, n_layers=1, n_q_heads=2, n_kv_heads=2, head_dim=16)
    layers = [synth.layer_weights(cfg, 0, 9)]
    # make W_o the identity and W_down zero so the stage output is x + v
    layers[0]["wo"] = np.eye(cfg.d_model, dtype=np.float32)
    layers[0]["w_down"] = np.zeros_like(layers[0]["w_down"])
    st = oracle.Stage(cfg, layers)
    hid = synth.hidden(cfg, 1, 0, 9)
    out = st.verify(0, 0, hid, 0, np.array([-1], dtype=np.int32))
    v = F.linear(F.rms_norm(torch.tensor(hid[0], dtype=torch.float64), (cfg.d_model,),
                            torch.tensor(layers[0]["rms_attn"], dtype=torch.float64), cfg.rms_eps),
                 torch.tensor(layers[0]["wv"], dtype=torch.float64)).numpy()
    np.testing.assert_allclose(out[0], hid[0] + v, rtol=1e-12, atol=1e-13)


def test_bf16_bit_pattern_weights_equal_widened_float_weights():
    cfg = TINY.with_(dtype="bf16")
    tree = synth.random_tree(8, 4, 3, 64, 11)
    hid = synth.hidden(cfg, 8, 0, 11)
    a, *_ = make_oracle_stage(cfg, 11)
    b, *_ = make_oracle_stage(cfg, 11, bf16_bits=True)
    assert np.array_equal(verify_whole_tree(a, cfg, tree.parent, hid, 8), verify_whole_tree(b, cfg, tree.parent, hid, 8))


def test_lm_head_and_argmax():
    cfg = TINY
    st, layers, prefix, (fn, lm) = make_oracle_stage(cfg, 2, head=True)
    hid = synth.hidden(cfg, 5, 3, 2).astype(np.float64)
    lg, am = st.logits(hid)
    ref = textbook.lm_head(cfg, fn, lm, hid)
    np.testing.assert_allclose(lg, ref.astype(np.float32), rtol=1e-6, atol=1e-7)
    assert (am == ref.argmax(1)).all()
    # ties: lowest index wins; NaN never wins; all-NaN row -> 0
    t = np.array([[1, 5, 5, 2], [np.nan, 3, 3, np.nan], [np.nan] * 4, [-np.inf] * 4], dtype=np.float32)
    assert oracle.argmax_rows(t).tolist() == [1, 1, 0, 0]


def test_dropping_the_prefix_or_the_mask_changes_the_result():
    """Guards against a vacuous pin: the per-path comparison above must be sensitive to mask and context."""
    cfg = TINY
    tree = synth.random_tree(12, 5, 3, 64, 0)
    st, layers, prefix, _ = make_oracle_stage(cfg, 0)
    hid = synth.hidden(cfg, 12, 0, 0)
    out = verify_whole_tree(st, cfg, tree.parent, hid, 12)
    chain = np.arange(-1, 11, dtype=np.int32)
    st2, *_ = make_oracle_stage(cfg, 0)
    out_chain = verify_whole_tree(st2, cfg, chain, hid, 12)
    assert np.abs(out - out_chain).max() > 1e-3
