"""Full-size configurations (the shapes bench.py launches) against the oracle on the same seeded inputs."""
import time

import numpy as np
import pytest

from paper_2507_02620_amd import synth

pytestmark = pytest.mark.gpu


def _full_pass(cfg, seed, head_rows=0):
    """Whole tree in score-ordered segments on both sides, then accept + compaction of the planted path."""
    import torch
    from oracle import oracle
    from paper_2507_02620_amd import flowspec as fs
    from tests.gpu_util import TOL, Pair, max_rel_err, row_rel_err, to_dev
    t0 = time.time()
    print(f"[case] {cfg.name}: {cfg.n_layers} layers d={cfg.d_model} heads={cfg.n_q_heads}/{cfg.n_kv_heads} ffn={cfg.d_ffn} "
          f"prefix={cfg.l_glo} T={cfg.tree_size} seg={cfg.seg_len}", flush=True)
    p = Pair(cfg, seed, head=head_rows > 0)
    print(f"  inputs + stage ready after {time.time() - t0:.1f} s", flush=True)
    tree = synth.config_tree(cfg, seed)
    hid = synth.hidden(cfg, tree.size, 0, seed)
    T = tree.size
    o_out = np.zeros((T, cfg.d_model))
    g_out = torch.zeros((T, cfg.d_model), dtype=p.tdtype, device="cuda")
    hid_dev = to_dev(hid, p.tdtype)
    for off, n in synth.segments(T, cfg.seg_len):
        p.gpu.tree_verify_stage(p.kv, cfg.l_glo, cfg.l_glo + off, hid_dev[off:off + n].contiguous(), off, tree.parent[: off + n], g_out[off:off + n])
        o_out[off:off + n] = p.orc.verify(cfg.l_glo, cfg.l_glo + off, hid[off:off + n], off, tree.parent[: off + n])
        g_seg = g_out[off:off + n].float().cpu().numpy()
        err, rerr = max_rel_err(g_seg, o_out[off:off + n]), row_rel_err(g_seg, o_out[off:off + n])
        print(f"  segment at {off}: max-rel-err {err:.3e}, worst row {rerr:.3e}  ({time.time() - t0:.1f} s)", flush=True)
        assert err < TOL[cfg.dtype] and rerr < 2 * TOL[cfg.dtype]
    L = cfg.l_glo + T
    nl = p.orc.kv.shape[0]
    kv_g, kv_o = p.kv[:nl, :, :, cfg.l_glo:L].float().cpu().numpy(), p.orc.kv[:, :, :, cfg.l_glo:L]
    kerr = max_rel_err(kv_g, kv_o)
    kerr_l = max(max_rel_err(kv_g[l, x], kv_o[l, x]) for l in range(nl) for x in (0, 1))  # per layer, K and V apart
    krow = row_rel_err(kv_g, kv_o)
    print(f"  appended K/V max-rel-err {kerr:.3e}, worst layer {kerr_l:.3e}, worst row {krow:.3e}", flush=True)
    assert kerr < TOL[cfg.dtype] and kerr_l < TOL[cfg.dtype] and krow < 3 * TOL[cfg.dtype]
    if head_rows:
        rows = min(head_rows, cfg.seg_len)
        o_lg, o_am = p.orc.logits(o_out[:rows])
        g_lg, g_am = p.gpu.tree_logits(g_out[:rows].contiguous())
        lerr = max_rel_err(g_lg.cpu().numpy(), o_lg)
        print(f"  logits ({rows} rows x {cfg.vocab}) max-rel-err {lerr:.3e}", flush=True)
        assert lerr < TOL[cfg.dtype]
    # accept on identical synthetic argmax, then compaction of the real cache: bit-exact against the oracle's gather
    amax = np.random.default_rng(seed).integers(0, max(cfg.vocab, 2), T).astype(np.int32)
    for r, t in synth.resolve_plants(synth.plant_path(tree, T, seed, 1, 0.0, 3.0), tree, max(cfg.vocab, 2)):
        amax[r] = t
    o_res, o_ret = oracle.accept(amax, tree.token, tree.parent, T)
    res, retain, work = fs.new_accept_buffers(T, T)
    fs.tree_accept(None, torch.from_numpy(amax).cuda(), torch.from_numpy(tree.token).cuda(), torch.from_numpy(tree.parent).cuda(), T, res,
                   retain, work)
    g_res, g_ret = fs.accept_result_to_host(res, retain, T)
    assert g_res.as_tuple() == o_res.as_tuple() and np.array_equal(g_ret, o_ret)
    bits = torch.int32 if cfg.dtype == "f32" else torch.int16
    before = p.kv.view(bits).cpu().numpy().copy()
    lens = oracle.kv_compact(before, cfg.l_glo, L, o_ret, o_res.n_acc)
    new_len = torch.zeros(2, dtype=torch.int32, device="cuda")
    p.gpu.kv_compact(p.kv, cfg.l_glo, L, retain, res=res, new_len=new_len)
    assert tuple(new_len.cpu().tolist()) == lens
    assert np.array_equal(p.kv.view(bits).cpu().numpy()[:, :, :, : lens[1]], before[:, :, :, : lens[1]])
    print(f"  accept {g_res.as_tuple()} and compaction bit-exact; done in {time.time() - t0:.1f} s", flush=True)


def test_c2_llama2_7b_shape_full_depth():
    _full_pass(synth.CONFIGS["C2"], 0, head_rows=16)


def test_c3_llama2_13b_shape_full_depth():
    _full_pass(synth.CONFIGS["C3"], 0, head_rows=24)


def test_c4_qwen2_7b_gqa_shape_full_depth():
    _full_pass(synth.CONFIGS["C4"], 0, head_rows=32)


def test_c5_long_context_shape_full_depth():
    _full_pass(synth.CONFIGS["C5"], 0, head_rows=64)
