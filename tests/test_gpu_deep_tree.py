"""Trees deeper than 32 levels that are not chains (the pointer-doubling route of the mask / position kernels) on the HIP
path: masks and rotary tables bit for bit / to rounding against the oracle's ancestor sets, and the forward against the
oracle in segments of 64, as one 1024-row segment, in f32 and bf16, and as one item of a batch."""
import numpy as np
import pytest

from paper_2507_02620_amd import synth

pytestmark = pytest.mark.gpu

BASE = synth.StageConfig("deep-bf16", "bf16", 1, 256, 2, 2, 128, 512, 0, 10, 1024, 64, 1024, 0)


def _tree(spine, seed=3, size=1024):
    tree = synth.spine_tree(size, spine, 32000, seed)
    assert tree.depth.max() > 32, "the test must reach the deep-tree kernel"
    assert not all(tree.parent[i] == i - 1 for i in range(tree.size)), "a chain would take the closed-form kernel"
    return tree


def _mask_bits(anc_words):
    w = np.ascontiguousarray(anc_words).view(np.uint64)
    return ((w[:, :, None] >> np.arange(64, dtype=np.uint64)[None, None, :]) & np.uint64(1)).reshape(w.shape[0], -1).astype(bool)


@pytest.mark.parametrize("spine,seg", [(40, 64), (200, 64), (900, 64), (200, 1024), (900, 1000)])
def test_mask_and_positions_bit_exact(spine, seg):
    """fs_tree_mask (the forward's own kernels) against orc_tree_ancestors: masks bit for bit; cos / sin of the positions
    l_glo + depth against fp64 values (a wrong depth moves the first rotary pair by a radian)."""
    from oracle import oracle
    from tests.gpu_util import Pair
    tree = _tree(spine)
    T, l_glo = tree.size, 37
    cfg = BASE.with_(l_glo=l_glo, seg_len=seg)
    print(f"[case] mask spine={spine} seg={seg} depth={tree.depth.max()}", flush=True)
    p = Pair(cfg, 1, max_tree=T, max_seg=seg)
    anc_o, depth_o = oracle.tree_ancestors(tree.parent)
    want = _mask_bits(anc_o)[:, :T]
    half = cfg.head_dim // 2
    inv_freq = cfg.rope_theta ** (-2.0 * np.arange(half) / cfg.head_dim)
    for off, n in synth.segments(T, seg):
        anc, rope = p.gpu.tree_mask(l_glo, off, n, tree.parent[: off + n])
        got = _mask_bits(anc.cpu().numpy())
        assert (got[:, :T] == want[off:off + n]).all() and not got[:, T:].any(), (spine, seg, off)
        ang = (l_glo + depth_o[off:off + n, None]) * inv_freq[None, :]
        r = rope.cpu().numpy().astype(np.float64)
        assert np.abs(r[:, :, 0] - np.cos(ang)).max() < 2e-6 and np.abs(r[:, :, 1] - np.sin(ang)).max() < 2e-6


@pytest.mark.parametrize("dtype,spine,seg", [("bf16", 40, 64), ("bf16", 200, 64), ("bf16", 900, 64), ("f32", 200, 64), ("f32", 900, 1024),
                                             ("bf16", 200, 1024)])
def test_deep_tree_forward(dtype, spine, seg):
    from tests.gpu_util import TOL, Pair, max_rel_err, row_rel_err
    tree = _tree(spine)
    cfg = BASE.with_(name=f"deep-{dtype}-spine{spine}-seg{seg}", dtype=dtype, seg_len=seg,
                     **(dict(head_dim=64, n_q_heads=4, n_kv_heads=2) if dtype == "f32" else {}))
    print(f"[case] {cfg.name} depth={tree.depth.max()}", flush=True)
    p = Pair(cfg, 2, max_tree=tree.size, max_seg=seg)
    hid = synth.hidden(cfg, tree.size, 0, 2)
    o, g = p.verify_tree(tree.parent, hid, seg)
    err, rerr = max_rel_err(g, o), row_rel_err(g, o)
    L = cfg.l_glo + tree.size
    kerr = max_rel_err(p.kv[:, :, :, cfg.l_glo:L].float().cpu().numpy(), p.orc.kv[:, :, :, cfg.l_glo:L])
    print(f"  hidden max-rel-err {err:.3e}, worst row {rerr:.3e}, appended K/V {kerr:.3e}", flush=True)
    assert err < TOL[dtype] and rerr < 2 * TOL[dtype] and kerr < TOL[dtype]


def test_deep_tree_as_one_item_of_a_batch():
    """Three requests in one fs_tree_verify_batch call: a shallow tree, a deep spine tree (pointer-doubling kernel writing into
    the stacked mask arrays behind the first request's rows) and a chain; each checked against the oracle run on it alone."""
    import torch
    from oracle import oracle
    from tests.gpu_util import TOL, max_rel_err, to_dev
    cfg = BASE.with_(dtype="f32", head_dim=64, n_q_heads=4, n_kv_heads=2, l_glo=20, seg_len=64)
    from paper_2507_02620_amd import flowspec as fs
    layers = [synth.layer_weights(cfg, l, 4) for l in range(cfg.n_layers)]
    dev_layers = [{k: to_dev(v, torch.float32) for k, v in lw.items()} for lw in layers]
    cap = 400
    gst = fs.stage_from_config(cfg, dev_layers, kv_capacity=cap, max_tree=256, max_seg=192)
    trees = [synth.random_tree(64, 6, 3, 32000, 4).parent, _tree(60, 5, 150).parent, np.arange(-1, 99, dtype=np.int32)]
    l_glos = [20, 33, 11]
    seg_off = [0, 86, 36]                     # the deep tree's and the chain's last 64 rows
    items, hids, orcs, kvs = [], [], [], []
    for r, (par, lg, off) in enumerate(zip(trees, l_glos, seg_off)):
        orc = oracle.Stage(cfg, layers, None, None, cap)
        kv = gst.new_kv_cache()
        for l in range(cfg.n_layers):
            pre = synth.prefix_kv(cfg.with_(l_glo=lg), l, cap, 10 + r)
            orc.load_prefix(l, pre)
            kv[l].copy_(to_dev(pre, torch.float32))
        hid = synth.hidden(cfg, len(par), r, 4)
        if off:  # earlier segments of this request go through the single-request entry point on both sides
            orc.verify(lg, lg, hid[:off], 0, par[:off])
            gst.tree_verify_stage(kv, lg, lg, to_dev(hid[:off], torch.float32), 0, par[:off])
        n = len(par) - off
        items.append((kv, lg, lg + off, off, n, par))
        hids.append(hid[off:])
        orcs.append((orc, lg, off, hid, par))
        kvs.append(kv)
    print("[case] batch of 3: shallow / deep spine / chain", flush=True)
    out = gst.tree_verify_batch(items, to_dev(np.concatenate(hids), torch.float32))
    torch.cuda.synchronize()
    row = 0
    for (orc, lg, off, hid, par), kv, h in zip(orcs, kvs, hids):
        want = orc.verify(lg, lg + off, hid[off:], off, par)
        got = out[row:row + len(h)].cpu().numpy()
        row += len(h)
        assert max_rel_err(got, want) < TOL["f32"]
        L = lg + len(par)
        assert max_rel_err(kv[:, :, :, lg:L].cpu().numpy(), orc.kv[:, :, :, lg:L]) < TOL["f32"]
