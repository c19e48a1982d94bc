"""HIP path vs oracle, element by element, on the same seeded inputs (through the C ABI).  Needs an MI355X."""
import numpy as np
import pytest
import torch

from paper_2507_02620_amd import synth

pytestmark = pytest.mark.gpu


def _pair(*a, **k):
    from tests.gpu_util import Pair
    return Pair(*a, **k)


def _check_stage(cfg, seed, seg_len, head=False, tol=None):
    from tests.gpu_util import TOL, max_rel_err, row_rel_err
    tol = tol or TOL[cfg.dtype]
    print(f"[case] {cfg.name} seed={seed} seg_len={seg_len} T={cfg.tree_size} l_glo={cfg.l_glo}", flush=True)
    p = _pair(cfg, seed, head=head)
    tree = synth.config_tree(cfg, seed)
    hid = synth.hidden(cfg, tree.size, 0, seed)
    o_out, g_out = p.verify_tree(tree.parent, hid, seg_len)
    err, rerr = max_rel_err(g_out, o_out), row_rel_err(g_out, o_out)
    print(f"  hidden max-rel-err {err:.3e} (tol {tol}), worst row {rerr:.3e}", flush=True)
    assert np.isfinite(g_out).all()
    assert err < tol and rerr < 2 * tol
    # the K/V rows the stage appended for the draft tokens
    L = cfg.l_glo + tree.size
    kv_g = p.kv[:, :, :, cfg.l_glo:L].float().cpu().numpy()
    kv_o = p.orc.kv[:, :, :, cfg.l_glo:L]
    kerr = max_rel_err(kv_g, kv_o)
    # per layer and K / V apart (one global maximum would let a layer with small values hide), and the worst single row
    kerr_l = max(max_rel_err(kv_g[l, x], kv_o[l, x]) for l in range(cfg.n_layers) for x in (0, 1))
    krow = row_rel_err(kv_g, kv_o)
    print(f"  appended K/V max-rel-err {kerr:.3e}, worst layer {kerr_l:.3e}, worst row {krow:.3e}", flush=True)
    assert kerr < tol and kerr_l < tol and krow < 3 * tol
    # prefix untouched, bit for bit
    for l in range(cfg.n_layers):
        pre = synth.prefix_kv(cfg, l, p.orc.cap, seed)[:, :, : cfg.l_glo]
        assert np.array_equal(p.kv[l, :, :, : cfg.l_glo].float().cpu().numpy(), pre)
    return p, tree, o_out, g_out


def test_c1_tiny_fp32_stage():
    cfg = synth.CONFIGS["C1"]
    _check_stage(cfg, 0, cfg.seg_len)


@pytest.mark.parametrize("seg_len", [5, 16])
def test_c1_ragged_segments(seg_len):
    cfg = synth.CONFIGS["C1"].with_(tree_size=37, l_glo=131)
    _check_stage(cfg, 1, seg_len)


SMALL_BF16 = synth.StageConfig("small-bf16", "bf16", 2, 512, 4, 4, 128, 1376, 2000, 200, 40, 16, 6, 4)


@pytest.mark.parametrize("name,cfg,seg", [
    ("mha-128", SMALL_BF16, 16),
    ("mha-128-ragged24", SMALL_BF16.with_(tree_size=50, l_glo=333), 24),
    ("gqa-bias", SMALL_BF16.with_(n_q_heads=8, n_kv_heads=2, d_model=1024, qkv_bias=True, rms_eps=1e-6, rope_theta=1e6, l_glo=500,
                                  tree_size=70), 32),
    ("hd64", SMALL_BF16.with_(n_q_heads=8, n_kv_heads=8, head_dim=64), 16),
    ("seg64", SMALL_BF16.with_(tree_size=130, l_glo=1000, max_depth=12), 64),
    ("f32-hd128", SMALL_BF16.with_(dtype="f32", l_glo=100), 16),
    # one KV head under a group of 8 query heads, 27-row segments (14 row tiles, the last one ragged) and 34 K/V tiles: the
    # split plan's four-wave row blocks for wide groups on a long context
    ("gqa-wide-group-long-context", SMALL_BF16.with_(n_q_heads=8, n_kv_heads=1, d_model=1024, l_glo=2100, tree_size=60), 27),
])
def test_small_stages(name, cfg, seg):
    _check_stage(cfg.with_(name=name, seg_len=seg), 2, seg)


@pytest.mark.parametrize("name,cfg,seg,wgs", [
    # few workgroups -> long KV splits: the attention kernels that keep two tiles in flight, with even and odd tile counts and
    # tails of 1 .. 3 tiles (l_glo + tree size spans 7, 10 and 13 tiles of 64 slots; 19 tiles of 32 slots for f32 / hd 128)
    ("deep-7-tiles", SMALL_BF16.with_(l_glo=400, tree_size=40), 16, 4),
    ("deep-10-tiles", SMALL_BF16.with_(l_glo=590, tree_size=48), 16, 4),
    ("deep-13-tiles-2-splits", SMALL_BF16.with_(l_glo=790, tree_size=40), 16, 8),
    ("deep-hd64", SMALL_BF16.with_(n_q_heads=8, n_kv_heads=8, head_dim=64, l_glo=520, tree_size=40), 16, 8),
    ("deep-f32-hd128", SMALL_BF16.with_(dtype="f32", l_glo=560, tree_size=40), 16, 4),
    ("deep-seg48-3-row-tiles", SMALL_BF16.with_(l_glo=600, tree_size=96, max_depth=10), 48, 4),
    ("deep-seg64-two-row-tiles-per-wave", SMALL_BF16.with_(l_glo=600, tree_size=128, max_depth=10), 64, 4),
])
def test_long_kv_splits(name, cfg, seg, wgs, monkeypatch):
    """Tree attention with many tiles per workgroup (the split plan is steered through its tuning knob)."""
    monkeypatch.setenv("FLOWSPEC_ATTN_WGS", str(wgs))
    _check_stage(cfg.with_(name=name, seg_len=seg), 5, seg)


@pytest.mark.parametrize("name,cfg,seg,wgs,nset", [
    # three and four K/V tiles in flight per workgroup: 13 tiles in one split (ring rounds + a ragged tail), two splits of 7 / 6,
    # head dim 64, and a context so short that most tiles are draft slots (mask words fetched ahead of every tile)
    ("ring3-13-tiles", SMALL_BF16.with_(l_glo=790, tree_size=40), 16, 4, 3),
    ("ring4-13-tiles", SMALL_BF16.with_(l_glo=790, tree_size=40), 16, 4, 4),
    ("ring3-two-splits", SMALL_BF16.with_(l_glo=790, tree_size=40), 16, 8, 3),
    ("ring4-hd64-17-tiles", SMALL_BF16.with_(n_q_heads=8, n_kv_heads=8, head_dim=64, l_glo=1040, tree_size=40), 16, 8, 4),
    ("ring4-mostly-draft-slots", SMALL_BF16.with_(l_glo=8, tree_size=640, max_depth=14), 16, 4, 4),
    ("ring3-mostly-draft-slots", SMALL_BF16.with_(l_glo=70, tree_size=500, max_depth=14), 16, 4, 3),
])
def test_long_kv_splits_deeper_rings(name, cfg, seg, wgs, nset, monkeypatch):
    monkeypatch.setenv("FLOWSPEC_ATTN_WGS", str(wgs))
    monkeypatch.setenv("FLOWSPEC_ATTN_NSET", str(nset))
    monkeypatch.setenv("FLOWSPEC_ATTN_MTW", "1")
    _check_stage(cfg.with_(name=name, seg_len=seg), 5, seg)


@pytest.mark.parametrize("bufs", [2, 3, 4])
@pytest.mark.parametrize("name,cfg,seg,wgs", [
    # the tree-attention kernel that copies K/V tiles straight into LDS (2 to 4 tile buffers): one split of 13 tiles with a
    # ragged tail, two splits, a split shorter than the buffer ring, 64-row segments (4 waves computing), a ragged 24-row
    # segment (two of the waves compute), and a context so short that most tiles are draft slots
    ("dma-13-tiles", SMALL_BF16.with_(l_glo=790, tree_size=40), 16, 4),
    ("dma-two-splits", SMALL_BF16.with_(l_glo=790, tree_size=40), 16, 8),
    ("dma-short-splits", SMALL_BF16.with_(l_glo=300, tree_size=40), 16, 16),
    ("dma-seg64", SMALL_BF16.with_(l_glo=600, tree_size=128, max_depth=10), 64, 4),
    ("dma-seg24-ragged", SMALL_BF16.with_(l_glo=333, tree_size=50), 24, 4),
    ("dma-mostly-draft-slots", SMALL_BF16.with_(l_glo=8, tree_size=640, max_depth=14), 16, 4),
    ("dma-gqa-row-blocks", SMALL_BF16.with_(n_q_heads=8, n_kv_heads=2, d_model=1024, l_glo=500, tree_size=70), 16, 8),
])
def test_long_kv_splits_direct_to_lds(name, cfg, seg, wgs, bufs, monkeypatch):
    if "row-blocks" in name:  # two one-tile waves per workgroup: the 64 stacked rows of a KV head make two row blocks
        monkeypatch.setenv("FLOWSPEC_ATTN_NWC", "2")
    monkeypatch.setenv("FLOWSPEC_ATTN_WGS", str(wgs))
    monkeypatch.setenv("FLOWSPEC_ATTN_DMA", str(bufs))
    _check_stage(cfg.with_(name=f"{name}-{bufs}", seg_len=seg), 5, seg)


@pytest.mark.parametrize("name,cfg,seg,wgs", [
    # one case per tree-attention variant, each with a context so short (l_glo <= 16) that the draft slots — the part the
    # ancestor mask governs — carry most of the attention weight
    ("mask-one-row-tile", SMALL_BF16.with_(l_glo=8), 16, None),
    ("mask-two-tiles-in-flight", SMALL_BF16.with_(l_glo=8, tree_size=300, max_depth=12), 16, 4),
    ("mask-two-row-tiles-per-wave", SMALL_BF16.with_(l_glo=16, tree_size=130, max_depth=12), 64, None),
    ("mask-two-row-tiles-long-split", SMALL_BF16.with_(l_glo=16, tree_size=320, max_depth=12), 64, 4),
    ("mask-hd64", SMALL_BF16.with_(n_q_heads=8, n_kv_heads=8, head_dim=64, l_glo=5, tree_size=200, max_depth=10), 16, 8),
    ("mask-gqa", SMALL_BF16.with_(n_q_heads=8, n_kv_heads=2, d_model=1024, l_glo=12, tree_size=100, max_depth=10), 32, None),
    ("mask-gqa-row-blocks", SMALL_BF16.with_(n_q_heads=8, n_kv_heads=2, d_model=1024, l_glo=3, tree_size=200, max_depth=10), 80, None),
    ("mask-gqa-four-wave-row-blocks", SMALL_BF16.with_(n_q_heads=8, n_kv_heads=2, d_model=1024, l_glo=12, tree_size=200, max_depth=10), 48, -4),
    ("mask-direct-to-lds", SMALL_BF16.with_(l_glo=8, tree_size=300, max_depth=12), 16, -100),
])
def test_bf16_comparison_would_notice_a_wrong_mask(name, cfg, seg, wgs, monkeypatch):
    """The bf16 tolerance is wide, so these cases show that the comparison still discriminates: the HIP path's distance
    from the oracle must stay below a quarter of the distance between the oracle and an oracle run on a tree with the same
    depths (same positions) but other ancestors."""
    from tests.gpu_util import max_rel_err
    from tests.helpers import make_oracle_stage, reparent_same_depth, verify_whole_tree
    if wgs == -100:  # the direct-to-LDS kernel, three tile buffers, long splits
        monkeypatch.setenv("FLOWSPEC_ATTN_DMA", "3")
        monkeypatch.setenv("FLOWSPEC_ATTN_WGS", "4")
    elif wgs and wgs < 0:  # at most -wgs one-tile waves per workgroup: row blocks of four-wave workgroups
        monkeypatch.setenv("FLOWSPEC_ATTN_NWC", str(-wgs))
        monkeypatch.setenv("FLOWSPEC_ATTN_MTW", "1")
    elif wgs:
        monkeypatch.setenv("FLOWSPEC_ATTN_WGS", str(wgs))
    cfg = cfg.with_(name=name, seg_len=seg)
    p, tree, o_out, g_out = _check_stage(cfg, 7, seg)
    wrong_parent, moved = reparent_same_depth(tree.parent, 7)
    assert moved >= tree.size // 2
    st2, _, _, _ = make_oracle_stage(cfg, 7, capacity=p.orc.cap)
    hid = synth.hidden(cfg, tree.size, 0, 7)
    o_wrong = verify_whole_tree(st2, cfg, wrong_parent, hid, seg)
    sens = max_rel_err(o_wrong, o_out)
    err = max_rel_err(g_out, o_out)
    L = cfg.l_glo + tree.size
    ksens = max_rel_err(st2.kv[:, :, :, cfg.l_glo:L], p.orc.kv[:, :, :, cfg.l_glo:L])
    kerr = max_rel_err(p.kv[:, :, :, cfg.l_glo:L].float().cpu().numpy(), p.orc.kv[:, :, :, cfg.l_glo:L])
    print(f"  wrong-mask distance: hidden {sens:.3e} (HIP path {err:.3e}), appended K/V {ksens:.3e} (HIP path {kerr:.3e})", flush=True)
    assert err < 0.25 * sens and kerr < 0.25 * ksens
