"""HIP path with 4-bit group weights (W4A16, the paper's 13B setting, Sec. IV-A) against the oracle run on the plain
matrices the codes stand for.  Same tolerance as the dense bf16 path: only activations, KV and outputs are rounded to
bf16; the weights are identical on both sides."""
import numpy as np
import pytest

from paper_2507_02620_amd import synth

pytestmark = pytest.mark.gpu

SMALL = synth.StageConfig("w4-small", "bf16", 2, 512, 4, 2, 128, 1408, 1000, 96, 40, 16, 5, 3, qkv_bias=True)


@pytest.mark.parametrize("seg", [16, 7, 24, 40])
def test_w4_small_stage(seg):
    import torch
    from tests.gpu_util import TOL, Pair, max_rel_err, to_dev
    cfg = SMALL.with_(seg_len=seg)
    print(f"case w4 small seg={seg}", flush=True)
    pair = Pair(cfg, seed=11, head=True, w4=True)
    tree = synth.config_tree(cfg, seed=11)
    hid = synth.hidden(cfg, cfg.tree_size, 0, 11)
    o, g = pair.verify_tree(tree.parent, hid, seg)
    err = max_rel_err(g, o)
    print(f"  hidden max-rel-err {err:.3e}", flush=True)
    assert err < TOL["bf16"]
    # logits of the last segment's rows
    n = min(seg, cfg.tree_size)
    rows = synth.storage(cfg, o[:n].astype(np.float32))
    lo, _ = pair.orc.logits(rows.astype(np.float64))
    lg, am = pair.gpu.tree_logits(to_dev(rows, torch.bfloat16))
    err = max_rel_err(lg.float().cpu().numpy(), lo)
    print(f"  logits max-rel-err {err:.3e}", flush=True)
    assert err < TOL["bf16"]


def test_w4_64_row_segment_head_dim_64():
    from tests.gpu_util import TOL, Pair, max_rel_err
    cfg = synth.StageConfig("w4-hd64", "bf16", 1, 384, 6, 3, 64, 896, 0, 70, 64, 64, 6, 4)
    print("case w4 hd64 seg=64", flush=True)
    pair = Pair(cfg, seed=5, w4=True)
    tree = synth.config_tree(cfg, seed=5)
    hid = synth.hidden(cfg, cfg.tree_size, 0, 5)
    o, g = pair.verify_tree(tree.parent, hid, 64)
    err = max_rel_err(g, o)
    print(f"  hidden max-rel-err {err:.3e}", flush=True)
    assert err < TOL["bf16"]


def test_w4_13b_shape_two_layers():
    """LLaMA2-13B layer shape (d 5120, 40 heads, FFN 13824, segment 24), two layers, with the head."""
    import torch
    from tests.gpu_util import TOL, Pair, max_rel_err, to_dev
    cfg = synth.CONFIGS["C3"].with_(n_layers=2)
    print("case w4 C3 shape, 2 layers", flush=True)
    pair = Pair(cfg, seed=2, head=True, w4=True)
    tree = synth.config_tree(cfg, seed=2)
    hid = synth.hidden(cfg, cfg.tree_size, 0, 2)
    o, g = pair.verify_tree(tree.parent, hid, cfg.seg_len)
    err = max_rel_err(g, o)
    print(f"  hidden max-rel-err {err:.3e}", flush=True)
    assert err < TOL["bf16"]
    rows = synth.storage(cfg, o[:cfg.seg_len].astype(np.float32))
    lo, _ = pair.orc.logits(rows.astype(np.float64))
    lg, am = pair.gpu.tree_logits(to_dev(rows, torch.bfloat16))
    lg = lg.float().cpu().numpy()
    err = max_rel_err(lg, lo)
    print(f"  logits max-rel-err {err:.3e}", flush=True)
    assert err < TOL["bf16"]
    # argmax: equal wherever the oracle's top two are further apart than the bf16-level error of a logit
    top2 = np.sort(lo, axis=1)[:, -2:]
    clear = (top2[:, 1] - top2[:, 0]) > 4 * TOL["bf16"] * np.abs(lo).max()
    assert np.array_equal(am.cpu().numpy()[clear], lo.argmax(axis=1)[clear])


def test_w4_many_row_chain():
    """A 200-row chain in one segment with 4-bit weights (row blocks of the few-row kernel)."""
    from tests.gpu_util import TOL, Pair, max_rel_err
    cfg = synth.StageConfig("w4-chain", "bf16", 2, 512, 4, 4, 128, 1408, 0, 60, 200, 200, 200, 1)
    print("case w4 chain 200 rows", flush=True)
    pair = Pair(cfg, seed=8, w4=True)
    hid = synth.hidden(cfg, 200, 0, 8)
    o, g = pair.verify_tree(np.arange(-1, 199, dtype=np.int32), hid, 200)
    err = max_rel_err(g, o)
    print(f"  hidden max-rel-err {err:.3e}", flush=True)
    assert err < TOL["bf16"]


def test_w4_rejects_f32_and_bad_shapes():
    from paper_2507_02620_amd import flowspec as fs
    with pytest.raises(fs.FlowSpecError):
        fs.Stage(n_layers=1, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ffn=512, vocab=0, dtype=fs.FS_F32, rms_eps=1e-5,
                 rope_theta=1e4, kv_capacity=64, max_tree=16, max_seg=16, layers=[], weight_format=fs.FS_WFMT_INT4_G128)


def _random_w4(i):
    r = np.random.default_rng(8200 + i)
    hd = int(r.choice([64, 128]))
    n_kv = int(r.choice([1, 2, 4]))
    n_q = n_kv * int(r.choice([1, 2, 4]))
    while (n_q * hd) % 128:   # one scale per 128 input columns of the attention output projection
        n_q += n_kv
    return synth.StageConfig(f"w4-rnd{i}", "bf16", int(r.integers(1, 3)), int(r.integers(2, 8)) * 128, n_q, n_kv, hd, int(r.integers(3, 12)) * 128,
                             int(r.choice([0, 777, 2000])), int(r.choice([0, 5, int(r.integers(6, 1200))])), int(r.integers(2, 120)),
                             int(r.integers(1, 66)), int(r.integers(2, 20)), int(r.choice([0, 2, 4])), qkv_bias=bool(i % 2))


@pytest.mark.parametrize("i", range(8))
def test_w4_random_shapes(i):
    """Seeded random 4-bit stages (widths in multiples of the 128-column scale group, ragged trees and segments, with and
    without head): hidden states, appended K/V and logits against the oracle."""
    import torch
    from tests.gpu_util import TOL, Pair, max_rel_err, to_dev
    cfg = _random_w4(i)
    print(f"[case] {cfg}", flush=True)
    pair = Pair(cfg, seed=60 + i, head=cfg.vocab > 0, w4=True)
    tree = synth.config_tree(cfg, seed=60 + i)
    hid = synth.hidden(cfg, tree.size, 0, 60 + i)
    o, g = pair.verify_tree(tree.parent, hid, cfg.seg_len)
    err = max_rel_err(g, o)
    L = cfg.l_glo + tree.size
    kerr = max_rel_err(pair.kv[:, :, :, cfg.l_glo:L].float().cpu().numpy(), pair.orc.kv[:, :, :, cfg.l_glo:L])
    print(f"  hidden max-rel-err {err:.3e}, appended K/V {kerr:.3e}", flush=True)
    assert err < TOL["bf16"] and kerr < TOL["bf16"]
    if cfg.vocab:
        n = min(cfg.seg_len, tree.size)
        rows = synth.storage(cfg, o[:n].astype(np.float32))
        lo, _ = pair.orc.logits(rows.astype(np.float64))
        lg, _ = pair.gpu.tree_logits(to_dev(rows, torch.bfloat16))
        lerr = max_rel_err(lg.float().cpu().numpy(), lo)
        print(f"  logits max-rel-err {lerr:.3e}", flush=True)
        assert lerr < TOL["bf16"]
