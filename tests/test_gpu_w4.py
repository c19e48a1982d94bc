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
