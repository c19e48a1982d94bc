"""Edge cases of the HIP path: degenerate sizes, ragged and over-long segments, aliasing, strided caches, error codes."""
import numpy as np
import pytest

from paper_2507_02620_amd import synth

pytestmark = pytest.mark.gpu

BASE = synth.StageConfig("edge-bf16", "bf16", 2, 256, 2, 2, 128, 512, 0, 70, 40, 16, 6, 3)


def _pair(*a, **k):
    from tests.gpu_util import Pair
    return Pair(*a, **k)


@pytest.mark.parametrize("seg", [1, 3, 17, 33, 65, 100])
def test_segment_lengths_including_more_than_64_rows(seg):
    """l_s = 1 (one MFMA row), ragged tails, and segments longer than one 64-row pass (the kernels loop over row blocks)."""
    from tests.gpu_util import TOL, max_rel_err
    cfg = BASE.with_(tree_size=131, seg_len=seg, l_glo=77, max_depth=9)
    print(f"[case] seg={seg}", flush=True)
    p = _pair(cfg, 9)
    tree = synth.config_tree(cfg, 9)
    hid = synth.hidden(cfg, tree.size, 0, 9)
    o, g = p.verify_tree(tree.parent, hid, seg)
    err = max_rel_err(g, o)
    print(f"  max-rel-err {err:.3e}", flush=True)
    assert err < TOL["bf16"]


def test_f32_long_segment_and_empty_prefix():
    from tests.gpu_util import TOL, max_rel_err
    cfg = synth.CONFIGS["C1"].with_(tree_size=90, seg_len=70, l_glo=0, forest=False, max_branch=3, max_depth=8)
    p = _pair(cfg, 4)
    tree = synth.config_tree(cfg, 4)
    hid = synth.hidden(cfg, tree.size, 0, 4)
    o, g = p.verify_tree(tree.parent, hid, 70)
    assert max_rel_err(g, o) < TOL["f32"]


def test_largest_tree_1024_nodes_deep_chain_segments_of_64():
    from tests.gpu_util import TOL, max_rel_err
    cfg = BASE.with_(tree_size=1024, seg_len=64, l_glo=10, max_depth=60, max_branch=2, n_layers=1)
    print("[case] T=1024", flush=True)
    p = _pair(cfg, 3)
    tree = synth.config_tree(cfg, 3)
    assert tree.depth.max() >= 15
    hid = synth.hidden(cfg, tree.size, 0, 3)
    o, g = p.verify_tree(tree.parent, hid, 64)
    assert max_rel_err(g, o) < TOL["bf16"]


def test_zero_length_segment_and_in_place_hidden():
    import torch
    from tests.gpu_util import TOL, max_rel_err, to_dev
    cfg = BASE
    p = _pair(cfg, 5)
    tree = synth.config_tree(cfg, 5)
    hid = synth.hidden(cfg, 16, 0, 5)
    before = p.kv.clone()
    empty = torch.empty((0, cfg.d_model), dtype=p.tdtype, device="cuda")
    p.gpu.tree_verify_stage(p.kv, cfg.l_glo, cfg.l_glo, empty, 0, tree.parent[:0], empty)   # no-op, returns OK
    torch.cuda.synchronize()
    assert torch.equal(before, p.kv)
    x = to_dev(hid, p.tdtype)
    p.gpu.tree_verify_stage(p.kv, cfg.l_glo, cfg.l_glo, x, 0, tree.parent[:16], x)           # hidden_out aliases hidden_in
    o = p.orc.verify(cfg.l_glo, cfg.l_glo, hid, 0, tree.parent[:16])
    assert max_rel_err(x.float().cpu().numpy(), o) < TOL["bf16"]


def test_strided_kv_cache_view():
    """Capacity padding per head and a wider token stride: only the descriptor's strides are used."""
    import torch
    from tests.gpu_util import TOL, max_rel_err, to_dev
    cfg = BASE
    p = _pair(cfg, 6)
    big = torch.zeros((cfg.n_layers, 2, cfg.n_kv_heads, p.orc.cap + 13, cfg.head_dim + 32), dtype=p.tdtype, device="cuda")
    view = big[:, :, :, : p.orc.cap, : cfg.head_dim]
    view.copy_(p.kv)
    tree = synth.config_tree(cfg, 6)
    hid = synth.hidden(cfg, 16, 0, 6)
    y = p.gpu.tree_verify_stage(view, cfg.l_glo, cfg.l_glo, to_dev(hid, p.tdtype), 0, tree.parent[:16])
    o = p.orc.verify(cfg.l_glo, cfg.l_glo, hid, 0, tree.parent[:16])
    assert max_rel_err(y.float().cpu().numpy(), o) < TOL["bf16"]
    assert float(big[..., cfg.head_dim:].abs().max()) == 0.0 and float(big[:, :, :, p.orc.cap:].abs().max()) == 0.0


def test_error_codes_with_a_live_stage():
    import torch
    from paper_2507_02620_amd import flowspec as fs
    from tests.gpu_util import to_dev
    cfg = BASE
    p = _pair(cfg, 7)
    x = to_dev(synth.hidden(cfg, 16, 0, 7), p.tdtype)
    par = synth.config_tree(cfg, 7).parent

    def code(fn):
        with pytest.raises(fs.FlowSpecError) as e:
            fn()
        return e.value.code

    assert code(lambda: p.gpu.tree_verify_stage(p.kv, cfg.l_glo, cfg.l_glo + 1, x, 0, par[:16])) == fs.FS_EINVAL   # l_cache != l_glo + seg_off
    bad = par[:16].copy(); bad[5] = 9
    assert code(lambda: p.gpu.tree_verify_stage(p.kv, cfg.l_glo, cfg.l_glo, x, 0, bad)) == fs.FS_ETOPO
    bad = par[:16].copy(); bad[0] = 0
    assert code(lambda: p.gpu.tree_verify_stage(p.kv, cfg.l_glo, cfg.l_glo, x, 0, bad)) == fs.FS_ETOPO
    far = p.orc.cap - 8
    assert code(lambda: p.gpu.tree_verify_stage(p.kv, far, far, x, 0, par[:16])) == fs.FS_ECAP                        # cache overflow
    x33 = torch.zeros((33, cfg.d_model), dtype=p.tdtype, device="cuda")
    assert code(lambda: p.gpu.tree_verify_stage(p.kv, cfg.l_glo, cfg.l_glo, x33, 0, par[:33])) == fs.FS_ECAP         # longer than max_seg
    assert code(lambda: p.gpu.tree_logits(x)) == fs.FS_EINVAL                                                          # stage has no head
    assert code(lambda: p.gpu.kv_compact(p.kv, 10, 5, [0, 1], n_acc=1)) == fs.FS_EINVAL                                # l_cache < l_glo
    assert code(lambda: p.gpu.kv_compact(p.kv, 10, 20, [3, 1], n_acc=1)) == fs.FS_EINVAL                               # not ascending
    # after all those refusals the stage still works
    y = p.gpu.tree_verify_stage(p.kv, cfg.l_glo, cfg.l_glo, x, 0, par[:16])
    torch.cuda.synchronize()
    assert torch.isfinite(y.float()).all()
