"""Chunked-prefill shape through the verification stage (Sec. III-A: the prompt passes through the same pipeline stages):
a chain "tree" of hundreds of rows in one segment.  Same oracle, same tolerances as the tree-shaped cases."""
import numpy as np
import pytest

from paper_2507_02620_amd import synth

pytestmark = pytest.mark.gpu


def _chain(n):
    return np.arange(-1, n - 1, dtype=np.int32)


@pytest.mark.parametrize("cfg,rows", [
    (synth.StageConfig("pf-bf16-gqa", "bf16", 2, 512, 8, 2, 64, 1408, 0, 200, 300, 300, 300, 1, qkv_bias=True), 300),
    (synth.StageConfig("pf-bf16-mha128", "bf16", 1, 1024, 8, 8, 128, 2816, 0, 77, 512, 512, 512, 1), 512),
    (synth.StageConfig("pf-f32", "f32", 1, 256, 4, 4, 64, 688, 0, 50, 130, 130, 130, 1), 130),
    (synth.StageConfig("pf-bf16-1024", "bf16", 1, 512, 4, 4, 128, 1024, 0, 0, 1024, 1024, 1024, 1), 1024),
    # feature counts that are not multiples of a workgroup's 256 features: padding tiles in every epilogue and in the K-split fix-up
    (synth.StageConfig("pf-bf16-odd-widths", "bf16", 2, 480, 6, 3, 64, 1056, 0, 33, 150, 150, 150, 1, qkv_bias=True), 150),
    # one partly filled row block of the many-row kernel (65 .. 127 rows), K slices for the residual projections
    (synth.StageConfig("pf-bf16-96", "bf16", 2, 1024, 8, 8, 128, 2816, 0, 60, 96, 96, 96, 1), 96),
    (synth.StageConfig("pf-bf16-81-gqa", "bf16", 2, 512, 8, 2, 64, 1408, 0, 100, 81, 81, 81, 1, qkv_bias=True), 81),
    # 17 .. 64 rows: gate/up and down projection through one 64-row block, the rest through the few-row kernel
    (synth.StageConfig("pf-bf16-50", "bf16", 2, 1024, 8, 8, 128, 2816, 0, 60, 50, 50, 50, 1), 50),
    (synth.StageConfig("pf-bf16-20-odd-widths", "bf16", 2, 480, 6, 3, 64, 1056, 0, 33, 20, 20, 20, 1, qkv_bias=True), 20),
])
def test_chain_segment(cfg, rows):
    from tests.gpu_util import TOL, Pair, max_rel_err
    print(f"[case] {cfg.name} rows={rows} l_glo={cfg.l_glo}", flush=True)
    pair = Pair(cfg, seed=4)
    hid = synth.hidden(cfg, rows, 0, 4)
    o, g = pair.verify_tree(_chain(rows), hid, rows)
    err = max_rel_err(g, o)
    print(f"  hidden max-rel-err {err:.3e}", flush=True)
    assert err < TOL[cfg.dtype]
    # appended K/V of the last layer
    l = cfg.n_layers - 1
    kv_g = pair.kv[l][:, :, cfg.l_glo:cfg.l_glo + rows].float().cpu().numpy()
    kv_o = pair.orc.kv[l][:, :, cfg.l_glo:cfg.l_glo + rows]
    assert max_rel_err(kv_g, kv_o) < TOL[cfg.dtype]


@pytest.mark.parametrize("cfg,rows,head", [
    # the 256-row projection kernel (both operands through LDS) forced on for every normed projection: QKV with bias and
    # rotation, gate/up and the LM head, with row counts that leave the last 256-row block partly filled and feature counts
    # that leave the last 256-feature (or 192-feature) block partly filled
    (synth.StageConfig("blk-bf16-gqa-400", "bf16", 2, 512, 8, 2, 64, 1408, 1000, 90, 400, 400, 400, 1, qkv_bias=True), 400, True),
    (synth.StageConfig("blk-bf16-mha128-640", "bf16", 1, 1024, 8, 8, 128, 2816, 0, 77, 640, 640, 640, 1), 640, False),
    (synth.StageConfig("blk-bf16-1024", "bf16", 1, 512, 4, 4, 128, 1024, 0, 0, 1024, 1024, 1024, 1), 1024, False),
])
@pytest.mark.parametrize("width", [1, 2])   # knob values: blocks of 256 features (16 tiles) / of 192 features (12 tiles)
def test_chain_segment_through_the_256_row_kernel(cfg, rows, head, width, monkeypatch):
    from tests.gpu_util import TOL, Pair, max_rel_err
    monkeypatch.setenv("FLOWSPEC_BLOCK_GEMM", str(width))
    print(f"[case] {cfg.name} rows={rows} block width knob {width}", flush=True)
    pair = Pair(cfg, seed=5, head=head)
    hid = synth.hidden(cfg, rows, 0, 5)
    o, g = pair.verify_tree(_chain(rows), hid, rows)
    err = max_rel_err(g, o)
    print(f"  hidden max-rel-err {err:.3e}", flush=True)
    assert err < TOL[cfg.dtype]
    kv_g = pair.kv[:, :, :, cfg.l_glo:cfg.l_glo + rows].float().cpu().numpy()
    assert max_rel_err(kv_g, pair.orc.kv[:, :, :, cfg.l_glo:cfg.l_glo + rows]) < TOL[cfg.dtype]
    if head:
        import torch
        o_lg, _ = pair.orc.logits(o)
        g_lg, _ = pair.gpu.tree_logits(torch.from_numpy(g).to("cuda", pair.tdtype))
        lerr = max_rel_err(g_lg.cpu().numpy(), o_lg)
        print(f"  logits max-rel-err {lerr:.3e}", flush=True)
        assert lerr < TOL[cfg.dtype]


def test_chain_in_two_chunks_matches_one():
    """A 400-row chain verified as 256 + 144 rows gives the rows of the single 400-row pass (bf16 level)."""
    from tests.gpu_util import TOL, Pair, max_rel_err
    cfg = synth.StageConfig("pf-split", "bf16", 2, 512, 4, 4, 128, 1408, 0, 100, 400, 256, 400, 1)
    print(f"[case] {cfg.name}", flush=True)
    pair = Pair(cfg, seed=6)
    hid = synth.hidden(cfg, 400, 0, 6)
    o, g = pair.verify_tree(_chain(400), hid, 256)
    assert max_rel_err(g, o) < TOL["bf16"]


def test_chain_at_bench_width():
    """Workload P1's layer shape and row count (512-row chain behind a 1024-token prefix, d_model 4096, FFN 11008) through one
    layer, in the launch configuration bench.py times: every output row against the oracle."""
    from tests.gpu_util import TOL, Pair, max_rel_err
    cfg = synth.CONFIGS["P1"].with_(n_layers=1)
    print(f"[case] {cfg.name} 1 layer rows={cfg.tree_size}", flush=True)
    pair = Pair(cfg, seed=0)
    hid = synth.hidden(cfg, cfg.tree_size, 0, 0)
    o, g = pair.verify_tree(_chain(cfg.tree_size), hid, cfg.seg_len)
    err = max_rel_err(g, o)
    print(f"  hidden max-rel-err {err:.3e}", flush=True)
    assert err < TOL["bf16"]
