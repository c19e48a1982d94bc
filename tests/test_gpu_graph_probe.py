"""HIP-graph capture of the stage's launches, and the measurement-aid probes."""
import numpy as np
import pytest

from paper_2507_02620_amd import synth

pytestmark = pytest.mark.gpu


def test_verify_and_logits_replay_from_a_graph():
    """Every launch of verify + logits + accept + compaction is capturable (trees travel as kernel arguments, nothing is
    allocated or cleared by memset): three replays, with eager work and synchronisations in between, each reproduce the
    eager results bit for bit."""
    import torch
    from paper_2507_02620_amd import flowspec as fs
    from tests.gpu_util import Pair, to_dev
    cfg = synth.StageConfig("graph", "bf16", 2, 512, 4, 2, 128, 1408, 1000, 96, 40, 16, 5, 3)
    print(f"[case] {cfg.name}", flush=True)
    pair = Pair(cfg, seed=9, head=True)
    tree = synth.config_tree(cfg, seed=9)
    T, dev = tree.size, "cuda"
    hid = to_dev(synth.hidden(cfg, T, 0, 9), torch.bfloat16)
    segs = synth.segments(T, cfg.seg_len)
    outs = [torch.empty_like(hid[o:o + n]) for o, n in segs]
    logits = torch.zeros((T, cfg.vocab), dtype=torch.float32, device=dev)
    amax = torch.zeros(T, dtype=torch.int32, device=dev)
    token_d, parent_d = torch.from_numpy(tree.token).to(dev), torch.from_numpy(tree.parent).to(dev)
    res, retain, work = fs.new_accept_buffers(T, T, dev)
    kv0 = pair.kv.clone()

    def step(stream=None):
        for i, (off, n) in enumerate(segs):
            pair.gpu.tree_verify_stage(pair.kv, cfg.l_glo, cfg.l_glo + off, hid[off:off + n], off, tree.parent[: off + n], outs[i], stream=stream)
            pair.gpu.tree_logits(outs[i], logits[off:off + n], amax[off:off + n], stream=stream)
        fs.tree_accept(logits, amax, token_d, parent_d, T, res, retain, work, stream=stream)
        pair.gpu.kv_compact(pair.kv, cfg.l_glo, cfg.l_glo + T, retain, res=res, stream=stream)

    step()
    torch.cuda.synchronize()
    want = [o.clone() for o in outs] + [logits.clone(), amax.clone(), res.clone(), retain.clone(), pair.kv.clone()]

    pair.kv.copy_(kv0)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(stream=torch.cuda.current_stream())
    for rep in range(3):
        # eager work between the replays: restore the cache, scribble over the outputs
        pair.kv.copy_(kv0)
        for o in outs:
            o.zero_()
        logits.fill_(-1.0)
        amax.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = outs + [logits, amax, res, retain, pair.kv]
        for k, (g, w) in enumerate(zip(got, want)):
            assert torch.equal(g, w), f"replay {rep}: tensor {k} differs from the eager run"


def test_probes_report_plausible_rates():
    import torch
    from paper_2507_02620_amd import flowspec as fs
    buf = torch.empty((1 << 30) + 64, dtype=torch.uint8, device="cuda")
    gbs = fs.probe_stream_read(buf, 64 << 20, 5)
    tf = fs.probe_mfma_bf16(buf, 2)
    print(f"  stream read {gbs:.0f} GB/s, bf16 MFMA loop {tf:.0f} TFLOP/s", flush=True)
    assert 500.0 < gbs < 8000.0 * 1.05      # below the datasheet HBM peak (within timer noise), above any plausible floor
    assert 200.0 < tf < 2500.0 * 1.05
    with pytest.raises(fs.FlowSpecError):
        fs.probe_stream_read(buf, (64 << 20) + 4096, 1)   # not a multiple of 256 KiB
