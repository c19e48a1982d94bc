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


@pytest.mark.parametrize("n_req", [3, 6])
def test_batched_verify_replays_from_a_graph(n_req):
    """The batched forward under capture: 3 requests x 16 rows take the few-row kernel plus the one-block many-row route for
    gate/up and the down projection, 6 x 16 rows the many-row kernel with K slices and the fix-up pass.  Three replays with
    eager work in between reproduce the eager hidden states and caches bit for bit."""
    import torch
    from paper_2507_02620_amd import flowspec as fs
    from tests.gpu_util import to_dev
    cfg = synth.StageConfig("graph-batch", "bf16", 2, 512, 4, 2, 128, 1408, 0, 90, 16, 16, 5, 3)
    print(f"[case] {cfg.name} requests={n_req}", flush=True)
    dev = "cuda"
    layers = [{k: (None if v is None else to_dev(v, torch.bfloat16)) for k, v in synth.layer_weights(cfg, l, 11).items()}
              for l in range(cfg.n_layers)]
    stage = fs.stage_from_config(cfg, layers, max_seg=n_req * cfg.seg_len)
    kvs, trees = [], []
    for r in range(n_req):
        kv = stage.new_kv_cache()
        for l in range(cfg.n_layers):
            kv[l, :, :, : cfg.l_glo] = to_dev(synth.prefix_kv(cfg, l, cfg.kv_capacity, 11 + r)[:, :, : cfg.l_glo], torch.bfloat16)
        kvs.append(kv)
        trees.append(synth.random_tree(cfg.tree_size, cfg.max_depth, cfg.max_branch, 1000, 11, stream=r))
    hid = torch.cat([to_dev(synth.hidden(cfg, cfg.tree_size, r, 11), torch.bfloat16) for r in range(n_req)], dim=0).contiguous()
    out = torch.empty_like(hid)
    kv0 = [kv.clone() for kv in kvs]
    items = [(kvs[r], cfg.l_glo, cfg.l_glo, 0, cfg.tree_size, trees[r].parent) for r in range(n_req)]

    stage.tree_verify_batch(items, hid, out)
    torch.cuda.synchronize()
    want = [out.clone()] + [kv.clone() for kv in kvs]

    for kv, k0 in zip(kvs, kv0):
        kv.copy_(k0)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        stage.tree_verify_batch(items, hid, out, stream=torch.cuda.current_stream())
    for rep in range(3):
        for kv, k0 in zip(kvs, kv0):
            kv.copy_(k0)
        out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, (g, w) in enumerate(zip([out] + kvs, want)):
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
