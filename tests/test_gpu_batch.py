"""Batched verification (several requests through one stage call, Sec. III-A's stage serving more than one request):
each request's rows against the oracle run on that request alone."""
import numpy as np
import pytest

from paper_2507_02620_amd import synth

pytestmark = pytest.mark.gpu


def _run_batch(cfg, specs, seed, head=False, w4=False):
    """specs: list of (l_glo, tree_size, max_depth, max_branch, seg_off, l_s).  Every request gets its own cache, tree and
    context; segments before seg_off are verified one request at a time first (they fill the cache)."""
    import torch
    from oracle import oracle
    from paper_2507_02620_amd import flowspec as fs
    from tests.gpu_util import Pair, to_dev
    pair = Pair(cfg, seed=seed, head=head, w4=w4)   # weights + one oracle stage (its cache is reloaded per request)
    tdt = pair.tdtype
    items, hid_rows, want = [], [], []
    caches = []
    for r, (l_glo, T, depth, branch, seg_off, l_s) in enumerate(specs):
        tree = synth.random_tree(T, depth, branch, 1000, seed, stream=10 + r)
        hid = synth.hidden(cfg, T, 20 + r, seed)
        kv = pair.gpu.new_kv_cache()
        orc = oracle.Stage(cfg, [oracle.dequant_layer(lw) for lw in pair.layers] if w4 else pair.layers, None, None, cfg.kv_capacity)
        for l in range(cfg.n_layers):
            pre = synth.prefix_kv(cfg, l, cfg.kv_capacity, seed + 100 * r)
            pre[:, :, l_glo:] = 0
            orc.load_prefix(l, pre)
            kv[l].copy_(to_dev(pre, tdt))
        # earlier rows of this request's S, one call per request
        if seg_off:
            orc.verify(l_glo, l_glo, hid[:seg_off], 0, tree.parent[:seg_off])
            pair.gpu.tree_verify_stage(kv, l_glo, l_glo, to_dev(hid[:seg_off], tdt), 0, tree.parent[:seg_off])
        want.append(orc.verify(l_glo, l_glo + seg_off, hid[seg_off:seg_off + l_s], seg_off, tree.parent[:seg_off + l_s]))
        items.append((kv, l_glo, l_glo + seg_off, seg_off, l_s, tree.parent[:seg_off + l_s]))
        hid_rows.append(hid[seg_off:seg_off + l_s])
        caches.append((kv, orc, l_glo, seg_off, l_s))
    stacked = to_dev(np.concatenate(hid_rows, axis=0), tdt)
    out = pair.gpu.tree_verify_batch(items, stacked)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), want, caches, cfg


@pytest.mark.parametrize("name,cfg,specs", [
    ("few-rows", synth.StageConfig("b-small", "bf16", 2, 512, 8, 2, 64, 1408, 0, 0, 64, 16, 6, 3, qkv_bias=True),
     [(50, 40, 6, 3, 16, 16), (0, 20, 4, 2, 0, 9), (130, 64, 8, 0, 32, 16), (77, 33, 5, 3, 16, 17)]),
    ("many-rows", synth.StageConfig("b-wide", "bf16", 2, 512, 4, 4, 128, 1408, 0, 0, 64, 16, 6, 3),
     [(100 + 13 * i, 48, 6, 3, 16, 16) for i in range(10)]),           # 160 stacked rows: the MFMA-bound projection kernel
    # one KV head under 8 query heads, long contexts: row blocks of four one-tile waves; the shorter request has no third row block
    ("wide-group-long-context", synth.StageConfig("b-gqa", "bf16", 1, 1024, 8, 1, 128, 1408, 0, 0, 64, 16, 6, 3),
     [(2100, 40, 6, 3, 16, 20), (1500, 30, 5, 3, 16, 12)]),
    # 16 requests x 32 KV heads = 512 attention workgroups of 7 K/V tiles each: the plan's direct-to-LDS kernel with two tile buffers
    ("many-heads-direct-to-lds", synth.StageConfig("b-dma", "bf16", 1, 512, 32, 32, 128, 1408, 0, 0, 64, 16, 6, 3),
     [(400 + 7 * i, 32, 5, 3, 16, 16) for i in range(16)]),
    ("f32", synth.StageConfig("b-f32", "f32", 1, 256, 4, 4, 64, 688, 0, 0, 64, 16, 5, 3),
     [(30, 24, 5, 3, 8, 8), (64, 16, 4, 2, 0, 16), (5, 40, 6, 3, 24, 16)]),
])
def test_batch_matches_per_request_oracle(name, cfg, specs):
    from tests.gpu_util import TOL, max_rel_err
    print(f"[case] batch {name}: {len(specs)} requests, {sum(s[5] for s in specs)} stacked rows", flush=True)
    cfg = cfg.with_(l_glo=max(s[0] for s in specs), tree_size=max(s[1] for s in specs))
    got, want, caches, cfg = _run_batch(cfg.with_(seg_len=max(64, sum(s[5] for s in specs))), specs, seed=12)
    row = 0
    for r, w in enumerate(want):
        n = w.shape[0]
        err = max_rel_err(got[row:row + n], w)
        print(f"  request {r}: {n} rows, hidden max-rel-err {err:.3e}", flush=True)
        assert err < TOL[cfg.dtype]
        row += n
    # the K/V rows of every request landed in that request's own cache
    for kv, orc, l_glo, seg_off, l_s in caches:
        l = cfg.n_layers - 1
        g = kv[l][:, :, l_glo + seg_off:l_glo + seg_off + l_s].float().cpu().numpy()
        o = orc.kv[l][:, :, l_glo + seg_off:l_glo + seg_off + l_s]
        assert max_rel_err(g, o) < TOL[cfg.dtype]


def test_batch_with_4bit_weights():
    """The batch path with 4-bit group weights (gains applied by the producing epilogue, row blocks of the few-row kernel)."""
    from tests.gpu_util import TOL, max_rel_err
    cfg = synth.StageConfig("b-w4", "bf16", 2, 512, 4, 2, 128, 1408, 0, 120, 48, 80, 6, 3)
    specs = [(60 + 20 * i, 48, 6, 3, 16, 16) for i in range(5)]       # 80 stacked rows
    print(f"[case] batch w4: {len(specs)} requests, 80 stacked rows", flush=True)
    got, want, caches, cfg = _run_batch(cfg, specs, seed=21, w4=True)
    row = 0
    for r, w in enumerate(want):
        n = w.shape[0]
        err = max_rel_err(got[row:row + n], w)
        print(f"  request {r}: hidden max-rel-err {err:.3e}", flush=True)
        assert err < TOL["bf16"]
        row += n


def test_batch_errors():
    import torch
    from paper_2507_02620_amd import flowspec as fs
    from tests.gpu_util import Pair, to_dev
    cfg = synth.StageConfig("b-err", "bf16", 1, 256, 4, 4, 64, 512, 0, 16, 32, 16, 4, 2)
    pair = Pair(cfg, seed=1)
    kv = pair.gpu.new_kv_cache()
    par = np.array([-1, 0, 0, 1], dtype=np.int32)
    hid = to_dev(synth.hidden(cfg, 8, 0, 1), torch.bfloat16)
    ok = (kv, 16, 16, 0, 4, par)
    pair.gpu.tree_verify_batch([ok, ok], hid)                                  # fine (two requests may even share a cache object here)
    with pytest.raises(fs.FlowSpecError) as e:
        pair.gpu.tree_verify_batch([ok, (kv, 16, 17, 0, 4, par)], hid)          # l_cache != l_glo + seg_off
    assert e.value.code == fs.FS_EINVAL
    with pytest.raises(fs.FlowSpecError) as e:
        pair.gpu.tree_verify_batch([ok, (kv, 16, 16, 0, 4, np.array([-1, 2, 0, 1], dtype=np.int32))], hid)
    assert e.value.code == fs.FS_ETOPO
    with pytest.raises(fs.FlowSpecError) as e:
        pair.gpu.tree_verify_batch([ok] * 5, to_dev(synth.hidden(cfg, 20, 0, 1), torch.bfloat16))   # 20 stacked rows > max_seg 16
    assert e.value.code == fs.FS_ECAP
    other = kv[:, :, :, ::2]                                                  # different token stride
    with pytest.raises(fs.FlowSpecError) as e:
        pair.gpu.tree_verify_batch([ok, (other, 0, 0, 0, 4, par)], hid)
    assert e.value.code == fs.FS_EINVAL


def _random_batch(i):
    r = np.random.default_rng(9100 + i)
    hd = int(r.choice([64, 128]))
    n_kv = int(r.choice([1, 2, 4]))
    n_q = n_kv * int(r.choice([1, 2, 4]))
    dtype = "f32" if i % 3 == 2 else "bf16"
    kt = 16 if dtype == "f32" else 32
    cfg = synth.StageConfig(f"b-rnd{i}", dtype, int(r.integers(1, 3)), int(r.integers(6, 20)) * kt, n_q, n_kv, hd, int(r.integers(10, 40)) * kt,
                            0, 0, 64, 16, 6, 3, qkv_bias=bool(i % 2))
    specs = []
    for _ in range(int(r.integers(2, 7))):
        T = int(r.integers(2, 90))
        seg_off = int(r.integers(0, T))
        specs.append((int(r.choice([0, 3, int(r.integers(4, 900))])), T, int(r.integers(2, 12)), int(r.choice([0, 2, 3])), seg_off,
                      int(r.integers(1, min(40, T - seg_off) + 1))))
    return cfg, specs


@pytest.mark.parametrize("i", range(8))
def test_random_batches(i):
    """Seeded random batches: 2 to 6 requests of unrelated context lengths, tree sizes, segment offsets and segment lengths."""
    from tests.gpu_util import TOL, max_rel_err
    cfg, specs = _random_batch(i)
    print(f"[case] random batch {i}: {cfg.dtype} heads {cfg.n_q_heads}/{cfg.n_kv_heads} x {cfg.head_dim}, specs {specs}", flush=True)
    cfg = cfg.with_(l_glo=max(s[0] for s in specs), tree_size=max(s[1] for s in specs))
    # the rows before a request's segment are verified in one call of their own: the stage must take that many rows too
    got, want, caches, cfg = _run_batch(cfg.with_(seg_len=max(64, sum(s[5] for s in specs), max(s[4] for s in specs))), specs, seed=40 + i)
    row = 0
    for rq, w in enumerate(want):
        n = w.shape[0]
        err = max_rel_err(got[row:row + n], w)
        print(f"  request {rq}: {n} rows, hidden max-rel-err {err:.3e}", flush=True)
        assert err < TOL[cfg.dtype]
        row += n
    for kv, orc, l_glo, seg_off, l_s in caches:
        for l in range(cfg.n_layers):
            g = kv[l][:, :, l_glo + seg_off:l_glo + seg_off + l_s].float().cpu().numpy()
            assert max_rel_err(g, orc.kv[l][:, :, l_glo + seg_off:l_glo + seg_off + l_s]) < TOL[cfg.dtype]
