"""HIP accept / argmax / KV compaction / segment pruning vs the oracle: integer and byte work, compared bit for bit."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2507_02620_amd import synth

pytestmark = pytest.mark.gpu


def _fs():
    from paper_2507_02620_amd import flowspec as fs
    return fs


def _i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def _gpu_accept(amax, token, parent, n_ver, logits=None):
    fs = _fs()
    T = len(token)
    res, retain, work = fs.new_accept_buffers(T, max(n_ver, 1))
    retain.fill_(-7)
    am = _i32(amax) if (n_ver > 0 and logits is None) else torch.zeros(max(n_ver, 1), dtype=torch.int32, device="cuda")
    lg = None if logits is None else torch.from_numpy(logits).cuda()
    fs.tree_accept(lg, am, _i32(token), _i32(parent), n_ver, res, retain, work)
    out, ret = fs.accept_result_to_host(res, retain, T)
    return out, ret, am.cpu().numpy()


@pytest.mark.parametrize("seed", range(25))
def test_accept_random_trees_bit_exact(seed):
    rng = np.random.default_rng(seed)
    T = int(rng.choice([1, 2, 3, 16, 63, 64, 65, 200, 256, 257, 1000, 1024]))
    vocab = int(rng.choice([3, 8, 50]))
    depth = int(rng.choice([2, 5, 12, 40]))
    tree = synth.random_tree(T, depth, int(rng.choice([0, 2, 4])), max(vocab, 2), seed, forest=bool(seed % 3 == 0))
    n_ver = int(rng.integers(0, T + 1))
    amax = rng.integers(0, vocab, max(n_ver, 1)).astype(np.int32)
    # plant a long accepted path half of the time
    if n_ver > 0 and seed % 2:
        t = synth.Tree(tree.parent, tree.token, tree.score, tree.depth)
        for row, tok in synth.resolve_plants(synth.plant_path(t, n_ver, seed, 0, 0.3, 4.0), t, max(vocab, 2)):
            amax[row] = tok
    print(f"[case] T={T} n_ver={n_ver} vocab={vocab} depth<={depth}", flush=True)
    o_res, o_ret = oracle.accept(amax, tree.token, tree.parent, n_ver)
    g_res, g_ret, _ = _gpu_accept(amax, tree.token, tree.parent, n_ver)
    assert g_res.as_tuple() == o_res.as_tuple()
    assert np.array_equal(g_ret, o_ret)


def test_accept_chain_and_star_extremes():
    T = 1024
    chain = np.arange(-1, T - 1, dtype=np.int32)
    token = np.arange(T, dtype=np.int32) + 5
    amax = token[1:].copy()                  # every node predicts its child: the whole verified chain is accepted
    for n_ver in (1, 500, 1023):
        o_res, o_ret = oracle.accept(amax[:n_ver], token, chain, n_ver)
        g_res, g_ret, _ = _gpu_accept(amax[:n_ver], token, chain, n_ver)
        assert g_res.as_tuple() == o_res.as_tuple() and np.array_equal(g_ret, o_ret)
        assert g_res.n_acc == n_ver and g_res.n_new == n_ver and g_res.n_retain == T
    star = np.full(T, 0, dtype=np.int32)
    star[0] = -1
    am = np.array([token[777]], dtype=np.int32)
    o_res, o_ret = oracle.accept(am, token, star, 1)
    g_res, g_ret, _ = _gpu_accept(am, token, star, 1)
    assert g_res.as_tuple() == o_res.as_tuple() == (1, int(token[777]), 777, 1, 2, 0)
    assert g_ret.tolist() == [0, 777]


def test_accept_reports_broken_topology_without_touching_outputs():
    parent = np.array([-1, 0, 3, 1], dtype=np.int32)
    g_res, g_ret, _ = _gpu_accept(np.zeros(2, np.int32), np.zeros(4, np.int32), parent, 2)
    assert g_res.n_acc == -1


@pytest.mark.parametrize("rows,vocab", [(1, 1), (3, 7), (16, 1024), (24, 32000), (5, 152064), (64, 32001), (70, 32000), (100, 4100)])
def test_argmax_from_logits_bit_exact_with_ties(rows, vocab):
    print(f"[case] rows={rows} vocab={vocab}", flush=True)
    lg = synth.random_logits(rows, vocab, 3, rows)
    rng = np.random.default_rng(rows)
    for r in range(rows):                    # plant exact ties of the maximum at random places
        idx = rng.integers(0, vocab, size=min(3, vocab))
        lg[r, idx] = 9.5
    if rows >= 3 and vocab >= 7:
        lg[1, :] = np.nan
        lg[2, :] = -np.inf
        lg[0, 0] = np.nan
    parent = np.arange(-1, rows - 1, dtype=np.int32)
    token = np.zeros(rows, dtype=np.int32)
    g_res, g_ret, g_amax = _gpu_accept(None, token, parent, rows, logits=lg)
    o_amax = oracle.argmax_rows(lg)
    assert np.array_equal(g_amax[:rows], o_amax)
    o_res, o_ret = oracle.accept(o_amax, token, parent, rows)
    assert g_res.as_tuple() == o_res.as_tuple() and np.array_equal(g_ret, o_ret)


def _stage_for_compact(dtype, n_layers, Hkv, hd, cap):
    fs = _fs()
    cfg = synth.StageConfig("cmp", dtype, n_layers, 64 * 2, 2 * (Hkv if Hkv > 1 else 1), Hkv, hd, 64, 0, 0, 16, 16, 4, 0)
    cfg = cfg.with_(d_model=cfg.n_q_heads * hd)
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    layers = []
    for l in range(n_layers):
        lw = synth.layer_weights(cfg, l, 0)
        layers.append({k: (None if v is None else torch.from_numpy(v).to("cuda", td)) for k, v in lw.items()})
    return fs.stage_from_config(cfg, layers, kv_capacity=cap, max_tree=1024, max_seg=16), td


@pytest.mark.parametrize("dtype,n_layers,Hkv,hd", [("bf16", 3, 4, 128), ("f32", 2, 2, 64), ("bf16", 1, 1, 64), ("f32", 1, 3, 128)])
def test_kv_compact_bit_exact(dtype, n_layers, Hkv, hd):
    fs = _fs()
    cap = 1500
    st, td = _stage_for_compact(dtype, n_layers, Hkv, hd, cap)
    rng = np.random.default_rng(7)
    npdt = np.float32 if dtype == "f32" else np.uint16
    for trial in range(12):
        l_glo = int(rng.integers(0, 300))
        n_draft = int(rng.choice([0, 1, 5, 64, 200, 1024]))
        l_cache = l_glo + n_draft
        T = min(1024, n_draft + int(rng.integers(0, 30)))
        k = int(rng.integers(0, T + 1))
        retain = np.sort(rng.choice(T, size=k, replace=False)).astype(np.int32) if T else np.zeros(0, np.int32)
        if trial % 4 == 0 and T:             # adversarial: everything shifts by exactly one slot
            retain = np.arange(1, T, dtype=np.int32)
        if trial % 4 == 1 and T:             # identity prefix then a gap
            retain = np.concatenate([np.arange(0, T // 2), np.arange(T // 2 + 1, T)]).astype(np.int32)
        n_acc = int(rng.integers(0, len(retain) + 1))
        print(f"[case] {dtype} trial={trial} l_glo={l_glo} n_draft={n_draft} |retain|={len(retain)}", flush=True)
        host = rng.integers(0, 60000, (n_layers, 2, Hkv, cap, hd)).astype(np.uint16 if npdt == np.uint16 else np.int32)
        if npdt == np.uint16:
            kv = torch.from_numpy(host.view(np.int16)).cuda().view(torch.bfloat16)
            o_cache = host.copy()
        else:
            host = host.astype(np.float32)
            kv = torch.from_numpy(host).cuda()
            o_cache = host.copy()
        o_lg, o_lc = oracle.kv_compact(o_cache, l_glo, l_cache, retain, n_acc)
        new_len = torch.zeros(2, dtype=torch.int32, device="cuda")
        if trial % 2 == 0:                   # the paper's case: the retain set arrives as a host list
            st.kv_compact(kv, l_glo, l_cache, retain, n_acc=n_acc, new_len=new_len)
        else:                                # device-resident list + result struct
            res = _i32([n_acc, 0, 0, 1, len(retain), 0])
            rd = _i32(np.concatenate([retain, np.zeros(1, np.int32)]))
            st.kv_compact(kv, l_glo, l_cache, rd, res=res, new_len=new_len)
        torch.cuda.synchronize()
        assert new_len.cpu().tolist() == [o_lg, o_lc]
        got = kv.view(torch.int16).cpu().numpy().view(np.uint16) if npdt == np.uint16 else kv.cpu().numpy()
        # slots below the new cache length are defined; above it the content is unspecified
        assert np.array_equal(got[:, :, :, :o_lc], o_cache[:, :, :, :o_lc])
        assert np.array_equal(got[:, :, :, :l_glo], host[:, :, :, :l_glo])


def test_kv_compact_strided_view():
    """The cache may be a strided view (capacity padded per head): strides travel in the descriptor."""
    fs = _fs()
    st, td = _stage_for_compact("bf16", 2, 4, 128, 300)
    big = torch.randn(2, 2, 4, 333, 160, device="cuda").to(torch.bfloat16)
    before = big.clone()
    kv = big[:, :, :, :300, :128]
    ref = kv.clone().contiguous()
    retain = np.array([0, 2, 3, 9, 40, 41], dtype=np.int32)
    st.kv_compact(kv, 100, 150, retain, n_acc=2)
    torch.cuda.synchronize()
    o = ref.view(torch.int16).cpu().numpy().copy()
    oracle.kv_compact(o, 100, 150, retain, 2)
    assert np.array_equal(kv.contiguous().view(torch.int16).cpu().numpy()[:, :, :, :106], o[:, :, :, :106])
    assert torch.equal(big[..., 128:], before[..., 128:]) and torch.equal(big[:, :, :, 300:], before[:, :, :, 300:])  # padding untouched


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_seg_prune_bit_exact(dtype):
    fs = _fs()
    rng = np.random.default_rng(11)
    for trial in range(10):
        l_s = int(rng.choice([1, 16, 24, 64]))
        d = int(rng.choice([64, 256, 4096]))
        off = int(rng.integers(0, 100))
        T = off + l_s + int(rng.integers(0, 20))
        retain = np.sort(rng.choice(T, size=int(rng.integers(0, T + 1)), replace=False)).astype(np.int32)
        seg = torch.randn(l_s, d, device="cuda").to(dtype)
        print(f"[case] trial={trial} l_s={l_s} d={d} off={off} |retain|={len(retain)}", flush=True)
        host = seg.view(torch.int16 if dtype == torch.bfloat16 else torch.int32).cpu().numpy()
        ref = oracle.seg_prune(host, off, retain)
        if trial % 2 == 0:
            out, n = fs.seg_prune(seg, off, retain)
        else:
            res = _i32([0, 0, 0, 1, len(retain), 0])
            out, n = fs.seg_prune(seg, off, _i32(np.concatenate([retain, np.zeros(1, np.int32)])), res=res)
        torch.cuda.synchronize()
        n = int(n.item())
        assert n == ref.shape[0]
        got = out.view(torch.int16 if dtype == torch.bfloat16 else torch.int32).cpu().numpy()[:n]
        assert np.array_equal(got, ref)
