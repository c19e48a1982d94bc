"""Stochastic acceptance on the HIP path vs the oracle: every decision is an integer comparison on both sides, so the
results must agree bit for bit."""
import numpy as np
import pytest

from oracle import oracle
from paper_2507_02620_amd import synth

pytestmark = pytest.mark.gpu


def _gpu(lg, temp, token, parent, n_ver, seed, step):
    import torch
    from paper_2507_02620_amd import flowspec as fs
    T = len(token)
    res, retain, _ = fs.new_accept_buffers(T, 1)
    retain.fill_(-9)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    fs.tree_accept_sample(d(lg), temp, d(token.astype(np.int32)), d(parent.astype(np.int32)), n_ver, seed, step, res, retain)
    out, ret = fs.accept_result_to_host(res, retain, T)
    return out.as_tuple(), ret


@pytest.mark.parametrize("seed", range(16))
def test_sampled_accept_bit_exact(seed):
    rng = np.random.default_rng(seed)
    T = int(rng.choice([1, 2, 9, 64, 65, 300, 1024]))
    vocab = int(rng.choice([2, 7, 50, 1000, 32000]))
    temp = float(rng.choice([1.0, 0.5, 1.7]))
    tree = synth.random_tree(T, int(rng.choice([3, 8, 30])), int(rng.choice([0, 2, 4])), vocab, seed, forest=bool(seed % 4 == 0))
    n_ver = int(rng.integers(0, T + 1))
    lg = (synth.random_logits(max(n_ver, 1), vocab, seed, 3) * 2).astype(np.float32)
    if seed % 2:   # make long accepted paths likely
        for r, t in synth.resolve_plants(synth.plant_path(tree, n_ver, seed, 0, 0.3, 5.0), tree, vocab):
            lg[r, t] += 6.0
    inv_temp = float(np.float32(1.0) / np.float32(temp))
    print(f"[case] T={T} n_ver={n_ver} vocab={vocab} temp={temp}", flush=True)
    for step in range(6):
        o_res, o_ret = oracle.accept_sample(lg[:max(n_ver, 1)], inv_temp, tree.token, tree.parent, n_ver, 1234 + seed, step)
        g_res, g_ret = _gpu(lg[:max(n_ver, 1)], temp, tree.token, tree.parent, n_ver, 1234 + seed, step)
        assert g_res == o_res.as_tuple(), (step, g_res, o_res.as_tuple())
        assert np.array_equal(g_ret, o_ret)


def test_sampled_accept_full_vocab_residual_and_chain():
    """Qwen-sized vocabulary with no children at the root (pure residual draw), and a 1024-node verified chain."""
    lg = synth.random_logits(1, 152064, 5, 9)
    tok, par = np.array([3], dtype=np.int32), np.array([-1], dtype=np.int32)
    for step in range(8):
        o_res, _ = oracle.accept_sample(lg, 1.0, tok, par, 1, 77, step)
        g_res, _ = _gpu(lg, 1.0, tok, par, 1, 77, step)
        assert g_res == o_res.as_tuple()
    T = 1024
    chain = np.arange(-1, T - 1, dtype=np.int32)
    token = (np.arange(T, dtype=np.int32) * 7 + 3) % 50
    lg = synth.random_logits(T, 50, 6, 9)
    lg[np.arange(T - 1), token[1:]] += 12.0
    o_res, o_ret = oracle.accept_sample(lg, 1.0, token, chain, T, 5, 0)
    g_res, g_ret = _gpu(lg, 1.0, token, chain, T, 5, 0)
    assert g_res == o_res.as_tuple() and np.array_equal(g_ret, o_ret) and o_res.n_acc > 100


def test_sampled_accept_errors():
    import torch
    from paper_2507_02620_amd import flowspec as fs
    res, retain, _ = fs.new_accept_buffers(4, 1)
    t = torch.zeros(4, dtype=torch.int32, device="cuda")
    lg = torch.zeros((1, 8), device="cuda")
    with pytest.raises(fs.FlowSpecError) as e:
        fs.tree_accept_sample(lg, 0.0, t, t, 1, 0, 0, res, retain)
    assert e.value.code == fs.FS_EINVAL
    bad = torch.tensor([-1, 2, 0, 0], dtype=torch.int32, device="cuda")
    fs.tree_accept_sample(lg, 1.0, t, bad, 1, 0, 0, res, retain)
    out, _ = fs.accept_result_to_host(res, retain, 4)
    assert out.n_acc == -1
