"""The entry point that allocates nothing (fs_tree_accept_noalloc: scratch in a static device array) against
fs_tree_accept on the same inputs, through the C ABI: two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

from paper_2507_02620_amd import synth

pytestmark = pytest.mark.gpu


def _both(T, n_ver, vocab, seed):
    import torch
    from paper_2507_02620_amd import flowspec as fs
    tree = synth.random_tree(T, 8, 3, vocab, seed)
    lg = synth.random_logits(n_ver, vocab, seed, 3)
    for row, tok in synth.resolve_plants(synth.plant_path(tree, n_ver, seed, 0, 0.0, 3.0), tree, vocab):
        lg[row, tok] += 100.0
    lg_d = torch.from_numpy(lg).cuda()
    tok_d, par_d = torch.from_numpy(tree.token).cuda(), torch.from_numpy(tree.parent).cuda()
    res_a, ret_a, work = fs.new_accept_buffers(T, n_ver)
    am_a = torch.full((n_ver,), -7, dtype=torch.int32, device="cuda")
    fs.tree_accept(lg_d, am_a, tok_d, par_d, n_ver, res_a, ret_a, work)
    res_b, ret_b, _ = fs.new_accept_buffers(T, n_ver)
    am_b = torch.full((n_ver,), -9, dtype=torch.int32, device="cuda")
    print(f"[case] noalloc T={T} n_ver={n_ver} vocab={vocab}", flush=True)
    fs.tree_accept_noalloc(lg_d, am_b, tok_d, par_d, n_ver, res_b, ret_b)
    a, ra = fs.accept_result_to_host(res_a, ret_a, T)
    b, rb = fs.accept_result_to_host(res_b, ret_b, T)
    assert torch.equal(am_a, am_b)
    assert a.as_tuple() == b.as_tuple() and np.array_equal(ra, rb)
    assert a.n_acc >= 1
    return a.as_tuple()


def test_noalloc_accept_matches_accept_twice_in_a_row_second_call_smaller():
    first = _both(200, 48, 32000, 11)     # 48 rows: the two-pass argmax, whose partial maxima live in the static array
    second = _both(40, 16, 1000, 12)      # smaller tree, fewer rows, smaller vocabulary: stale partials must not matter
    third = _both(300, 300, 5000, 13)     # 64 rows and more take the single-pass argmax (no scratch at all)
    print("  results:", first, second, third, flush=True)


def test_noalloc_rejects_sizes_beyond_its_scratch():
    import torch
    from paper_2507_02620_amd import flowspec as fs
    tok = torch.zeros(2000, dtype=torch.int32, device="cuda")
    res, ret, _ = fs.new_accept_buffers(2000, 1)
    with pytest.raises(fs.FlowSpecError) as e:
        fs.tree_accept_noalloc(None, tok, tok, tok, 1, res, ret)
    assert e.value.code == fs.FS_ECAP
