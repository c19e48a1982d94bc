"""Seeded random stage shapes against the oracle: widths, head counts, group sizes, context lengths, tree sizes and segment
lengths that no hand-picked case uses (ragged everything), so that the launch plans (tiles per workgroup, KV splits, row
blocks, kernels by row count) are exercised off their tuned points."""
import numpy as np
import pytest

from paper_2507_02620_amd import synth

pytestmark = pytest.mark.gpu


def _draw(i):
    r = np.random.default_rng(7000 + i)
    dtype = "f32" if i % 4 == 3 else "bf16"
    hd = int(r.choice([64, 128]))
    n_kv = int(r.choice([1, 2, 3, 4, 6]))
    group = int(r.choice([1, 1, 2, 4, 7]))
    n_q = n_kv * group
    kt = 16 if dtype == "f32" else 32
    d_model = int(r.integers(4, 24)) * kt            # need not equal n_q * hd
    d_ffn = int(r.integers(10, 50)) * kt
    tree = int(r.integers(3, 200))
    seg = int(r.integers(1, 72))
    l_glo = int(r.choice([0, 1, int(r.integers(2, 64)), int(r.integers(64, 700)), int(r.integers(700, 2600))]))
    depth = int(r.integers(2, 40))
    branch = int(r.choice([0, 1, 2, 3, 5]))
    bias = bool(r.integers(0, 2))
    return synth.StageConfig(f"rnd{i}", dtype, int(r.integers(1, 3)), d_model, n_q, n_kv, hd, d_ffn, 0, l_glo, tree, seg, depth, branch,
                             forest=bool(i % 5 == 4), qkv_bias=bias, rms_eps=1e-6 if bias else 1e-5, rope_theta=1e6 if i % 2 else 1e4)


@pytest.mark.parametrize("i", range(16))
def test_random_stage_shape(i):
    from tests.test_gpu_parity import _check_stage
    cfg = _draw(i)
    print(f"[case] {cfg}", flush=True)
    _check_stage(cfg, 100 + i, cfg.seg_len)
