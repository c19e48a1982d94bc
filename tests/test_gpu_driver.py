"""Multi-step schedule (verify -> logits -> accept -> compact -> prune -> refill) on the HIP path vs the oracle running
the same schedule: integer traces bit-exact, stage outputs within tolerance at every step."""
import numpy as np
import pytest

from paper_2507_02620_amd import synth
from tests import driver

pytestmark = pytest.mark.gpu


def _run_both(cfg, seed, lag, steps, capacity, oracle_layers=None):
    from tests.gpu_util import TOL, Pair, max_rel_err
    p = Pair(cfg, seed, head=cfg.vocab > 0, capacity=capacity, max_tree=cfg.tree_size, max_seg=cfg.seg_len)
    sched = driver.Schedule(cfg, seed, lag, steps)
    g_trace, g_out = driver.run(driver.HipBackend(p.gpu, p.kv), sched, cfg.l_glo,
                                on_step=lambda k, t: print(f"  [hip] step {k}: T={t[0]} n_proc={t[1]} n_ver={t[2]} acc={t[3]} cont={t[6]} retain={t[7]}", flush=True))
    o_trace, o_out = driver.run(driver.OracleBackend(p.orc), sched, cfg.l_glo,
                                on_step=lambda k, t: print(f"  [oracle] step {k}", flush=True) if k % 8 == 0 else None)
    assert g_trace == o_trace
    worst = 0.0
    for k, (g, o) in enumerate(zip(g_out, o_out)):
        assert g.shape == o.shape
        if g.size:
            worst = max(worst, max_rel_err(g, o))
    print(f"  worst stage-output max-rel-err over {steps} steps: {worst:.3e}", flush=True)
    assert worst < TOL[cfg.dtype]
    # final caches agree on the valid region
    lg, lc = g_trace[-1][9], g_trace[-1][10]
    nl = p.orc.kv.shape[0]
    assert max_rel_err(p.kv[:nl, :, :, :lc].float().cpu().numpy(), p.orc.kv[:, :, :, :lc]) < TOL[cfg.dtype]
    return g_trace


SMALL = synth.StageConfig("drv-bf16", "bf16", 2, 512, 4, 2, 128, 1376, 3000, 150, 48, 16, 8, 3)


@pytest.mark.parametrize("lag", [0, 1, 2])
def test_schedule_small_bf16(lag):
    print(f"[case] {SMALL.name} lag={lag}", flush=True)
    tr = _run_both(SMALL, 5, lag, 16, capacity=600)
    assert any(t[6] for t in tr) and any(not t[6] for t in tr)


def test_schedule_tiny_fp32():
    cfg = synth.CONFIGS["C1"].with_(forest=False, max_branch=3, tree_size=24, seg_len=8)
    print(f"[case] {cfg.name} lag=1", flush=True)
    _run_both(cfg, 6, 1, 12, capacity=400)


def test_schedule_long_context_shape_32_steps():
    """The long-context stress shape (prefix 16384, 256-node trees, segments of 64, accept + compaction every step for
    32 consecutive steps) at full width, with one layer so that the oracle finishes in about a minute."""
    cfg = synth.CONFIGS["C5"].with_(n_layers=1, vocab=2048)
    print(f"[case] {cfg.name} 1 layer, 32 steps, lag=1", flush=True)
    _run_both(cfg, 0, 1, 32, capacity=cfg.l_glo + 32 * 16 + 2 * cfg.tree_size)
