"""The long-context stress configuration as written: LLaMA2-7B-shaped 8-layer last stage with its 32 000-entry head, KV
prefix 16384, 256-node trees in segments of 64, accept + KV compaction on every one of 32 consecutive steps (Sec. III-C state
machine), as the last stage (lag 0) and as the stage before it (lag 1).

The integer trace of every step (tree size, verified prefix, accept tuple, new l_glo / l_cache, pruned segment length, retain
list) must equal the free-running oracle's; accept and compaction are also checked bit for bit inside every step; the
forward, the appended K/V and the logits are compared with the oracle at sampled steps (first, middle, last), the oracle's
cache brought to the HIP path's state before each of them."""
import time

import numpy as np
import pytest

from paper_2507_02620_amd import synth
from tests import driver

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("lag,samples", [(0, (0, 13, 31)), (1, (0, 17, 31))])
def test_c5_as_written_32_steps(lag, samples):
    import torch
    from tests.gpu_util import TOL, Pair
    cfg = synth.CONFIGS["C5"]
    steps = 32
    t0 = time.time()
    cap = cfg.l_glo + steps * 16 + (2 + lag) * cfg.tree_size
    print(f"[case] {cfg.name}: {cfg.n_layers} layers, vocab {cfg.vocab}, {steps} steps, lag {lag}, capacity {cap}", flush=True)
    p = Pair(cfg, 0, head=True, capacity=cap, max_tree=cfg.tree_size, max_seg=cfg.seg_len)
    print(f"  stage + oracle ready after {time.time() - t0:.1f} s", flush=True)
    prefix0 = p.kv[:, :, :, : cfg.l_glo].clone()
    sched = driver.Schedule(cfg, 0, lag, steps, closed=True)
    hip = driver.CheckedHipBackend(p.gpu, p.kv, p.orc, cfg.l_glo, samples, TOL[cfg.dtype], log=lambda m: print(m, flush=True))
    g_trace, _ = driver.run(hip, sched, cfg.l_glo,
                            on_step=lambda k, t: print(f"  [hip] step {k}: T={t[0]} n_proc={t[1]} n_ver={t[2]} acc={t[3]} cont={t[6]} retain={t[7]} "
                                                       f"l_glo'={t[9]} l_cache'={t[10]} ({time.time() - t0:.0f} s)", flush=True))
    o_trace, _ = driver.run(driver.IntegerOracleBackend(cfg, cap), sched, cfg.l_glo)
    assert g_trace == o_trace
    assert sorted(hip.checked_steps) == sorted(samples)
    assert any(t[6] for t in g_trace) and any(not t[6] for t in g_trace)         # continuing and broken rounds both occur
    assert g_trace[-1][9] > cfg.l_glo + steps                                     # the context grew by at least a token per step
    assert torch.equal(p.kv[:, :, :, : cfg.l_glo], prefix0)                      # the prompt's K/V: untouched, bit for bit
    print(f"  worst over sampled steps {sorted(samples)}: {hip.worst}; done in {time.time() - t0:.0f} s", flush=True)
