"""LM head + row argmax of the HIP path vs the oracle."""
import numpy as np
import pytest

from paper_2507_02620_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg,rows", [
    (synth.CONFIGS["C1"], 16),
    (synth.StageConfig("lg-bf16", "bf16", 1, 512, 4, 4, 128, 1376, 32000, 8, 16, 24, 4, 3), 24),
    (synth.StageConfig("lg-bf16-odd-vocab", "bf16", 1, 1024, 8, 2, 128, 1376, 50257, 8, 16, 64, 4, 3), 64),
    (synth.StageConfig("lg-f32", "f32", 1, 256, 4, 4, 64, 688, 1000, 8, 16, 5, 4, 3), 5),
    # LM head through the many-row kernel: one 64-row block (40 rows), one partly filled 128-row block with padding tiles (100 rows)
    (synth.StageConfig("lg-bf16-40", "bf16", 1, 512, 4, 4, 128, 1376, 32000, 8, 16, 40, 4, 3), 40),
    (synth.StageConfig("lg-bf16-100-odd-vocab", "bf16", 1, 1024, 8, 2, 128, 1376, 50257, 8, 16, 100, 4, 3), 100),
])
def test_logits_and_argmax(cfg, rows):
    import torch
    from tests.gpu_util import TOL, Pair, max_rel_err, to_dev
    print(f"[case] {cfg.name} rows={rows} vocab={cfg.vocab}", flush=True)
    p = Pair(cfg, 3, head=True)
    hid = synth.hidden(cfg, rows, 7, 3)
    o_lg, o_am = p.orc.logits(hid.astype(np.float64))
    g_lg, g_am = p.gpu.tree_logits(to_dev(hid, p.tdtype))
    torch.cuda.synchronize()
    g_lg, g_am = g_lg.cpu().numpy(), g_am.cpu().numpy()
    err = max_rel_err(g_lg, o_lg)
    print(f"  logits max-rel-err {err:.3e}", flush=True)
    assert err < TOL[cfg.dtype]
    # the device argmax is exact for the device's own fp32 logits (lowest index on ties) ...
    assert np.array_equal(g_am, np.argmax(g_lg, axis=1))
    # ... and agrees with the oracle wherever the oracle's top-2 gap exceeds the numerical error bound
    top2 = np.sort(o_lg, axis=1)[:, -2:]
    clear = (top2[:, 1] - top2[:, 0]) > 2 * TOL[cfg.dtype] * np.abs(o_lg).max()
    assert np.array_equal(g_am[clear], o_am[clear])
    # elsewhere the chosen entry must be within the bound of the oracle's maximum
    for r in np.nonzero(~clear)[0]:
        assert o_lg[r, g_am[r]] >= top2[r, 1] - 2 * TOL[cfg.dtype] * np.abs(o_lg).max()
