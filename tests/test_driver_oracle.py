"""The multi-step schedule run on the oracle alone: state-machine invariants over many steps.  CPU only."""
import numpy as np
import pytest

from paper_2507_02620_amd import synth
from tests import driver
from tests.helpers import TINY, make_oracle_stage


@pytest.mark.parametrize("lag", [0, 1, 2])
def test_schedule_invariants(lag):
    cfg = TINY.with_(tree_size=20, seg_len=4, l_glo=6, vocab=64, max_branch=3)
    st, *_ = make_oracle_stage(cfg, 4, capacity=400, head=True)
    sched = driver.Schedule(cfg, 4, lag, 24)
    seen = []
    trace, outs = driver.run(driver.OracleBackend(st), sched, cfg.l_glo, on_step=lambda k, t: seen.append(t))
    l_glo = cfg.l_glo
    n_cont = 0
    for t in trace:
        T, n_proc, n_ver, n_acc, x_new, n_new, cont, n_retain, n_prv, lg, lc, n_local = t[:12]
        retain = np.array(t[12:])
        assert n_acc >= 1 and lg == l_glo + n_acc            # l_glo grows by |S_acc|
        assert n_prv == 0                                     # a real accept leaves no verified draft node
        assert lc - lg == int(((retain[n_acc:]) < n_proc).sum())
        if lag == 0:
            assert lc == lg                                   # last stage: compacted cache == accepted path
        l_glo = lg
        n_cont += cont
    assert 0 < n_cont < len(trace)                            # both continuing and ending rounds occur
    assert any(t[2] > 0 and t[11] > 0 for t in trace) or lag == 0
