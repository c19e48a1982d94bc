"""Multi-step state machine of one verification stage (harness logic only): verify segments, take last-stage
outputs, plant acceptance, accept, prune cache / in-flight segment / tree, refill the tree.

Two back ends run the same schedule: the oracle and the HIP library.  `lag` emulates stage V(N - lag): the stage
has processed `lag` segments more than have been verified when a retain set arrives, so its cache holds draft
K/V beyond the verified prefix and I_incache / I_local are non-trivial.  lag = 0 is the last stage: it produces
the logits itself (LM head), and acceptance runs on them after planting.
"""
import numpy as np

from oracle import oracle
from paper_2507_02620_amd import synth

PLANT = 100.0


class Schedule:
    """Everything both back ends must agree on, drawn from the seed: trees, hidden inputs, plants."""

    def __init__(self, cfg, seed, lag, steps):
        self.cfg, self.seed, self.lag, self.steps = cfg, seed, lag, steps

    def fresh_tree(self, k):
        t = synth.random_tree(self.cfg.tree_size, self.cfg.max_depth, self.cfg.max_branch, max(self.cfg.vocab, 2), self.seed, stream=1000 + k)
        return t.parent, t.token

    def hidden_rows(self, n, k):
        return synth.hidden(self.cfg, n, call=100 + k, seed=self.seed)

    def plants(self, parent, token, n_ver, k):
        t = synth.Tree(parent, token, np.zeros(len(parent)), synth._depths(parent))
        return synth.resolve_plants(synth.plant_path(t, n_ver, self.seed, k, p_stop=0.2, mean_extra=1.0), t, max(self.cfg.vocab, 2))

    def synthetic_amax(self, n, k):
        return np.random.default_rng(self.seed * 7919 + k).integers(0, max(self.cfg.vocab, 2), n).astype(np.int32)


class OracleBackend:
    name = "oracle"

    def __init__(self, stage):
        self.st = stage

    def verify(self, l_glo, l_cache, hid, seg_off, parent):
        return self.st.verify(l_glo, l_cache, hid, seg_off, parent)

    def logits_amax(self, rows):
        return self.st.logits(rows)

    def accept(self, lg, amax, token, parent, n_ver):
        if lg is not None:
            amax = oracle.argmax_rows(lg)
        res, retain = oracle.accept(amax, token, parent, n_ver)
        return res.as_tuple(), retain

    def compact(self, l_glo, l_cache, retain, n_acc):
        return oracle.kv_compact(self.st.kv, l_glo, l_cache, retain, n_acc)

    def seg_prune(self, seg, off, retain):
        return oracle.seg_prune(np.ascontiguousarray(seg), off, retain)

    def plant(self, lg, pairs):
        for r, t in pairs:
            lg[r, t] += PLANT
        return lg

    def to_np(self, x):
        return np.asarray(x, dtype=np.float64)


class HipBackend:
    name = "hip"

    def __init__(self, stage, kv):
        import torch
        from paper_2507_02620_amd import flowspec as fs
        self.torch, self.fs = torch, fs
        self.st, self.kv = stage, kv

    def _dev(self, a, dt=None):
        t = self.torch.from_numpy(np.ascontiguousarray(a)).cuda()
        return t if dt is None else t.to(dt)

    def verify(self, l_glo, l_cache, hid, seg_off, parent):
        return self.st.tree_verify_stage(self.kv, l_glo, l_cache, self._dev(hid, self.st.dtype), seg_off, parent)

    def logits_amax(self, rows):
        lg, am = self.st.tree_logits(rows.contiguous())
        return lg, am

    def accept(self, lg, amax, token, parent, n_ver):
        T = len(token)
        self.res, self.retain, work = self.fs.new_accept_buffers(T, max(n_ver, 1))
        am = self.torch.zeros(max(n_ver, 1), dtype=self.torch.int32, device="cuda") if lg is not None else self._dev(amax)
        self.fs.tree_accept(lg, am, self._dev(token), self._dev(parent), n_ver, self.res, self.retain, work)
        out, ret = self.fs.accept_result_to_host(self.res, self.retain, T)
        return out.as_tuple(), ret

    def compact(self, l_glo, l_cache, retain, n_acc, device_list=False):
        new_len = self.torch.zeros(2, dtype=self.torch.int32, device="cuda")
        if device_list:
            self.st.kv_compact(self.kv, l_glo, l_cache, self.retain, res=self.res, new_len=new_len)
        else:
            self.st.kv_compact(self.kv, l_glo, l_cache, retain, n_acc=n_acc, new_len=new_len)
        return tuple(new_len.cpu().tolist())

    def seg_prune(self, seg, off, retain):
        out, n = self.fs.seg_prune(self._dev(seg, self.st.dtype), off, retain)
        return out[: int(n.item())]

    def plant(self, lg, pairs):
        if pairs:
            r = self.torch.tensor([p[0] for p in pairs], device="cuda")
            t = self.torch.tensor([p[1] for p in pairs], device="cuda")
            lg[r, t] += PLANT
        return lg

    def to_np(self, x):
        return x.float().cpu().numpy().astype(np.float64)


def run(backend, sched, l_glo0, on_step=None):
    """Runs sched.steps steps; returns the integer trace and, per step, the stage outputs of the rows verified in it."""
    cfg, lag, seg = sched.cfg, sched.lag, sched.cfg.seg_len
    l_glo = l_glo0
    parent, token = sched.fresh_tree(0)
    hid = sched.hidden_rows(len(parent), 0)
    n_proc = n_ver = 0
    out_rows = {}          # S index -> stage output row (backend-native) for lag == 0 logits
    trace, outputs = [], []
    for k in range(sched.steps):
        T = len(parent)
        # 1. the stage runs ahead of verification by `lag` segments
        target = min(T, n_ver + (lag + 1) * seg)
        step_out = []
        while n_proc < target:
            n = min(seg, target - n_proc)
            y = backend.verify(l_glo, l_glo + n_proc, hid[n_proc:n_proc + n], n_proc, parent[: n_proc + n])
            step_out.append(backend.to_np(y))
            for r in range(n):
                out_rows[n_proc + r] = y[r]
            n_proc += n
        # 2. verification outputs arrive for the next segment of S
        new_ver = min(T, n_ver + seg)
        pairs = sched.plants(parent, token, new_ver, k)
        if lag == 0 and cfg.vocab > 0:
            rows = [out_rows[i] for i in range(new_ver)]
            if backend.name == "oracle":
                lg, _ = backend.logits_amax(np.stack(rows))
            else:
                import torch
                parts = []
                stacked = torch.stack(rows)
                for o in range(0, new_ver, seg):
                    parts.append(backend.logits_amax(stacked[o:o + seg])[0])
                lg = torch.cat(parts)
            lg = backend.plant(lg, pairs)
            res, retain = backend.accept(lg, None, token, parent, new_ver)
        else:
            amax = sched.synthetic_amax(new_ver, k)
            for r, t in pairs:
                amax[r] = t
            res, retain = backend.accept(None, amax, token, parent, new_ver)
        n_acc, x_new, n_new, cont, n_retain, n_prv = res
        # 3. prune: the KV cache, and the segment that would be in flight next
        nxt = hid[n_proc:n_proc + seg]
        pruned = backend.seg_prune(nxt, n_proc, retain) if len(nxt) else nxt
        if backend.name == "hip" and k % 2 == 1:
            lens = backend.compact(l_glo, l_glo + n_proc, retain, n_acc, device_list=True)
        else:
            lens = backend.compact(l_glo, l_glo + n_proc, retain, n_acc)
        trace.append((T, n_proc, new_ver) + tuple(res) + tuple(int(v) for v in lens) + (int(len(pruned)),) + tuple(int(v) for v in retain))
        outputs.append(np.concatenate(step_out) if step_out else np.zeros((0, cfg.d_model)))
        if on_step:
            on_step(k, trace[-1])
        l_glo, l_cache = lens
        # 4. next tree: S_pr keeps its order, new nodes are appended; a broken round starts over
        keep = retain[n_acc:]
        if cont:
            parent, token = oracle.tree_remap(parent, token, retain, n_acc)
            hid = hid[keep]
            rows_kept = {j: out_rows[i] for j, i in enumerate(keep) if i in out_rows and i < n_proc}
            n_proc = int((keep < n_proc).sum())
            n_ver = n_prv
            out_rows = {j: v for j, v in rows_kept.items() if j < n_proc}
            assert l_cache - l_glo == n_proc
            parent, token = synth.extend_tree(parent, token, cfg.tree_size, cfg.max_depth + 64, cfg.max_branch, max(cfg.vocab, 2), sched.seed, k)
            if len(parent) > len(hid):
                hid = np.concatenate([hid, sched.hidden_rows(len(parent) - len(hid), k + 1)])
        else:
            assert l_cache == l_glo
            parent, token = sched.fresh_tree(k + 1)
            hid = sched.hidden_rows(len(parent), k + 1)
            n_proc = n_ver = 0
            out_rows = {}
    return trace, outputs
