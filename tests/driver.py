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

    def __init__(self, cfg, seed, lag, steps, closed=False):
        # closed: every node of the accepted path gets a planted output, also the last one, so that the integer trace does not
        # depend on any un-planted logit (needed when one side runs without a forward)
        self.cfg, self.seed, self.lag, self.steps, self.closed = cfg, seed, lag, steps, closed

    def fresh_tree(self, k):
        t = synth.random_tree(self.cfg.tree_size, self.cfg.max_depth, self.cfg.max_branch, max(self.cfg.vocab, 2), self.seed, stream=1000 + k)
        return t.parent, t.token

    def hidden_rows(self, n, k):
        return synth.hidden(self.cfg, n, call=100 + k, seed=self.seed)

    def plants(self, parent, token, n_ver, k):
        t = synth.Tree(parent, token, np.zeros(len(parent)), synth._depths(parent))
        pairs = synth.resolve_plants(synth.plant_path(t, n_ver, self.seed, k, p_stop=0.2, mean_extra=1.0), t, max(self.cfg.vocab, 2))
        if self.closed and pairs:
            vocab = max(self.cfg.vocab, 2)
            row, tok = pairs[-1]
            while True:  # the last plant may point at a verified child: that child is accepted too and needs an output of its own
                hit = [c for c in range(len(parent)) if parent[c] == row and token[c] == tok and c < n_ver]
                if not hit:
                    break
                row = hit[0]
                kids = [c for c in range(len(parent)) if parent[c] == row]
                late = [c for c in kids if c >= n_ver]
                if late:
                    tok = int(token[late[0]])
                else:
                    forbid = {int(token[c]) for c in kids}
                    tok = (row * 7919 + k) % vocab
                    while tok in forbid:
                        tok = (tok + 1) % vocab
                pairs.append((row, tok))
        return pairs

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


class IntegerOracleBackend:
    """The oracle's integer side alone (accept, compaction lengths, segment pruning), free-running: no forward.  Acceptance
    is planted on every node of the accepted path and sibling tokens are distinct, so the integer trace of a schedule does
    not depend on the un-planted logits; zeros stand in for them.  Lets a long schedule at full depth be traced in seconds."""
    name = "oracle"

    def __init__(self, cfg, capacity):
        self.cfg = cfg
        self.kv = np.zeros((1, 2, 1, capacity, 1), dtype=np.int8)   # only its lengths matter

    def verify(self, l_glo, l_cache, hid, seg_off, parent):
        return np.zeros((len(hid), 1))

    def logits_amax(self, rows):
        return np.zeros((len(rows), self.cfg.vocab), dtype=np.float32), None

    accept = OracleBackend.accept
    seg_prune = OracleBackend.seg_prune
    plant = OracleBackend.plant
    to_np = OracleBackend.to_np

    def compact(self, l_glo, l_cache, retain, n_acc):
        return oracle.kv_compact(self.kv, l_glo, l_cache, retain, n_acc)


class CheckedHipBackend(HipBackend):
    """The HIP path running a schedule, checked against the oracle as it goes:
      every step   accept against orc_accept on the HIP path's own argmax, compaction against orc_kv_compact applied to a
                   snapshot of the draft slots (both bit for bit);
      sampled steps  the oracle's cache is brought to the HIP path's state (its draft slots are copied over; the context
                   below l_glo0 is the shared seeded prefix, which nothing may touch) and the step's forward and logits are
                   compared within the tolerance."""

    def __init__(self, stage, kv, orc, l_glo0, sample_steps, tol, log=print):
        super().__init__(stage, kv)
        self.orc, self.l_glo0, self.samples, self.tol, self.log = orc, l_glo0, set(sample_steps), tol, log
        self.k = -1
        self.worst = {"hidden": 0.0, "hidden_row": 0.0, "kv": 0.0, "logits": 0.0}
        self.checked_steps = []

    def begin_step(self, k):
        self.k = k

    def _sampled(self):
        return self.k in self.samples

    def _sync_oracle(self, l_cache):
        n = l_cache - self.l_glo0
        if n > 0:
            self.orc.kv[:, :, :, self.l_glo0:l_cache] = self.kv[:, :, :, self.l_glo0:l_cache].float().cpu().numpy()

    def verify(self, l_glo, l_cache, hid, seg_off, parent):
        y = super().verify(l_glo, l_cache, hid, seg_off, parent)
        if self._sampled():
            from tests.gpu_util import max_rel_err, row_rel_err
            n = len(hid)
            self._sync_oracle(l_cache)
            want = self.orc.verify(l_glo, l_cache, hid, seg_off, parent)
            got = self.to_np(y)
            e, er = max_rel_err(got, want), row_rel_err(got, want)
            ke = max(max_rel_err(self.kv[l, x, :, l_cache:l_cache + n].float().cpu().numpy(), self.orc.kv[l, x, :, l_cache:l_cache + n])
                     for l in range(self.orc.kv.shape[0]) for x in (0, 1))
            self.log(f"    step {self.k}: {n} rows at l_glo={l_glo} l_cache={l_cache}: hidden {e:.3e} (worst row {er:.3e}), appended K/V worst layer {ke:.3e}")
            self.worst["hidden"] = max(self.worst["hidden"], e)
            self.worst["hidden_row"] = max(self.worst["hidden_row"], er)
            self.worst["kv"] = max(self.worst["kv"], ke)
            assert e < self.tol and er < 2 * self.tol and ke < self.tol, (self.k, e, er, ke)
            if self.k not in self.checked_steps:
                self.checked_steps.append(self.k)
        return y

    def logits_amax(self, rows):
        lg, am = super().logits_amax(rows)
        if self._sampled() and self.orc.lm_head is not None:
            from tests.gpu_util import max_rel_err
            want, _ = self.orc.logits(self.to_np(rows))
            e = max_rel_err(lg.cpu().numpy(), want)
            self.worst["logits"] = max(self.worst["logits"], e)
            assert e < self.tol, (self.k, e)
        return lg, am

    def accept(self, lg, amax, token, parent, n_ver):
        T = len(token)
        self.res, self.retain, work = self.fs.new_accept_buffers(T, max(n_ver, 1))
        am = self.torch.zeros(max(n_ver, 1), dtype=self.torch.int32, device="cuda") if lg is not None else self._dev(amax)
        self.fs.tree_accept(lg, am, self._dev(token), self._dev(parent), n_ver, self.res, self.retain, work)
        out, ret = self.fs.accept_result_to_host(self.res, self.retain, T)
        o_res, o_ret = oracle.accept(am.cpu().numpy()[:n_ver], token, parent, n_ver)
        assert out.as_tuple() == o_res.as_tuple() and np.array_equal(ret, o_ret), (self.k, out.as_tuple(), o_res.as_tuple())
        return out.as_tuple(), ret

    def compact(self, l_glo, l_cache, retain, n_acc, device_list=False):
        bits = self.torch.int16 if self.kv.element_size() == 2 else self.torch.int32
        n = l_cache - l_glo
        snap = np.ascontiguousarray(self.kv[:, :, :, l_glo:l_cache].contiguous().view(bits).cpu().numpy()) if n > 0 else None
        lens = super().compact(l_glo, l_cache, retain, n_acc, device_list)
        if n > 0:
            rel = oracle.kv_compact(snap, 0, n, retain, n_acc)
            assert lens == (l_glo + rel[0], l_glo + rel[1]), (self.k, lens, rel)
            after = self.kv[:, :, :, l_glo:lens[1]].contiguous().view(bits).cpu().numpy()
            assert np.array_equal(after, snap[:, :, :, : rel[1]]), f"step {self.k}: compacted cache differs from the oracle's gather"
        return lens


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
        if hasattr(backend, "begin_step"):
            backend.begin_step(k)
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
