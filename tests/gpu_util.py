"""GPU-side test plumbing: the same seeded inputs go to the oracle (numpy) and to the HIP library (device copies)."""
import numpy as np
import torch

from oracle import oracle
from paper_2507_02620_amd import flowspec as fs
from paper_2507_02620_amd import synth


def to_dev(a, dtype):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(device="cuda", dtype=dtype)


class Pair:
    """An oracle stage and a HIP stage built from identical inputs."""

    def __init__(self, cfg, seed=0, head=False, capacity=None, max_tree=None, max_seg=None, oracle_layers=None, w4=False):
        self.cfg = cfg
        self.seed = seed
        self.tdtype = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
        cap = capacity or cfg.kv_capacity
        nl_o = cfg.n_layers if oracle_layers is None else oracle_layers
        lm_s = None
        if w4:
            # 4-bit group storage: the HIP stage gets codes and scales, the oracle the plain matrices they stand for
            layers = [synth.layer_weights_w4(cfg, l, seed) for l in range(cfg.n_layers)]
            fn, lm, lm_s = synth.head_weights_w4(cfg, seed) if head else (None, None, None)
            self.orc = oracle.Stage(cfg.with_(n_layers=nl_o), [oracle.dequant_layer(lw) for lw in layers[:nl_o]], fn,
                                    None if lm is None else oracle.dequant_w4(lm, lm_s), cap)
            dev_layers = [{k: to_dev(v, torch.uint8 if k in oracle.W4_SCALES else self.tdtype) for k, v in lw.items()} for lw in layers]
            self.dev_lm = to_dev(lm, torch.uint8)
        else:
            layers = [synth.layer_weights(cfg, l, seed) for l in range(cfg.n_layers)]
            fn, lm = synth.head_weights(cfg, seed) if head else (None, None)
            self.orc = oracle.Stage(cfg.with_(n_layers=nl_o), layers[:nl_o], fn, lm, cap)
            dev_layers = [{k: to_dev(v, self.tdtype) for k, v in lw.items()} for lw in layers]
            self.dev_lm = to_dev(lm, self.tdtype)
        self.dev_fn, self.dev_lm_s = to_dev(fn, self.tdtype), to_dev(lm_s, self.tdtype)
        self.gpu = fs.stage_from_config(cfg, dev_layers, self.dev_fn, self.dev_lm, kv_capacity=cap, max_tree=max_tree, max_seg=max_seg,
                                        lm_head_scale=self.dev_lm_s, weight_format=fs.FS_WFMT_INT4_G128 if w4 else fs.FS_WFMT_DENSE)
        torch.cuda.synchronize()
        del dev_layers  # the stage keeps its own re-tiled copy
        self.kv = self.gpu.new_kv_cache()
        for l in range(cfg.n_layers):
            pre = synth.prefix_kv(cfg, l, cap, seed)
            if l < nl_o:
                self.orc.load_prefix(l, pre)
            self.kv[l].copy_(to_dev(pre, self.tdtype))
        self.layers = layers

    def verify_tree(self, parent, hid, seg_len, l_glo=None):
        """Both sides verify S in consecutive segments; returns (oracle rows fp64, gpu rows fp32 numpy)."""
        cfg = self.cfg
        l_glo = cfg.l_glo if l_glo is None else l_glo
        T = len(parent)
        o_out = np.zeros((T, cfg.d_model))
        g_out = np.zeros((T, cfg.d_model), dtype=np.float32)
        hid_dev = to_dev(hid, self.tdtype)
        for off, n in synth.segments(T, seg_len):
            o_out[off:off + n] = self.orc.verify(l_glo, l_glo + off, hid[off:off + n], off, parent[: off + n])
            y = self.gpu.tree_verify_stage(self.kv, l_glo, l_glo + off, hid_dev[off:off + n].contiguous(), off, parent[: off + n])
            g_out[off:off + n] = y.float().cpu().numpy()
        torch.cuda.synchronize()
        return o_out, g_out


def max_rel_err(got, ref):
    """max |got - ref| / max |ref| over the whole tensor."""
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(np.asarray(got, dtype=np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def row_rel_err(got, ref):
    """Worst row: max over rows of max |got_row - ref_row| / max |ref_row| (rows = leading axes, values = last axis)."""
    ref = np.asarray(ref, dtype=np.float64)
    d = np.abs(np.asarray(got, dtype=np.float64) - ref).reshape(-1, ref.shape[-1]).max(axis=1)
    m = np.abs(ref).reshape(-1, ref.shape[-1]).max(axis=1)
    return float((d / np.maximum(m, 1e-30)).max())


TOL = {"f32": 1e-4, "bf16": 2e-2}
