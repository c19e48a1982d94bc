"""Thin ctypes binding over libflowspec_hip.so (include/flowspec.h): argument marshalling only.

PyTorch supplies device memory (`tensor.data_ptr()`) and the stream; every step of the path runs in
the library's HIP kernels.  If the library has not been built (`python -m paper_2507_02620_amd.build`)
importing this module raises: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflowspec_hip.so")

FS_OK, FS_EINVAL, FS_ETOPO, FS_ECAP, FS_EDTYPE, FS_EHIP, FS_EWS = 0, -1, -2, -3, -4, -5, -6
FS_F32, FS_BF16 = 0, 1
FS_MAX_TREE = 1024
FS_ARGMAX_CHUNKS = 64
_ERR = {FS_EINVAL: "FS_EINVAL", FS_ETOPO: "FS_ETOPO", FS_ECAP: "FS_ECAP", FS_EDTYPE: "FS_EDTYPE", FS_EHIP: "FS_EHIP", FS_EWS: "FS_EWS"}

KERNEL_KINDS = ("prepare", "qkv", "attn", "oproj", "gateup", "down", "head", "argmax", "compact")

EXPORTS = ("fs_stage_workspace_bytes", "fs_stage_create", "fs_stage_destroy", "fs_last_hip_error", "fs_stage_profile_begin",
           "fs_stage_profile_end", "fs_tree_verify_stage", "fs_tree_verify_batch", "fs_tree_mask",
           "fs_tree_logits", "fs_tree_accept", "fs_tree_accept_noalloc", "fs_tree_accept_sample", "fs_accept_result_to_host", "fs_kv_compact", "fs_seg_prune", "fs_tree_segment",
           "fs_tree_prune", "fs_tree_merge", "fs_probe_stream_read", "fs_probe_mfma_bf16", "fs_probe_fill")


class FlowSpecError(RuntimeError):
    def __init__(self, code, what, hip=0):
        super().__init__(f"{what}: {_ERR.get(code, code)}" + (f" (hipError {hip})" if code == FS_EHIP else ""))
        self.code = code
        self.hip = hip


class StageDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int), ("d_model", C.c_int), ("n_q_heads", C.c_int), ("n_kv_heads", C.c_int), ("head_dim", C.c_int),
                ("d_ffn", C.c_int), ("vocab", C.c_int), ("dtype", C.c_int), ("rms_eps", C.c_float), ("rope_theta", C.c_float),
                ("kv_capacity", C.c_int), ("max_tree", C.c_int), ("max_seg", C.c_int), ("weight_format", C.c_int)]


_W = ("rms_attn", "wq", "wk", "wv", "wo", "rms_ffn", "w_gate", "w_up", "w_down", "bq", "bk", "bv",
      "sq", "sk", "sv", "so", "s_gate", "s_up", "s_down")
_W_CODES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")
FS_WFMT_DENSE, FS_WFMT_INT4_G128 = 0, 1


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _W]


class KVCache(C.Structure):
    _fields_ = [("base", C.c_void_p), ("stride_layer", C.c_longlong), ("stride_kv", C.c_longlong), ("stride_head", C.c_longlong),
                ("stride_tok", C.c_longlong)]


class BatchItem(C.Structure):
    _fields_ = [("kv", KVCache), ("l_glo", C.c_int), ("l_cache", C.c_int), ("seg_off", C.c_int), ("l_s", C.c_int), ("parent", C.POINTER(C.c_int32))]


FS_MAX_BATCH = 32


class AcceptResult(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_acc", "x_new", "n_new", "continuous", "n_retain", "n_pr_verified")]

    def as_tuple(self):
        return tuple(int(getattr(self, n)) for n, _ in self._fields_)


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2507_02620_amd.build` (no fallback path exists)")
    lib = C.CDLL(LIB_PATH)
    vp, ci, i32p = C.c_void_p, C.c_int, C.c_void_p
    lib.fs_stage_workspace_bytes.restype = C.c_size_t
    lib.fs_stage_workspace_bytes.argtypes = [C.POINTER(StageDesc)]
    lib.fs_stage_create.argtypes = [C.POINTER(StageDesc), C.POINTER(LayerWeights), vp, vp, vp, vp, C.c_size_t, vp, C.POINTER(vp)]
    lib.fs_stage_destroy.argtypes = [vp]
    lib.fs_stage_profile_begin.argtypes = [vp, ci]
    lib.fs_stage_profile_end.argtypes = [vp, vp, C.POINTER(C.c_double), C.POINTER(C.c_longlong)]
    lib.fs_tree_verify_stage.argtypes = [vp, KVCache, ci, ci, vp, ci, ci, i32p, vp, vp]
    lib.fs_tree_verify_batch.argtypes = [vp, C.POINTER(BatchItem), ci, vp, vp, vp]
    lib.fs_tree_logits.argtypes = [vp, vp, ci, vp, vp, vp]
    lib.fs_tree_mask.argtypes = [vp, ci, ci, ci, i32p, vp, vp, vp]
    lib.fs_tree_accept.argtypes = [vp, vp, ci, vp, vp, ci, ci, vp, vp, vp, vp]
    lib.fs_tree_accept_noalloc.argtypes = [vp, vp, ci, vp, vp, ci, ci, vp, vp, vp]
    lib.fs_tree_accept_sample.argtypes = [vp, ci, C.c_float, vp, vp, ci, ci, C.c_uint64, C.c_uint64, vp, vp, vp, vp]
    lib.fs_accept_result_to_host.argtypes = [vp, vp, ci, C.POINTER(AcceptResult), i32p, vp]
    lib.fs_kv_compact.argtypes = [vp, KVCache, ci, ci, vp, vp, ci, ci, vp, vp]
    lib.fs_seg_prune.argtypes = [vp, ci, C.c_size_t, ci, vp, vp, ci, vp, vp, vp]
    lib.fs_tree_segment.argtypes = [vp, vp, vp, ci, ci, vp, vp, vp, vp]
    lib.fs_tree_prune.argtypes = [vp, vp, ci, vp, ci, ci, vp, vp]
    lib.fs_tree_merge.argtypes = [vp, vp, ci, vp, vp, ci, ci, ci, vp, vp, vp, vp]
    lib.fs_probe_stream_read.argtypes = [vp, C.c_size_t, C.c_size_t, ci, vp, C.POINTER(C.c_double)]
    lib.fs_probe_mfma_bf16.argtypes = [vp, ci, vp, C.POINTER(C.c_double)]
    lib.fs_probe_fill.argtypes = [vp, C.c_size_t, ci, ci, ci, ci, ci, ci, ci, vp, C.POINTER(C.c_double)]
    for n in EXPORTS:
        if n not in ("fs_stage_workspace_bytes",):
            getattr(lib, n).restype = C.c_int
    return lib


_lib = _load()


def lib():
    return _lib


def _check(rc, what):
    if rc != FS_OK:
        raise FlowSpecError(rc, what, _lib.fs_last_hip_error() if rc == FS_EHIP else 0)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dp(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _host_i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.c_void_p)


def torch_dtype(code):
    return torch.float32 if code == FS_F32 else torch.bfloat16


def kv_descriptor(kv: torch.Tensor) -> KVCache:
    """kv: device tensor [n_layers, 2, n_kv_heads, capacity, head_dim] (any strides with a contiguous last dim)."""
    assert kv.dim() == 5 and kv.shape[1] == 2 and kv.stride(4) == 1
    return KVCache(kv.data_ptr(), kv.stride(0), kv.stride(1), kv.stride(2), kv.stride(3))


class Stage:
    """One verification stage: owns the workspace tensor and the opaque handle."""

    def __init__(self, *, n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, dtype, rms_eps, rope_theta, kv_capacity,
                 max_tree, max_seg, layers, final_norm=None, lm_head=None, lm_head_scale=None, weight_format=FS_WFMT_DENSE, device="cuda",
                 stream=None):
        self.desc = StageDesc(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, dtype, rms_eps, rope_theta, kv_capacity,
                              max_tree, max_seg, weight_format)
        self.dtype = torch_dtype(dtype)
        self.device = torch.device(device)
        nbytes = _lib.fs_stage_workspace_bytes(C.byref(self.desc))
        if nbytes == 0:
            # let the library name the reason
            h = C.c_void_p()
            _check(_lib.fs_stage_create(C.byref(self.desc), None, None, None, None, None, 0, None, C.byref(h)) or FS_EINVAL, "fs_stage_create")
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = self.workspace.data_ptr()
        self._ws_ptr = (base + 255) // 256 * 256
        arr = (LayerWeights * n_layers)()
        for i, lw in enumerate(layers):
            for n in _W:
                t = lw.get(n)
                if t is not None:
                    want = torch.uint8 if (weight_format == FS_WFMT_INT4_G128 and n in _W_CODES) else self.dtype
                    assert t.is_cuda and t.is_contiguous() and t.dtype == want, n
                setattr(arr[i], n, None if t is None else t.data_ptr())
        self._handle = C.c_void_p()
        _check(_lib.fs_stage_create(C.byref(self.desc), arr, _dp(final_norm), _dp(lm_head), _dp(lm_head_scale), C.c_void_p(self._ws_ptr), nbytes,
                                    _stream(stream), C.byref(self._handle)), "fs_stage_create")
        self.workspace_bytes = nbytes

    def close(self):
        if getattr(self, "_handle", None):
            if _lib is not None:  # at interpreter exit the module's globals may already be gone; the process frees the stage then
                _lib.fs_stage_destroy(self._handle)
            self._handle = None

    def __del__(self):
        self.close()

    def profile_begin(self, max_records=65536):
        _check(_lib.fs_stage_profile_begin(self._handle, int(max_records)), "fs_stage_profile_begin")

    def profile_end(self, stream=None):
        """{kind: (total_ms, launches)} of everything the stage enqueued since profile_begin."""
        n = len(KERNEL_KINDS)
        ms, cnt = (C.c_double * n)(), (C.c_longlong * n)()
        _check(_lib.fs_stage_profile_end(self._handle, _stream(stream), ms, cnt), "fs_stage_profile_end")
        return {k: (float(ms[i]), int(cnt[i])) for i, k in enumerate(KERNEL_KINDS)}

    def new_kv_cache(self) -> torch.Tensor:
        d = self.desc
        return torch.zeros((d.n_layers, 2, d.n_kv_heads, d.kv_capacity, d.head_dim), dtype=self.dtype, device=self.device)

    def tree_verify_stage(self, kv, l_glo, l_cache, hidden_in, seg_off, parent, hidden_out=None, stream=None):
        l_s = int(hidden_in.shape[0])
        if hidden_out is None:
            hidden_out = torch.empty_like(hidden_in)
        par, pp = _host_i32(parent)
        assert par.shape[0] >= seg_off + l_s
        _check(_lib.fs_tree_verify_stage(self._handle, kv_descriptor(kv), int(l_glo), int(l_cache), _dp(hidden_in), int(seg_off), l_s, pp,
                                         _dp(hidden_out), _stream(stream)), "fs_tree_verify_stage")
        return hidden_out

    def tree_verify_batch(self, items, hidden_in, hidden_out=None, stream=None):
        """items: sequence of (kv tensor, l_glo, l_cache, seg_off, l_s, parent) — one segment per request; hidden_in holds the
        items' rows stacked in item order."""
        if hidden_out is None:
            hidden_out = torch.empty_like(hidden_in)
        arr = (BatchItem * len(items))()
        keep = []
        for i, (kv, l_glo, l_cache, seg_off, l_s, parent) in enumerate(items):
            par = np.ascontiguousarray(parent, dtype=np.int32)
            keep.append(par)
            arr[i] = BatchItem(kv_descriptor(kv), int(l_glo), int(l_cache), int(seg_off), int(l_s), par.ctypes.data_as(C.POINTER(C.c_int32)))
        _check(_lib.fs_tree_verify_batch(self._handle, arr, len(items), _dp(hidden_in), _dp(hidden_out), _stream(stream)), "fs_tree_verify_batch")
        return hidden_out

    def tree_mask(self, l_glo, seg_off, l_s, parent, stream=None):
        """(anc int64 [l_s, 16] holding the uint64 mask words, rope float32 [l_s, head_dim/2, 2]) of a segment, as the forward derives them."""
        par, pp = _host_i32(parent)
        assert par.shape[0] >= seg_off + l_s
        anc = torch.zeros((l_s, FS_MAX_TREE // 64), dtype=torch.int64, device=self.device)
        rope = torch.zeros((l_s, self.desc.head_dim // 2, 2), dtype=torch.float32, device=self.device)
        _check(_lib.fs_tree_mask(self._handle, int(l_glo), int(seg_off), int(l_s), pp, _dp(anc), _dp(rope), _stream(stream)), "fs_tree_mask")
        return anc, rope

    def tree_logits(self, hidden, logits=None, amax=None, stream=None):
        l_s = int(hidden.shape[0])
        if logits is None:
            logits = torch.empty((l_s, self.desc.vocab), dtype=torch.float32, device=self.device)
        if amax is None:
            amax = torch.empty((l_s,), dtype=torch.int32, device=self.device)
        _check(_lib.fs_tree_logits(self._handle, _dp(hidden), l_s, _dp(logits), _dp(amax), _stream(stream)), "fs_tree_logits")
        return logits, amax

    def kv_compact(self, kv, l_glo, l_cache, retain, res=None, n_acc=None, new_len=None, stream=None):
        """retain: device int32 tensor together with `res` (device AcceptResult buffer), or a host sequence with n_acc."""
        if res is not None:
            _check(_lib.fs_kv_compact(self._handle, kv_descriptor(kv), int(l_glo), int(l_cache), _dp(retain), _dp(res), 0, 0, _dp(new_len),
                                      _stream(stream)), "fs_kv_compact")
        else:
            r, rp = _host_i32(retain)
            _check(_lib.fs_kv_compact(self._handle, kv_descriptor(kv), int(l_glo), int(l_cache), rp, None, int(r.shape[0]), int(n_acc),
                                      _dp(new_len), _stream(stream)), "fs_kv_compact")


def new_accept_buffers(T, n_ver_max, device="cuda"):
    """Device buffers for tree_accept: (res [6] int32, retain [T] int32, work int32)."""
    res = torch.zeros(6, dtype=torch.int32, device=device)
    retain = torch.zeros(max(T, 1), dtype=torch.int32, device=device)
    work = torch.zeros(2 * max(n_ver_max, 1) * FS_ARGMAX_CHUNKS, dtype=torch.int32, device=device)
    return res, retain, work


def probe_stream_read(buf, bytes_per_launch, launches=20, stream=None) -> float:
    """GB/s of a one-pass read of bytes_per_launch bytes, rotating through the device tensor `buf` (measurement aid)."""
    out = C.c_double()
    _check(_lib.fs_probe_stream_read(_dp(buf), C.c_size_t(buf.numel() * buf.element_size()), C.c_size_t(int(bytes_per_launch)), int(launches),
                                     _stream(stream), C.byref(out)), "fs_probe_stream_read")
    return out.value


def probe_mfma_bf16(scratch, launches=5, stream=None) -> float:
    """TFLOP/s of a register-resident bf16 MFMA loop (measurement aid)."""
    out = C.c_double()
    _check(_lib.fs_probe_mfma_bf16(_dp(scratch), int(launches), _stream(stream), C.byref(out)), "fs_probe_mfma_bf16")
    return out.value


def probe_fill(buf, grid, waves, region_kib, iters, share=1, to_lds=True, launches=5, stream=None) -> float:
    """GB/s (all workgroups together) at which compute units pull data from a cache-resident region (measurement aid)."""
    out = C.c_double()
    _check(_lib.fs_probe_fill(_dp(buf), C.c_size_t(buf.numel() * buf.element_size()), int(grid), int(waves), int(region_kib), int(iters),
                              int(share), int(bool(to_lds)), int(launches), _stream(stream), C.byref(out)), "fs_probe_fill")
    return out.value


def tree_accept(logits, amax, token, parent, n_ver, res, retain, work=None, stream=None):
    T = int(token.shape[0])
    vocab = int(logits.shape[1]) if logits is not None else 0
    _check(_lib.fs_tree_accept(_dp(logits), _dp(amax), vocab, _dp(token), _dp(parent), T, int(n_ver), _dp(res), _dp(retain), _dp(work),
                               _stream(stream)), "fs_tree_accept")


def tree_accept_noalloc(logits, amax, token, parent, n_ver, res, retain, stream=None):
    """tree_accept without a caller-provided scratch buffer (the library's static device array takes its place)."""
    T = int(token.shape[0])
    vocab = int(logits.shape[1]) if logits is not None else 0
    _check(_lib.fs_tree_accept_noalloc(_dp(logits), _dp(amax), vocab, _dp(token), _dp(parent), T, int(n_ver), _dp(res), _dp(retain),
                                       _stream(stream)), "fs_tree_accept_noalloc")


def tree_accept_sample(logits, temperature, token, parent, n_ver, seed, step, res, retain, work=None, stream=None):
    """Stochastic acceptance (temperature > 0); `work` is any 16-byte aligned device buffer of >= 16 + 12 * n_ver bytes."""
    T = int(token.shape[0])
    if work is None:
        work = torch.empty(16 + 12 * max(int(n_ver), 1) + 16, dtype=torch.uint8, device=token.device)
    _check(_lib.fs_tree_accept_sample(_dp(logits), int(logits.shape[1]), float(temperature), _dp(token), _dp(parent), T, int(n_ver),
                                      int(seed), int(step), _dp(res), _dp(retain), _dp(work), _stream(stream)), "fs_tree_accept_sample")


def accept_result_to_host(res, retain, T, stream=None):
    out = AcceptResult()
    buf = np.zeros(max(T, 1), dtype=np.int32)
    _check(_lib.fs_accept_result_to_host(_dp(res), _dp(retain), int(T), C.byref(out), buf.ctypes.data_as(C.c_void_p), _stream(stream)),
           "fs_accept_result_to_host")
    n = max(out.n_retain, 0)
    return out, buf[:n].copy()


def seg_prune(seg_in, off, retain, res=None, seg_out=None, l_s_out=None, stream=None):
    l_s = int(seg_in.shape[0])
    row_bytes = seg_in.element_size() * int(np.prod(seg_in.shape[1:]))
    if seg_out is None:
        seg_out = torch.empty_like(seg_in)
    if l_s_out is None:
        l_s_out = torch.zeros(1, dtype=torch.int32, device=seg_in.device)
    if res is not None:
        _check(_lib.fs_seg_prune(_dp(seg_in), l_s, row_bytes, int(off), _dp(retain), _dp(res), 0, _dp(seg_out), _dp(l_s_out), _stream(stream)),
               "fs_seg_prune")
    else:
        r, rp = _host_i32(retain)
        _check(_lib.fs_seg_prune(_dp(seg_in), l_s, row_bytes, int(off), rp, None, int(r.shape[0]), _dp(seg_out), _dp(l_s_out), _stream(stream)),
               "fs_seg_prune")
    return seg_out, l_s_out


def stage_from_config(cfg, layers, final_norm=None, lm_head=None, kv_capacity=None, max_tree=None, max_seg=None, device="cuda",
                      lm_head_scale=None, weight_format=FS_WFMT_DENSE):
    """Build a Stage from a synth.StageConfig-like object and device weight tensors."""
    return Stage(n_layers=cfg.n_layers, d_model=cfg.d_model, n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                 d_ffn=cfg.d_ffn, vocab=(cfg.vocab if lm_head is not None else 0), dtype=FS_F32 if cfg.dtype == "f32" else FS_BF16,
                 rms_eps=cfg.rms_eps, rope_theta=cfg.rope_theta, kv_capacity=kv_capacity or cfg.kv_capacity,
                 max_tree=max_tree or cfg.tree_size, max_seg=max_seg or cfg.seg_len, layers=layers, final_norm=final_norm, lm_head=lm_head,
                 lm_head_scale=lm_head_scale, weight_format=weight_format, device=device)


# ---- host-side tree bookkeeping (no GPU) -------------------------------------------------------------------------------

def _hp(a):
    return a.ctypes.data_as(C.c_void_p)


def tree_segment(parent_base, token_base, conf, L0):
    """Score-based draft segmentation: returns (parent, token, score, base_index) of S."""
    pb, tb = np.ascontiguousarray(parent_base, dtype=np.int32), np.ascontiguousarray(token_base, dtype=np.int32)
    cf = np.ascontiguousarray(conf, dtype=np.float32)
    n = min(int(L0), pb.shape[0])
    par, tok, sc, bi = np.zeros(n, np.int32), np.zeros(n, np.int32), np.zeros(n, np.float64), np.zeros(n, np.int32)
    rc = _lib.fs_tree_segment(_hp(pb), _hp(tb), _hp(cf), pb.shape[0], int(L0), _hp(par), _hp(tok), _hp(sc), _hp(bi))
    if rc < 0:
        raise FlowSpecError(rc, "fs_tree_segment")
    return par[:rc], tok[:rc], sc[:rc], bi[:rc]


def tree_prune(parent, token, retain, n_acc):
    par, tok = np.ascontiguousarray(parent, dtype=np.int32), np.ascontiguousarray(token, dtype=np.int32)
    ret = np.ascontiguousarray(retain, dtype=np.int32)
    n = max(ret.shape[0] - int(n_acc), 1)
    npar, ntok = np.zeros(n, np.int32), np.zeros(n, np.int32)
    rc = _lib.fs_tree_prune(_hp(par), _hp(tok), par.shape[0], _hp(ret), int(n_acc), ret.shape[0], _hp(npar), _hp(ntok))
    if rc < 0:
        raise FlowSpecError(rc, "fs_tree_prune")
    return npar[:rc].copy(), ntok[:rc].copy()


def tree_merge(parent_pr, token_pr, parent_new, token_new, limit=-1, max_out=None):
    """Merge T_new into T_pr: returns (parent, token, app_src, map_new) with S = S_pr || S_app."""
    ppr, tpr = np.ascontiguousarray(parent_pr, dtype=np.int32), np.ascontiguousarray(token_pr, dtype=np.int32)
    pnw, tnw = np.ascontiguousarray(parent_new, dtype=np.int32), np.ascontiguousarray(token_new, dtype=np.int32)
    cap = int(max_out) if max_out is not None else ppr.shape[0] + pnw.shape[0]
    par, tok = np.zeros(max(cap, 1), np.int32), np.zeros(max(cap, 1), np.int32)
    app, mp = np.zeros(max(pnw.shape[0], 1), np.int32), np.zeros(max(pnw.shape[0], 1), np.int32)
    rc = _lib.fs_tree_merge(_hp(ppr), _hp(tpr), ppr.shape[0], _hp(pnw), _hp(tnw), pnw.shape[0], int(limit), cap, _hp(par), _hp(tok), _hp(app),
                            _hp(mp))
    if rc < 0:
        raise FlowSpecError(rc, "fs_tree_merge")
    return par[:rc].copy(), tok[:rc].copy(), app[: rc - ppr.shape[0]].copy(), mp[: pnw.shape[0]].copy()
