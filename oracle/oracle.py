"""ctypes/numpy wrapper around the C oracle.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
module; it shares no code with the HIP library and never loads it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "flowspec_oracle.c")
_LIB = os.path.join(_HERE, "libflowspec_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (AVX2-level code so the library also runs on the GPU host)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=x86-64-v3", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-std=gnu11", "-Wall", "-o", _LIB, _SRC,
               "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Desc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab", "wdtype")] + [
        ("rms_eps", C.c_double), ("rope_theta", C.c_double), ("kv_capacity", C.c_int)]


class _Layer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("rms_attn", "wq", "wk", "wv", "wo", "rms_ffn", "w_gate", "w_up", "w_down", "bq", "bk", "bv")]


class AcceptResult(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_acc", "x_new", "n_new", "continuous", "n_retain", "n_pr_verified")]

    def as_tuple(self):
        return tuple(int(getattr(self, n)) for n, _ in self._fields_)


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _check(rc, what):
    if rc != 0:
        raise OracleError(rc, what)


class OracleError(RuntimeError):
    def __init__(self, rc, what):
        super().__init__(f"{what} failed with code {rc}")
        self.rc = rc


def tree_ancestors(parent):
    parent = _i32(parent)
    T = parent.shape[0]
    W = (T + 63) // 64
    anc = np.zeros((T, max(W, 1)), dtype=np.uint64)
    depth = np.zeros(T, dtype=np.int32)
    _check(lib().orc_tree_ancestors(_ptr(parent), T, _ptr(anc), _ptr(depth)), "orc_tree_ancestors")
    return anc, depth


def rmsnorm(x, g, eps):
    x = _f64(x)
    g = np.ascontiguousarray(g, dtype=np.float32)
    out = np.empty_like(x)
    lib().orc_rmsnorm(_ptr(x), _ptr(g), 0, x.shape[0], C.c_double(eps), _ptr(out))
    return out


def rope(v, pos, theta):
    v = _f64(v).copy()
    lib().orc_rope(_ptr(v), v.shape[0], C.c_double(pos), C.c_double(theta))
    return v


W4_SCALES = {"wq": "sq", "wk": "sk", "wv": "sv", "wo": "so", "w_gate": "s_gate", "w_up": "s_up", "w_down": "s_down"}


def dequant_w4(codes, scales):
    """4-bit group storage to plain weights: w[n][k] = scale[n][k // 128] * (code[n][k] - 8), column k even in the low
    nibble of byte k // 2.  The product of a bf16 scale and an integer in [-8, 7] is exact in float32."""
    codes = np.asarray(codes, dtype=np.uint8)
    n, half = codes.shape
    q = np.empty((n, half, 2), dtype=np.int16)
    q[:, :, 0] = codes & 15
    q[:, :, 1] = codes >> 4
    q = (q.reshape(n, half * 2 // 128, 128) - 8).astype(np.float32)
    return np.ascontiguousarray((q * np.asarray(scales, dtype=np.float32)[:, :, None]).reshape(n, half * 2))


def dequant_layer(lw):
    """A layer dict with 4-bit matrices (codes + s* scales) as plain float32 matrices."""
    out = {k: v for k, v in lw.items() if k not in W4_SCALES.values()}
    for name, sname in W4_SCALES.items():
        out[name] = dequant_w4(lw[name], lw[sname])
    return out


class Stage:
    """Oracle-side state of one stage: weights (float32 arrays, or uint16 bf16 bit patterns) and a fp64 KV cache."""

    def __init__(self, cfg, layers, final_norm=None, lm_head=None, kv_capacity=None, bf16_bits=False):
        self.cfg = cfg
        self.cap = int(kv_capacity if kv_capacity is not None else cfg.kv_capacity)
        self.wdtype = 1 if bf16_bits else 0
        wt = np.uint16 if bf16_bits else np.float32
        self._keep = []
        self._layers = (_Layer * cfg.n_layers)()
        for i, lw in enumerate(layers):
            for name, _ in _Layer._fields_:
                a = lw.get(name)
                if a is not None:
                    a = np.ascontiguousarray(a, dtype=wt)
                    self._keep.append(a)
                setattr(self._layers[i], name, None if a is None else a.ctypes.data)
        self.final_norm = None if final_norm is None else np.ascontiguousarray(final_norm, dtype=wt)
        self.lm_head = None if lm_head is None else np.ascontiguousarray(lm_head, dtype=wt)
        self.desc = _Desc(cfg.n_layers, cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn,
                          cfg.vocab if lm_head is not None else 0, self.wdtype, cfg.rms_eps, cfg.rope_theta, self.cap)
        self.kv = np.zeros((cfg.n_layers, 2, cfg.n_kv_heads, self.cap, cfg.head_dim), dtype=np.float64)

    def load_prefix(self, layer, kv_f32):
        """kv_f32: [2, H_kv, >=n, hd]; copies all its slots into the cache of `layer`."""
        n = kv_f32.shape[2]
        self.kv[layer, :, :, :n, :] = kv_f32

    def verify(self, l_glo, l_cache, hidden_in, seg_off, parent):
        hidden_in = _f64(hidden_in)
        l_s = hidden_in.shape[0]
        parent = _i32(parent)
        assert parent.shape[0] >= seg_off + l_s
        out = np.zeros_like(hidden_in)
        _check(lib().orc_verify_stage(C.byref(self.desc), self._layers, _ptr(self.kv), int(l_glo), int(l_cache), _ptr(hidden_in),
                                      int(seg_off), int(l_s), _ptr(parent), _ptr(out)), "orc_verify_stage")
        return out

    def logits(self, hidden):
        hidden = _f64(hidden)
        rows = hidden.shape[0]
        lg = np.zeros((rows, self.cfg.vocab), dtype=np.float32)
        am = np.zeros(rows, dtype=np.int32)
        _check(lib().orc_lm_head(C.byref(self.desc), _ptr(self.final_norm), _ptr(self.lm_head), _ptr(hidden), rows, _ptr(lg), _ptr(am)),
               "orc_lm_head")
        return lg, am


def argmax_rows(logits):
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    am = np.zeros(logits.shape[0], dtype=np.int32)
    lib().orc_argmax_rows(_ptr(logits), logits.shape[0], logits.shape[1], _ptr(am))
    return am


def accept(amax, token, parent, n_ver):
    token, parent = _i32(token), _i32(parent)
    amax = _i32(amax) if n_ver > 0 else np.zeros(1, dtype=np.int32)
    T = token.shape[0]
    res = AcceptResult()
    retain = np.full(T, -1, dtype=np.int32)
    _check(lib().orc_accept(_ptr(amax), _ptr(token), _ptr(parent), T, int(n_ver), C.byref(res), _ptr(retain)), "orc_accept")
    return res, retain[: res.n_retain].copy()


def tree_remap(parent, token, retain, n_acc):
    parent, token, retain = _i32(parent), _i32(token), _i32(retain)
    n = retain.shape[0] - n_acc
    npar = np.zeros(max(n, 1), dtype=np.int32)
    ntok = np.zeros(max(n, 1), dtype=np.int32)
    m = lib().orc_tree_remap(_ptr(parent), _ptr(token), parent.shape[0], _ptr(retain), int(n_acc), retain.shape[0], _ptr(npar), _ptr(ntok))
    return npar[:m].copy(), ntok[:m].copy()


def kv_compact(cache, l_glo, l_cache, retain, n_acc):
    """cache: C-contiguous array [n_layers, 2, H_kv, cap, hd] of any dtype, compacted in place.  Returns (l_glo', l_cache')."""
    assert cache.flags["C_CONTIGUOUS"] and cache.ndim == 5 and cache.shape[1] == 2
    retain = _i32(retain)
    out = np.zeros(2, dtype=np.int32)
    _check(lib().orc_kv_compact(_ptr(cache), C.c_size_t(cache.itemsize), cache.shape[0], cache.shape[2], cache.shape[3], cache.shape[4],
                                int(l_glo), int(l_cache), _ptr(retain), retain.shape[0], int(n_acc), _ptr(out)), "orc_kv_compact")
    return int(out[0]), int(out[1])


def seg_prune(seg, off, retain):
    """seg: [l_s, ...] array of any dtype; off = l_cache - l_glo.  Returns the retained rows in order."""
    seg = np.ascontiguousarray(seg)
    retain = _i32(retain)
    out = np.zeros_like(seg)
    row = seg.itemsize * int(np.prod(seg.shape[1:]))
    n = lib().orc_seg_prune(_ptr(seg), seg.shape[0], C.c_size_t(row), int(off), _ptr(retain), retain.shape[0], _ptr(out))
    return out[:n].copy()


def row_weights(logits_row, inv_temp):
    """Integer probability weights E[v] of one row and their sum Z (the sampling distribution is E / Z)."""
    row = np.ascontiguousarray(logits_row, dtype=np.float32)
    E = np.zeros(row.shape[0], dtype=np.uint64)
    lib().orc_row_weights.restype = C.c_uint64
    Z = lib().orc_row_weights(_ptr(row), row.shape[0], C.c_float(inv_temp), _ptr(E))
    return E, int(Z)


def accept_sample(logits, inv_temp, token, parent, n_ver, seed, step):
    token, parent = _i32(token), _i32(parent)
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T = token.shape[0]
    res = AcceptResult()
    retain = np.full(T, -1, dtype=np.int32)
    _check(lib().orc_accept_sample(_ptr(logits), logits.shape[1], C.c_float(inv_temp), _ptr(token), _ptr(parent), T, int(n_ver),
                                   C.c_uint64(seed), C.c_uint64(step), C.byref(res), _ptr(retain)), "orc_accept_sample")
    return res, retain[: res.n_retain].copy()
