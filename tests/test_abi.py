"""The C-ABI library loads and exports every symbol include/flowspec.h declares; host-side validation paths
that need no GPU return their error codes.  CPU only (no kernel is launched)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _fs():
    from paper_2507_02620_amd import flowspec as fs
    return fs


def test_every_declared_symbol_is_exported():
    fs = _fs()
    hdr = open(os.path.join(ROOT, "include", "flowspec.h")).read()
    declared = set(re.findall(r"\b(fs_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(fs.EXPORTS)
    for name in declared:
        assert hasattr(fs.lib(), name), name


def test_header_constants_match_binding():
    fs = _fs()
    hdr = open(os.path.join(ROOT, "include", "flowspec.h")).read()
    for name in ("FS_OK", "FS_EINVAL", "FS_ETOPO", "FS_ECAP", "FS_EDTYPE", "FS_EHIP", "FS_EWS", "FS_F32", "FS_BF16", "FS_MAX_TREE",
                 "FS_ARGMAX_CHUNKS"):
        m = re.search(r"#define\s+%s\s+\(?(-?\d+)\)?" % name, hdr)
        assert m and int(m.group(1)) == getattr(fs, name), name
    assert C.sizeof(fs.AcceptResult) == 24 and C.sizeof(fs.StageDesc) == 14 * 4


def test_descriptor_validation_without_gpu():
    fs = _fs()
    good = dict(n_layers=8, d_model=4096, n_q_heads=32, n_kv_heads=32, head_dim=128, d_ffn=11008, vocab=0, dtype=fs.FS_BF16, rms_eps=1e-5,
                rope_theta=1e4, kv_capacity=2048, max_tree=64, max_seg=16, weight_format=0)

    def ws(**kw):
        d = fs.StageDesc(**{**good, **kw})
        return fs.lib().fs_stage_workspace_bytes(C.byref(d))

    n = ws()
    weights = 8 * (3 * 4096 * 4096 + 4096 * 4096 + 3 * 4096 * 11008) * 2
    assert weights <= n < weights * 1.1               # re-tiled weights + a small scratch area
    assert ws(dtype=7) == 0 and ws(head_dim=96) == 0 and ws(n_kv_heads=5) == 0 and ws(max_tree=2000) == 0 and ws(d_model=100) == 0

    def create(**kw):
        d = fs.StageDesc(**{**good, **kw})
        h = C.c_void_p()
        return fs.lib().fs_stage_create(C.byref(d), None, None, None, None, None, 0, None, C.byref(h))

    assert create(dtype=7) == fs.FS_EDTYPE
    assert create(max_tree=4096) == fs.FS_ECAP
    assert create(head_dim=96) == fs.FS_EINVAL
    assert create() == fs.FS_EINVAL                    # no weights given
    assert create(weight_format=1, dtype=fs.FS_F32) == fs.FS_EDTYPE      # 4-bit weights need bf16 activations
    assert create(weight_format=1, d_ffn=11008 + 32) == fs.FS_EINVAL     # ... and 128-column groups
    n4 = ws(weight_format=1)
    assert weights / 4 <= n4 < weights / 4 * 1.2       # codes are a quarter of the bf16 bytes, plus scales and scratch


def test_entry_points_reject_bad_arguments_before_any_gpu_work():
    fs = _fs()
    L = fs.lib()
    kv = fs.KVCache(None, 0, 0, 0, 0)
    par = np.array([-1, 0], dtype=np.int32)
    assert L.fs_tree_verify_stage(None, kv, 0, 0, None, 0, 1, par.ctypes.data_as(C.c_void_p), None, None) == fs.FS_EINVAL
    assert L.fs_tree_logits(None, None, 1, None, None, None) == fs.FS_EINVAL
    assert L.fs_tree_accept(None, None, 0, None, None, 4, 1, None, None, None, None) == fs.FS_EINVAL
    dummy = C.c_void_p(256)
    assert L.fs_tree_accept(None, dummy, 0, dummy, dummy, 5000, 1, dummy, dummy, None, None) == fs.FS_ECAP
    assert L.fs_kv_compact(None, kv, 0, 0, None, None, 0, 0, None, None) == fs.FS_EINVAL
    assert L.fs_seg_prune(dummy, 4, 6, 0, dummy, None, 0, C.c_void_p(512), None, None) == fs.FS_EINVAL   # row_bytes not a multiple of 4
    bad = np.array([3, 1], dtype=np.int32)                                                                    # not ascending
    assert L.fs_seg_prune(dummy, 4, 8, 0, bad.ctypes.data_as(C.c_void_p), None, 2, C.c_void_p(512), None, None) == fs.FS_EINVAL
    assert L.fs_last_hip_error() == 0
