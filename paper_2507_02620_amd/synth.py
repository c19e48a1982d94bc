"""Seeded synthetic inputs for the tree-verification stage.

This module only *draws* inputs: tensors of the configured shapes, random draft
trees in descending cumulative-score order, token ids and the planted-acceptance
schedule.  It holds none of the stage's arithmetic (no norm, projection,
attention, accept or compaction logic) and is imported by the tests, the bench
and the smoke check so that the CPU oracle and the HIP path see the same bytes.

Stand-ins: the paper evaluates on public chat / code / maths / summarisation /
QA prompt sets with trained LLaMA2/Vicuna + EAGLE weights (Sec. IV-A).  None of
those is available or reproduced here; tensors below only take their shapes
(decoder width, heads, FFN, vocabulary), and trees take the structure the
drafting stage outputs (Sec. III-B: nodes sorted by descending cumulative
score, Eq. 1, which makes every parent precede its children).
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_CHUNK = 1 << 22  # elements per independently keyed Philox stream


@dataclasses.dataclass(frozen=True)
class StageConfig:
    """Shape of one verification stage and of its workload."""

    name: str
    dtype: str            # "f32" | "bf16": storage type of weights, activations and KV
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int            # 0: stage has no LM head
    l_glo: int            # KV prefix (context) length
    tree_size: int        # nodes of the draft tree (T)
    seg_len: int          # segment length l_s (<= L_max of Sec. III-B)
    max_depth: int
    max_branch: int       # 0: unlimited
    forest: bool = False  # literal "parent uniform in [-1, i-1]" trees (several roots)
    qkv_bias: bool = False
    rms_eps: float = 1e-5
    rope_theta: float = 1e4

    @property
    def kv_capacity(self) -> int:
        return self.l_glo + self.tree_size + self.seg_len

    def with_(self, **kw) -> "StageConfig":
        return dataclasses.replace(self, **kw)


CONFIGS = {
    # tiny fp32 stage
    "C1": StageConfig("C1-tiny-f32", "f32", 1, 256, 4, 4, 64, 688, 1024, 128, 16, 16, 5, 0, forest=True),
    # LLaMA2-7B-shaped 8-layer stage; the 32000-entry head is LLaMA2's and only used when the
    # stage is driven as the last one
    "C2": StageConfig("C2-llama2-7b-bf16", "bf16", 8, 4096, 32, 32, 128, 11008, 32000, 1024, 64, 16, 6, 4),
    "C3": StageConfig("C3-llama2-13b-bf16", "bf16", 10, 5120, 40, 40, 128, 13824, 32000, 2048, 96, 24, 8, 4),
    "C4": StageConfig("C4-qwen2-7b-gqa-bf16", "bf16", 7, 3584, 28, 4, 128, 18944, 152064, 4096, 128, 32, 10, 0,
                      qkv_bias=True, rms_eps=1e-6, rope_theta=1e6),
    # chunked prefill through the same stage (Sec. III-A: the prompt is pushed through the pipeline before drafting starts):
    # a chain of 512 / 1024 rows behind a 1024-token prefix, one segment
    "P1": StageConfig("P1-prefill-chunk512-7b-bf16", "bf16", 8, 4096, 32, 32, 128, 11008, 0, 1024, 512, 512, 512, 1),
    "P2": StageConfig("P2-prefill-chunk1024-7b-bf16", "bf16", 8, 4096, 32, 32, 128, 11008, 0, 1024, 1024, 1024, 1024, 1),
    "C5": StageConfig("C5-longctx-bf16", "bf16", 8, 4096, 32, 32, 128, 11008, 32000, 16384, 256, 64, 12, 4),
}

# tensor ids (second half of the Philox key)
TID_LAYER = 100        # + 16 * layer + slot
TID_FINAL_NORM = 10
TID_LM_HEAD = 11
TID_PREFIX_KV = 20     # + layer
TID_HIDDEN = 30        # + call index
TID_TREE = 40
TID_PLANT = 50
TID_LOGITS = 60

_LAYER_SLOTS = ("rms_attn", "wq", "wk", "wv", "wo", "rms_ffn", "w_gate", "w_up", "w_down", "bq", "bk", "bv")


def _gen(seed: int, tid: int, chunk: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(int(seed) << 32) | int(tid), int(chunk)]))


def normal(seed: int, tid: int, shape, std: float = 1.0, mean: float = 0.0, threads: int = 8, bf16: bool = False) -> np.ndarray:
    """N(mean, std^2) float32 tensor; element values depend only on (seed, tid, flat index).
    bf16=True rounds every value to the nearest bfloat16 (the result stays float32)."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    nchunk = (n + _CHUNK - 1) // _CHUNK

    def fill(c):
        lo = c * _CHUNK
        hi = min(n, lo + _CHUNK)
        v = _gen(seed, tid, c).standard_normal(hi - lo, dtype=np.float32)
        if std != 1.0:
            v *= np.float32(std)
        if mean != 0.0:
            v += np.float32(mean)
        out[lo:hi] = round_bf16(v) if bf16 else v

    if nchunk <= 1:
        for c in range(nchunk):
            fill(c)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(nchunk)))
    return out.reshape(shape)


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


def _bits_chunk(u: np.ndarray) -> np.ndarray:
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def f32_to_bf16_bits(x: np.ndarray, threads: int = 8) -> np.ndarray:
    """bfloat16 bit patterns (uint16) of float32 values, round to nearest even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.reshape(-1).view(np.uint32)
    n = u.shape[0]
    if n <= _CHUNK:
        return _bits_chunk(u).reshape(x.shape)
    out = np.empty(n, dtype=np.uint16)

    def one(c):
        out[c * _CHUNK:(c + 1) * _CHUNK] = _bits_chunk(u[c * _CHUNK:(c + 1) * _CHUNK])

    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(one, range((n + _CHUNK - 1) // _CHUNK)))
    return out.reshape(x.shape)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def storage(cfg: StageConfig, x: np.ndarray) -> np.ndarray:
    """Values as the stage stores them: rounded once to bf16 for bf16 configs (still float32)."""
    return round_bf16(x) if cfg.dtype == "bf16" else np.ascontiguousarray(x, dtype=np.float32)


def layer_weights(cfg: StageConfig, layer: int, seed: int = 0) -> dict:
    """One decoder layer's tensors, row-major [out, in]; N(0, 0.02^2), gains 1 + N(0, 0.02^2)."""
    d, hd = cfg.d_model, cfg.head_dim
    nq, nkv, f = cfg.n_q_heads * hd, cfg.n_kv_heads * hd, cfg.d_ffn
    shapes = {"rms_attn": (d,), "wq": (nq, d), "wk": (nkv, d), "wv": (nkv, d), "wo": (d, nq),
              "rms_ffn": (d,), "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
              "bq": (nq,), "bk": (nkv,), "bv": (nkv,)}
    out = {}
    for slot, name in enumerate(_LAYER_SLOTS):
        if name.startswith("b") and not cfg.qkv_bias:
            out[name] = None
            continue
        mean = 1.0 if name.startswith("rms") else 0.0
        out[name] = normal(seed, TID_LAYER + 16 * layer + slot, shapes[name], 0.02, mean, bf16=cfg.dtype == "bf16")
    return out


def head_weights(cfg: StageConfig, seed: int = 0):
    """(final_norm [d], lm_head [vocab, d]) or (None, None) when the stage has no head."""
    if cfg.vocab <= 0:
        return None, None
    fn = normal(seed, TID_FINAL_NORM, (cfg.d_model,), 0.02, 1.0, bf16=cfg.dtype == "bf16")
    lm = normal(seed, TID_LM_HEAD, (cfg.vocab, cfg.d_model), 0.02, bf16=cfg.dtype == "bf16")
    return fn, lm


_W4_MATRICES = {"wq": "sq", "wk": "sk", "wv": "sv", "wo": "so", "w_gate": "s_gate", "w_up": "s_up", "w_down": "s_down"}
W4_GROUP = 128


def quantize_w4(w: np.ndarray):
    """Group-wise 4-bit storage of a [out, in] matrix: per row and per 128 input columns one bf16 scale (largest
    magnitude of the group / 7) and codes in [0, 15] (nearest multiple of the scale, shifted by 8).
    Returns (codes uint8 [out, in/2], column k even in the low nibble; scales float32 [out, in/128], bf16-exact)."""
    n, k = w.shape
    assert k % W4_GROUP == 0
    g = np.ascontiguousarray(w, dtype=np.float32).reshape(n, k // W4_GROUP, W4_GROUP)
    scale = round_bf16(np.maximum(np.abs(g).max(axis=2), np.float32(1e-8)) / np.float32(7.0))
    q = np.clip(np.rint(g / scale[:, :, None]), -8, 7).astype(np.int16) + 8
    q = q.reshape(n, k // 2, 2).astype(np.uint8)
    return np.ascontiguousarray(q[:, :, 0] | (q[:, :, 1] << 4)), scale


def layer_weights_w4(cfg: StageConfig, layer: int, seed: int = 0) -> dict:
    """layer_weights with the seven matrices in 4-bit group storage: codes under the matrix's name, scales under s*."""
    out = layer_weights(cfg, layer, seed)
    for name, sname in _W4_MATRICES.items():
        out[name], out[sname] = quantize_w4(out[name])
    return out


def head_weights_w4(cfg: StageConfig, seed: int = 0):
    """(final_norm, lm_head codes, lm_head scales)."""
    fn, lm = head_weights(cfg, seed)
    if lm is None:
        return None, None, None
    codes, scales = quantize_w4(lm)
    return fn, codes, scales


def prefix_kv(cfg: StageConfig, layer: int, capacity: int | None = None, seed: int = 0) -> np.ndarray:
    """K and V of one layer, [2, H_kv, capacity, hd]; slots < l_glo are N(0,1) (K taken as already rotated)."""
    cap = cfg.kv_capacity if capacity is None else capacity
    kv = np.zeros((2, cfg.n_kv_heads, cap, cfg.head_dim), dtype=np.float32)
    if cfg.l_glo > 0:
        kv[:, :, : cfg.l_glo, :] = normal(seed, TID_PREFIX_KV + layer, (2, cfg.n_kv_heads, cfg.l_glo, cfg.head_dim), bf16=cfg.dtype == "bf16")
    return kv


def hidden(cfg: StageConfig, rows: int, call: int = 0, seed: int = 0) -> np.ndarray:
    """Hidden states entering the stage for `rows` draft tokens, N(0,1)."""
    return normal(seed, TID_HIDDEN + call, (rows, cfg.d_model), bf16=cfg.dtype == "bf16")


@dataclasses.dataclass
class Tree:
    parent: np.ndarray   # int32 [T], S order, parent[i] < i, parent[0] = -1
    token: np.ndarray    # int32 [T]
    score: np.ndarray    # float64 [T] cumulative score, non-increasing
    depth: np.ndarray    # int32 [T]

    @property
    def size(self) -> int:
        return int(self.parent.shape[0])


def _depths(parent: np.ndarray) -> np.ndarray:
    d = np.zeros(parent.shape[0], dtype=np.int32)
    for i in range(parent.shape[0]):
        d[i] = 0 if parent[i] < 0 else d[parent[i]] + 1
    return d


def random_tree(size: int, max_depth: int, max_branch: int = 0, vocab: int = 32000, seed: int = 0,
                stream: int = 0, forest: bool = False) -> Tree:
    """Random draft tree relabelled in descending cumulative-score order (Sec. III-B, Eq. 1).

    Growth: node i draws its parent uniformly among earlier nodes whose depth and child count
    allow it (forest=True also allows -1 for i > 0, the literal tiny-config recipe).  Each
    node gets a confidence U(0,1) (the root 1.0); the cumulative score is the product along
    the path; a stable descending sort gives S.  Sibling tokens are distinct while the vocabulary allows.
    """
    g = _gen(seed, TID_TREE, stream)
    par = np.full(size, -1, dtype=np.int64)
    dep = np.zeros(size, dtype=np.int64)
    nch = np.zeros(size, dtype=np.int64)
    conf = g.random(size)
    conf[0] = 1.0
    for i in range(1, size):
        ok = [j for j in range(i) if dep[j] + 1 <= max_depth and (max_branch <= 0 or nch[j] < max_branch)]
        cands = ([-1] if forest else []) + ok
        if not cands:
            cands = [-1] if forest else [0]
        p = cands[int(g.integers(0, len(cands)))]
        par[i] = p
        if p >= 0:
            dep[i] = dep[p] + 1
            nch[p] += 1
    return _score_order(par, conf, g, vocab)


def _score_order(par: np.ndarray, conf: np.ndarray, g: np.random.Generator, vocab: int) -> Tree:
    """Relabel a tree (parents before children) in descending cumulative-score order and draw its token ids."""
    size = par.shape[0]
    cum = np.empty(size, dtype=np.float64)
    for i in range(size):
        cum[i] = conf[i] * (cum[par[i]] if par[i] >= 0 else 1.0)
    order = np.argsort(-cum, kind="stable")
    rank = np.empty(size, dtype=np.int64)
    rank[order] = np.arange(size)
    new_par = np.array([(-1 if par[o] < 0 else rank[par[o]]) for o in order], dtype=np.int32)
    assert new_par[0] == -1 and all(new_par[i] < i for i in range(size))
    tok = np.zeros(size, dtype=np.int32)
    used: dict[int, set] = {}
    for i in range(size):
        s = used.setdefault(int(new_par[i]), set())
        while True:
            t = int(g.integers(0, vocab))
            if t not in s or len(s) >= vocab:  # more siblings than token ids: duplicates are unavoidable
                break
        s.add(t)
        tok[i] = t
    return Tree(new_par, tok, cum[order], _depths(new_par))


def spine_tree(size: int, spine: int, vocab: int = 32000, seed: int = 0, stream: int = 0) -> Tree:
    """A deep tree that is not a chain: `spine` nodes in a row (confidences near 1, so the spine keeps a high score),
    every other node a leaf or a short twig under a random earlier node; relabelled in score order like random_tree.
    Stands in for the draft tree of a long greedy continuation with a few alternatives at every depth."""
    assert 1 <= spine <= size
    g = _gen(seed, TID_TREE, 2_000_000 + stream)
    par = np.full(size, -1, dtype=np.int64)
    conf = g.random(size)
    conf[:spine] = 0.9 + 0.1 * conf[:spine]
    conf[0] = 1.0
    for i in range(1, spine):
        par[i] = i - 1
    for i in range(spine, size):
        par[i] = int(g.integers(0, i))
    return _score_order(par, conf, g, vocab)


def config_tree(cfg: StageConfig, seed: int = 0, stream: int = 0) -> Tree:
    return random_tree(cfg.tree_size, cfg.max_depth, cfg.max_branch, max(cfg.vocab, 2), seed, stream, cfg.forest)


def segments(n: int, seg_len: int):
    """Consecutive slices of S of at most seg_len nodes."""
    return [(o, min(seg_len, n - o)) for o in range(0, n, seg_len)]


def plant_path(tree: Tree, n_ver: int, seed: int = 0, step: int = 0, p_stop: float = 0.2, mean_extra: float = 1.0):
    """Pick the (parent, child-token) pairs whose logits get boosted so that acceptance happens.

    Stands in for the acceptance statistics of Table II: from the root, keep descending into a
    random child with a geometric number of accepted draft tokens (mean `mean_extra`); with
    probability `p_stop` the bonus token matches no child (round ends), otherwise it is made to
    match one child of the last accepted node when it has any.  Returns a list of
    (row, token) pairs: row = S index of a verified node, token = id to force as its argmax.
    Rows >= n_ver are skipped (no logits yet).
    """
    g = _gen(seed, TID_PLANT, step)
    children = [[] for _ in range(tree.size)]
    for i in range(1, tree.size):
        if tree.parent[i] >= 0:
            children[tree.parent[i]].append(i)
    pairs = []
    cur = 0
    n_extra = int(g.geometric(1.0 / (1.0 + mean_extra))) - 1
    while n_extra > 0 and cur < n_ver:
        ch = [c for c in children[cur] if c < n_ver]
        if not ch:
            break
        nxt = ch[int(g.integers(0, len(ch)))]
        pairs.append((cur, int(tree.token[nxt])))
        cur = nxt
        n_extra -= 1
    if cur < n_ver:
        stop = g.random() < p_stop
        ch = children[cur]
        if ch and not stop:
            # prefer a child that is not verified yet: that is what a continuing round looks like
            late = [c for c in ch if c >= n_ver] or ch
            nxt = late[int(g.integers(0, len(late)))]
            pairs.append((cur, int(tree.token[nxt])))
        else:
            forbid = {int(tree.token[c]) for c in ch}
            t = int(g.integers(0, 1 << 30))
            while t in forbid:
                t += 1
            pairs.append((cur, -1 - t))  # negative: "any id not among the children", resolved modulo vocab by caller
    return pairs


def resolve_plants(pairs, tree: Tree, vocab: int):
    """Turn plant_path's output into concrete (row, token id) pairs for a given vocabulary."""
    out = []
    for row, tok in pairs:
        if tok >= 0:
            out.append((row, tok))
            continue
        forbid = {int(tree.token[c]) for c in range(tree.size) if tree.parent[c] == row}
        t = (-1 - tok) % vocab
        while t in forbid:
            t = (t + 1) % vocab
        out.append((row, t))
    return out


def random_logits(rows: int, vocab: int, seed: int = 0, stream: int = 0) -> np.ndarray:
    return normal(seed, TID_LOGITS + stream, (rows, vocab))


def extend_tree(parent: np.ndarray, token: np.ndarray, target: int, max_depth: int, max_branch: int, vocab: int, seed: int = 0,
                stream: int = 0):
    """Append random nodes after the retained sequence until the tree has `target` nodes (stand-in for the
    appended segment S_app of context-aware expansion, Sec. III-D: new nodes go behind S_pr, each under an
    existing node).  Returns (parent, token) as int32 arrays."""
    g = _gen(seed, TID_TREE, 1_000_000 + stream)
    par = [int(p) for p in parent]
    tok = [int(t) for t in token]
    dep = list(_depths(np.asarray(par, dtype=np.int32))) if par else []
    nch = [0] * len(par)
    sib: dict[int, set] = {}
    for i, p in enumerate(par):
        if p >= 0:
            nch[p] += 1
        sib.setdefault(p, set()).add(tok[i])
    while len(par) < target:
        i = len(par)
        if i == 0:
            par.append(-1); dep.append(0); nch.append(0); tok.append(int(g.integers(0, vocab)))
            continue
        ok = [j for j in range(i) if dep[j] + 1 <= max_depth and (max_branch <= 0 or nch[j] < max_branch)] or [0]
        p = ok[int(g.integers(0, len(ok)))]
        s = sib.setdefault(p, set())
        while True:
            t = int(g.integers(0, vocab))
            if t not in s or len(s) >= vocab:
                break
        s.add(t)
        par.append(p); dep.append(dep[p] + 1); nch.append(0); nch[p] += 1; tok.append(t)
    return np.asarray(par, dtype=np.int32), np.asarray(tok, dtype=np.int32)
