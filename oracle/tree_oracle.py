"""Oracle for the draft-stage tree bookkeeping (Sec. III-B, III-C, III-D).  TEST INFRASTRUCTURE ONLY.

Pure Python over explicit root-to-node token paths, written from the definitions: cumulative score = product of
confidences along the path (Eq. 1); S = top-L0 nodes by cumulative score in descending order; a node of the new
tree is new iff its path is not a path of the pruned tree (N_new of Sec. III-D); S = S_pr || S_app.
"""
from __future__ import annotations


def path_tokens(parent, token, i):
    p = []
    while i >= 0:
        p.append(int(token[i]))
        i = int(parent[i])
    return tuple(reversed(p))


def cumulative_scores(parent, conf):
    """Eq. 1 by walking each node's path (no recurrence): product of the confidences of the path's nodes, root = 1."""
    out = []
    for i in range(len(parent)):
        s, j = 1.0, i
        chain = []
        while j > 0:
            chain.append(j)
            j = int(parent[j])
        for j in reversed(chain):      # multiply from the root down, as the recurrence c(n) * c_cu(parent) does
            s = float(conf[j]) * s
        out.append(s)
    return out


def segment(parent_base, token_base, conf, L0):
    """Top-L0 by cumulative score, descending, ties by lower base index; returns (parent, token, score, base_index)."""
    n = len(parent_base)
    cu = cumulative_scores(parent_base, conf)
    order = sorted(range(n), key=lambda i: (-cu[i], i))[: min(L0, n)]
    rank = {b: j for j, b in enumerate(order)}
    parent = [(-1 if parent_base[b] < 0 else rank[int(parent_base[b])]) for b in order]
    return parent, [int(token_base[b]) for b in order], [cu[b] for b in order], order


def merge(parent_pr, token_pr, parent_new, token_new, limit=-1):
    """S = S_pr || S_app: append the nodes of T_new whose path is not in T_pr (at most `limit`), in T_new's order."""
    parent = [int(p) for p in parent_pr]
    token = [int(t) for t in token_pr]
    paths = {}
    for i in range(len(parent)):
        paths.setdefault(path_tokens(parent, token, i), i)
    app_src, map_new = [], []
    for j in range(len(parent_new)):
        pt = path_tokens(parent_new, token_new, j)
        if pt in paths:
            map_new.append(paths[pt])
            continue
        pj = int(parent_new[j])
        parent_merged = -1 if pj < 0 else map_new[pj]
        if (pj >= 0 and parent_merged < 0) or (limit >= 0 and len(app_src) >= limit):
            map_new.append(-1)
            continue
        parent.append(parent_merged)
        token.append(int(token_new[j]))
        paths[pt] = len(parent) - 1
        map_new.append(len(parent) - 1)
        app_src.append(j)
    return parent, token, app_src, map_new
