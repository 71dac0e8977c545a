"""Draft approval and cache compaction, reference version (test infrastructure, not product code).

Sec. 2.4: at every position the model's own token is compared with the draft token; a matching draft
token is approved, and from the first mismatch on the draft is discarded.  With greedy sampling
(Sec. 4.1, the experiments' default) the model's token at node i is argmax(logits_i).
"""
from __future__ import annotations

import numpy as np


def argmax_margin(logits: np.ndarray):
    """Per row: index of the maximum (lowest index on exact ties) and top-1 minus top-2."""
    logits = np.asarray(logits)
    if np.isnan(logits).any():
        raise ValueError("NaN in logits")
    a = np.argmax(logits, axis=-1)
    top2 = np.partition(logits, -2, axis=-1)[..., -2:]
    return a.astype(np.int64), (top2[..., 1] - top2[..., 0])


def accept_walk(parent, token, model_token):
    """Longest approved root-to-node path.

    Node i (i > 0) is approved iff its parent is approved and token[i] equals the model's token at
    the parent; the root is always approved.  The chosen end node is the deepest approved node, the
    lowest index among equally deep ones.  Returns (accepted_tokens, path): path = node indices from
    the root to the end node; accepted_tokens = the draft tokens on the path below the root followed
    by the model's token at the end node (so at least one token is always produced)."""
    n = len(parent)
    ok = [False] * n
    depth = [0] * n
    ok[0] = True
    for i in range(1, n):
        p = int(parent[i])
        depth[i] = depth[p] + 1
        ok[i] = ok[p] and int(token[i]) == int(model_token[p])
    best = 0
    for i in range(n):
        if ok[i] and depth[i] > depth[best]:
            best = i
    path = []
    v = best
    while v >= 0:
        path.append(v)
        v = int(parent[v])
    path.reverse()
    accepted = [int(token[v]) for v in path[1:]] + [int(model_token[best])]
    return accepted, path


def compact_rows(prefix_rows: np.ndarray, tree_rows: np.ndarray, path) -> np.ndarray:
    """New cache = old prefix rows followed by the tree rows of the accepted path, in path order."""
    return np.concatenate([prefix_rows, tree_rows[np.asarray(path, dtype=np.int64)]], axis=0)
