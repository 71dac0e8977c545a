"""Stochastic approval: the model's token at a node is SAMPLED (test infrastructure, not product code).

Sec. 2.4 (Draft Construction and Verification) states the approval rule in its general form: at each
position a token is sampled from the target model's conditional distribution and compared with the draft
token; Sec. 4.4 varies the sampling temperature and top-p.  Greedy decoding is the special case in which
the "sample" is the argmax.  Only the way the model's token at a node is obtained changes; the walk that
compares it with the draft tokens (accept.py) stays the same.

Definition used here (the paper names temperature and top-p and nothing more):
  p_i      = softmax(logits / temperature)_i
  nucleus  = the fewest highest-probability tokens whose probabilities sum to at least top_p;
             tokens whose probability EQUALS that of the last admitted one are all admitted
             (so the set does not depend on how ties are ordered)
  token    = inverse CDF over the nucleus in token-id order: the smallest id j in the nucleus with
             sum_{i in nucleus, i <= j} p_i  >  u * sum_{i in nucleus} p_i,   u in [0, 1) given by the caller
The uniform numbers are inputs: one per tree node, drawn by whoever runs the decoding loop.
"""
from __future__ import annotations

import numpy as np


def nucleus(p: np.ndarray, top_p: float) -> np.ndarray:
    """Boolean mask of the nucleus of a probability vector (see the module text)."""
    order = np.argsort(-p, kind="stable")
    cum = np.cumsum(p[order])
    k = int(np.searchsorted(cum, top_p, side="left"))  # first k with cum[k] >= top_p
    k = min(k, len(p) - 1)
    return p >= p[order[k]]


def sample_top_p(logits: np.ndarray, temperature: float, top_p: float, u: float):
    """One row.  Returns (token, info): info holds the two distances that say how close the decision was to
    flipping: 'nucleus_slack' = how far top_p is from admitting one token fewer or needing one more
    ('edge_mass' = the probability that would then enter or leave the nucleus),
    'cdf_slack' = distance of u from the nearest CDF step (both as probabilities)."""
    x = np.asarray(logits, dtype=np.float64) / float(temperature)
    e = np.exp(x - x.max())
    p = e / e.sum()
    keep = nucleus(p, top_p)
    ids = np.flatnonzero(keep)
    cdf = np.cumsum(p[ids])
    total = cdf[-1]
    j = int(np.searchsorted(cdf, u * total, side="right"))  # first j with cdf[j] > u * total
    j = min(j, len(ids) - 1)
    steps = np.concatenate([[0.0], cdf]) / total
    # how far top_p is from admitting one token fewer / needing one token more
    order = np.argsort(-p, kind="stable")
    cum = np.cumsum(p[order])
    k = min(int(np.searchsorted(cum, top_p, side="left")), len(p) - 1)
    fewer = top_p - cum[k - 1] if k > 0 else np.inf
    more = cum[k] - top_p if k < len(p) - 1 else np.inf
    edge = p[order[k]] + (p[order[k + 1]] if k + 1 < len(p) else 0.0)  # mass that a flipped boundary would move
    info = {"nucleus_size": int(keep.sum()), "cdf_slack": float(np.abs(steps - u).min()),
            "nucleus_slack": float(min(fewer, more)), "edge_mass": float(edge)}
    return int(ids[j]), info


def sample_rows(logits: np.ndarray, temperature: float, top_p: float, u: np.ndarray):
    """Every row of [n][V] with its own uniform number: (tokens [n], list of info dicts)."""
    out = [sample_top_p(logits[i], temperature, top_p, float(u[i])) for i in range(len(logits))]
    return np.array([t for t, _ in out], dtype=np.int64), [i for _, i in out]
