"""fp64 reference of the verification forward pass (test infrastructure, not product code).

The verification step of Sec. 2.4 (Draft Construction and Verification) feeds the target model one
pseudo-sequence that holds every draft token once, with an attention mask under which a draft token
sees the context and its own ancestors only.  The target models are Llama-2 / Vicuna decoders
(Sec. 4.1, Models and Datasets): pre-norm blocks, RMSNorm, rotary positions on q and k, causal
soft-max attention (optionally grouped-query), SwiGLU feed-forward, final RMSNorm, untied LM head.

Everything here is the plain definition in fp64: explicit boolean masks, exp(s - max) / sum soft-max,
no blocking, no online soft-max, no cache aliasing.  Weights arrive as fp32 arrays or as bf16 bit
patterns (uint16) and are widened exactly.

Model container (built by ded_inputs.make_weights):
  w["emb"] [V][d], w["lm_head"] [V][d], w["final_norm"] [d],
  w["layers"][l] = {wq [H*hd][d], wk, wv [Hkv*hd][d], wo [d][H*hd], wg, wu [F][d], wd [d][F],
                    norm_attn [d], norm_ffn [d]}          (every linear map is y = W x)
cfg needs: n_layers, d_model, n_heads, n_kv_heads, head_dim, rope_base, rms_eps.
"""
from __future__ import annotations

import numpy as np


def _widen_block(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def widen(a: np.ndarray) -> np.ndarray:
    """Exact conversion to fp64.  uint16 arrays are bf16 bit patterns.  (Large matrices are converted
    in row blocks on a few threads; the arithmetic is the same element-wise widening.)"""
    a = np.asarray(a)
    if a.ndim == 2 and a.size >= (1 << 24):
        from concurrent.futures import ThreadPoolExecutor
        out = np.empty(a.shape, dtype=np.float64)
        step = max(1, (1 << 22) // a.shape[1])

        def job(r0):
            out[r0:r0 + step] = _widen_block(a[r0:r0 + step])
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(job, range(0, a.shape[0], step)))
        return out
    return _widen_block(a)


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """y = x / sqrt(mean(x^2) + eps) * gain, over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * widen(gain)


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding, "rotate-half" pairing: element i is paired with i + hd/2 and the pair is
    rotated by the angle pos * base^(-2i/hd).  x: [n][heads][hd], pos: [n]."""
    hd = x.shape[-1]
    half = hd // 2
    theta = base ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = np.asarray(pos, dtype=np.float64)[:, None, None] * theta[None, None, :]
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(a: np.ndarray) -> np.ndarray:
    return a / (1.0 + np.exp(-a))


def masked_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, visible: np.ndarray) -> np.ndarray:
    """out[i,h] = sum_j softmax_j(q[i,h].k[j,g(h)] / sqrt(hd) over visible[i,j]) v[j,g(h)].

    q [n][H][hd]; k, v [m][Hkv][hd]; visible bool [n][m]; query head h reads KV head
    g(h) = floor(h * Hkv / H).  Every row must see at least one key."""
    n, H, hd = q.shape
    Hkv = k.shape[1]
    out = np.empty((n, H, hd), dtype=np.float64)
    for h in range(H):
        g = (h * Hkv) // H
        s = q[:, h, :] @ k[:, g, :].T / np.sqrt(float(hd))
        s = np.where(visible, s, -np.inf)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ v[:, g, :]
    return out


def node_depths(parent) -> np.ndarray:
    """depth[0] = 0, depth[i] = depth[parent[i]] + 1 (parents precede children)."""
    parent = np.asarray(parent)
    d = np.zeros(len(parent), dtype=np.int64)
    for i in range(1, len(parent)):
        d[i] = d[parent[i]] + 1
    return d


def ancestor_mask(parent) -> np.ndarray:
    """A[i][j] = True iff j == i or j is an ancestor of i (the tree-attention mask of Sec. 2.4)."""
    n = len(parent)
    A = np.zeros((n, n), dtype=bool)
    for i in range(n):
        j = i
        while j >= 0:
            A[i, j] = True
            j = int(parent[j])
    return A


def forward_rows(cfg, w, tokens, pos, visible, prefix_k=None, prefix_v=None):
    """Decoder forward over n rows that attend to P given prefix keys plus each other.

    tokens [n], pos [n] (absolute positions), visible bool [n][P + n] (columns: the P prefix keys,
    then the n rows themselves).  prefix_k / prefix_v: per layer [P][Hkv][hd] (keys already rotated),
    or None when P == 0.  Returns (logits [n][V], k_rows, v_rows) with k_rows[l] [n][Hkv][hd]."""
    n = len(tokens)
    H, Hkv, hd = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    x = widen(w["emb"][np.asarray(tokens)])
    k_rows, v_rows = [], []
    for l, lw in enumerate(w["layers"]):
        y = rmsnorm(x, lw["norm_attn"], cfg.rms_eps)
        q = (y @ widen(lw["wq"]).T).reshape(n, H, hd)
        k = (y @ widen(lw["wk"]).T).reshape(n, Hkv, hd)
        v = (y @ widen(lw["wv"]).T).reshape(n, Hkv, hd)
        q = rope(q, pos, cfg.rope_base)
        k = rope(k, pos, cfg.rope_base)
        k_rows.append(k)
        v_rows.append(v)
        if prefix_k is not None and len(prefix_k[l]):
            k_all = np.concatenate([widen(prefix_k[l]), k], axis=0)
            v_all = np.concatenate([widen(prefix_v[l]), v], axis=0)
        else:
            k_all, v_all = k, v
        o = masked_attention(q, k_all, v_all, visible).reshape(n, H * hd)
        x = x + o @ widen(lw["wo"]).T
        y = rmsnorm(x, lw["norm_ffn"], cfg.rms_eps)
        hgate = silu(y @ widen(lw["wg"]).T) * (y @ widen(lw["wu"]).T)
        x = x + hgate @ widen(lw["wd"]).T
    logits = rmsnorm(x, w["final_norm"], cfg.rms_eps) @ widen(w["lm_head"]).T
    return logits, k_rows, v_rows


def prefill(cfg, w, tokens):
    """Plain causal forward over `tokens` at positions 0..P-1: (logits [P][V], k, v per layer)."""
    P = len(tokens)
    vis = np.tril(np.ones((P, P), dtype=bool))
    return forward_rows(cfg, w, tokens, np.arange(P), vis)


def verify_tree(cfg, w, parent, token, prefix_k=None, prefix_v=None):
    """One verification forward (Sec. 2.4): every tree node attends to the whole prefix and to its
    ancestors-or-self; node i sits at position P + depth(i).  Node 0 is the root (the last committed
    token, whose K/V is not in the prefix yet).  Returns (logits [N][V], k_rows, v_rows)."""
    N = len(parent)
    P = 0 if prefix_k is None else len(prefix_k[0])
    vis = np.concatenate([np.ones((N, P), dtype=bool), ancestor_mask(parent)], axis=1)
    pos = P + node_depths(parent)
    return forward_rows(cfg, w, token, pos, vis, prefix_k, prefix_v)


# ---------------------------------------------------------------------------------------------
# Plain autoregressive decoding, one token at a time, written without any mask: the new token's
# query simply attends to every key cached so far.  Used by the invariants only.
# ---------------------------------------------------------------------------------------------


def _ar_token(cfg, w, tok, position, cache_k, cache_v):
    H, Hkv, hd = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    x = widen(w["emb"][int(tok)])
    p = np.array([position])
    for l, lw in enumerate(w["layers"]):
        y = rmsnorm(x, lw["norm_attn"], cfg.rms_eps)
        q = rope((widen(lw["wq"]) @ y).reshape(1, H, hd), p, cfg.rope_base)[0]
        k = rope((widen(lw["wk"]) @ y).reshape(1, Hkv, hd), p, cfg.rope_base)[0]
        v = (widen(lw["wv"]) @ y).reshape(Hkv, hd)
        cache_k[l].append(k)
        cache_v[l].append(v)
        K = np.stack(cache_k[l])  # [t][Hkv][hd]
        Vv = np.stack(cache_v[l])
        o = np.empty((H, hd))
        for h in range(H):
            g = (h * Hkv) // H
            s = K[:, g, :] @ q[h] / np.sqrt(float(hd))
            e = np.exp(s - s.max())
            o[h] = (e / e.sum()) @ Vv[:, g, :]
        x = x + widen(lw["wo"]) @ o.reshape(-1)
        y = rmsnorm(x, lw["norm_ffn"], cfg.rms_eps)
        x = x + widen(lw["wd"]) @ (silu(widen(lw["wg"]) @ y) * (widen(lw["wu"]) @ y))
    return widen(w["lm_head"]) @ rmsnorm(x, w["final_norm"], cfg.rms_eps)


def autoregressive_logits(cfg, w, tokens):
    """Feed `tokens` one at a time; returns logits [len(tokens)][V] (row t predicts token t+1)."""
    ck = [[] for _ in w["layers"]]
    cv = [[] for _ in w["layers"]]
    return np.stack([_ar_token(cfg, w, t, i, ck, cv) for i, t in enumerate(tokens)])


def autoregressive_decode(cfg, w, tokens, n_new):
    """Greedy decoding: after consuming `tokens`, emit n_new tokens (lowest id on exact ties)."""
    ck = [[] for _ in w["layers"]]
    cv = [[] for _ in w["layers"]]
    logits = None
    for i, t in enumerate(tokens):
        logits = _ar_token(cfg, w, t, i, ck, cv)
    out = []
    for j in range(n_new):
        nxt = int(np.argmax(logits))
        out.append(nxt)
        if j + 1 < n_new:
            logits = _ar_token(cfg, w, nxt, len(tokens) + j, ck, cv)
    return out
