"""Seeded synthetic inputs for draft-tree verification (shared by the CPU oracle and the GPU path).

This module holds NO arithmetic of the method itself: it only draws numbers and builds index
structures.  Everything is derived from integer seeds through numpy's counter-based Philox
generator, so the same call returns the same bits on every machine.

What it provides
  * model shapes (the benchmark configurations) and random-init weights, N(0, 0.02),
    optionally rounded once to bf16 (round-to-nearest-even) and kept as uint16 bit patterns;
  * Zipf(1.1) token streams over a permuted vocabulary;
  * a lazily materialised synthetic tri-gram count matrix keyed by the bigram context
    (the drafter's "LLM representative", Sec. 2.2, Eq. (1));
  * draft trees (parent indices + token ids): tri-gram seeded, uniformly random, chains,
    and the exhaustive list of all trees with a given number of nodes;
  * attention-only inputs (q, K, V ~ N(0,1) rounded to bf16).
"""
from __future__ import annotations

import itertools
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

# --------------------------------------------------------------------------------------
# bf16 bit helpers (storage format only)
# --------------------------------------------------------------------------------------


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp32 exactly."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 -> nearest bf16 value, returned as fp32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


# --------------------------------------------------------------------------------------
# model shapes
# --------------------------------------------------------------------------------------


@dataclass(frozen=True)
class ModelConfig:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float = 10000.0
    rms_eps: float = 1e-5
    dtype: str = "bf16"  # "fp32" or "bf16": storage type of weights / KV / GEMM inputs

    @property
    def q_dim(self) -> int:
        return self.n_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def with_layers(self, n_layers: int) -> "ModelConfig":
        return replace(self, n_layers=n_layers, name=f"{self.name}-L{n_layers}")


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration: model shape + prefix / tree / batch sizes."""
    model: ModelConfig
    prefix_len: int
    n_nodes: int  # tree rows fed to the forward, root included
    depth: int  # maximum node depth, root at depth 0
    batch: int = 1
    topk: Tuple[int, ...] = ()  # per-depth child cap of the tri-gram tree


TINY = ModelConfig("tiny", 2, 256, 4, 4, 64, 688, 4096, dtype="fp32")
LLAMA2_7B = ModelConfig("llama2-7b", 32, 4096, 32, 32, 128, 11008, 32000)
LLAMA2_13B = ModelConfig("llama2-13b", 40, 5120, 40, 40, 128, 13824, 32000)
LLAMA3_8B = ModelConfig("llama3-8b", 32, 4096, 32, 8, 128, 14336, 128256, rope_base=500000.0)
ATTN_ONLY = ModelConfig("attn-only", 1, 4096, 32, 32, 128, 0, 0)

WORKLOADS: Dict[str, Workload] = {
    "c1": Workload(TINY, 128, 16, 4, 1, (4, 2, 1, 1)),
    "c2": Workload(ATTN_ONLY, 4096, 64, 8, 1),
    "c3": Workload(LLAMA2_7B, 1024, 64, 6, 1, (4, 4, 4, 4, 4, 4)),
    "c4": Workload(LLAMA2_13B, 2048, 128, 8, 4, (4,) * 8),
    "c5": Workload(LLAMA3_8B, 16384, 256, 10, 8, (4,) * 10),
}


# --------------------------------------------------------------------------------------
# random numbers
# --------------------------------------------------------------------------------------


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream)]))


def _stream_id(*parts: int) -> int:
    """Mix small integers into one 64-bit stream id (splitmix64 finaliser; not cryptographic)."""
    h = 0x9E3779B97F4A7C15
    for p in parts:
        h = (h ^ (int(p) & 0xFFFFFFFFFFFFFFFF)) & 0xFFFFFFFFFFFFFFFF
        h = (h + 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF
        z = h
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
        h = z ^ (z >> 31)
    return h


def normal_matrix(seed: int, stream: int, shape: Sequence[int], std: float, dtype: str) -> np.ndarray:
    """i.i.d. N(0, std) drawn in fp32 (one Philox stream per matrix, filled in 1 Mi-element blocks);
    dtype 'bf16' -> uint16 bit patterns (one RNE rounding)."""
    g = _rng(seed, stream)
    n = int(np.prod(shape))
    blk = 1 << 20
    if dtype != "bf16":
        out = np.empty(n, np.float32)
        for s in range(0, n, blk):
            f = out[s:min(s + blk, n)]
            g.standard_normal(out=f, dtype=np.float32)
            f *= np.float32(std)
        return out.reshape(tuple(shape))
    out = np.empty(n, np.uint16)
    buf = np.empty(blk, np.float32)
    tmp = np.empty(blk, np.uint32)
    for s in range(0, n, blk):
        e = min(s + blk, n)
        f, t = buf[: e - s], tmp[: e - s]
        g.standard_normal(out=f, dtype=np.float32)
        f *= np.float32(std)
        u = f.view(np.uint32)  # round to nearest even on the bit pattern
        np.right_shift(u, 16, out=t)
        t &= 1
        t += 0x7FFF
        t += u
        t >>= 16
        out[s:e] = t
    return out.reshape(tuple(shape))


# --------------------------------------------------------------------------------------
# weights
# --------------------------------------------------------------------------------------

# Every linear map is stored [out_features][in_features], row-major (y = W x).
_LAYER_MATS = ("wq", "wk", "wv", "wo", "wg", "wu", "wd")


def _layer_shapes(cfg: ModelConfig) -> Dict[str, Tuple[int, int]]:
    return {
        "wq": (cfg.q_dim, cfg.d_model),
        "wk": (cfg.kv_dim, cfg.d_model),
        "wv": (cfg.kv_dim, cfg.d_model),
        "wo": (cfg.d_model, cfg.q_dim),
        "wg": (cfg.d_ffn, cfg.d_model),
        "wu": (cfg.d_ffn, cfg.d_model),
        "wd": (cfg.d_model, cfg.d_ffn),
    }


def make_weights(cfg: ModelConfig, seed: int = 0, gain_jitter: float = 0.0, std: float = 0.02,
                 threads: int = 8) -> dict:
    """Random-init weights.  Matrices ~ N(0, std) in cfg.dtype storage; norm gains are fp32,
    equal to 1 (or 1 + N(0, gain_jitter), which lets a parity test notice a dropped gain)."""
    shapes = _layer_shapes(cfg)

    def gain(stream):
        g = np.ones(cfg.d_model, dtype=np.float32)
        if gain_jitter:
            g += _rng(seed, stream).standard_normal(cfg.d_model, dtype=np.float32) * np.float32(gain_jitter)
        return g

    jobs = [(li, mi, name) for li in range(cfg.n_layers) for mi, name in enumerate(_LAYER_MATS)]

    def draw(job):
        li, mi, name = job
        return normal_matrix(seed, _stream_id(1, li, mi), shapes[name], std, cfg.dtype)

    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        mats = list(ex.map(draw, jobs))
        top = list(ex.map(lambda i: normal_matrix(seed, _stream_id(3, i), (cfg.vocab, cfg.d_model), std, cfg.dtype),
                          range(2)))
    layers = []
    for li in range(cfg.n_layers):
        lw = {name: mats[li * len(_LAYER_MATS) + mi] for mi, name in enumerate(_LAYER_MATS)}
        lw["norm_attn"] = gain(_stream_id(2, li, 0))
        lw["norm_ffn"] = gain(_stream_id(2, li, 1))
        layers.append(lw)
    w = {"layers": layers}
    w["emb"], w["lm_head"] = top
    w["final_norm"] = gain(_stream_id(2, 1 << 20, 0))
    return w


# --------------------------------------------------------------------------------------
# tokens
# --------------------------------------------------------------------------------------


class ZipfVocab:
    """Zipf(s) over ranks 1..V, ranks mapped to token ids by a seeded permutation."""

    def __init__(self, vocab: int, seed: int = 0, s: float = 1.1):
        self.vocab = vocab
        w = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
        self.cdf = np.cumsum(w)
        self.cdf /= self.cdf[-1]
        self.perm = _rng(seed, _stream_id(10, vocab)).permutation(vocab).astype(np.int32)

    def draw(self, g: np.random.Generator, n: int) -> np.ndarray:
        ranks = np.searchsorted(self.cdf, g.random(n), side="left")
        return self.perm[np.minimum(ranks, self.vocab - 1)]


def zipf_tokens(vocab: int, n: int, seed: int = 0, stream: int = 0, s: float = 1.1) -> np.ndarray:
    """n i.i.d. Zipf(s) token ids (int32)."""
    return ZipfVocab(vocab, seed, s).draw(_rng(seed, _stream_id(11, stream)), n).astype(np.int32)


# --------------------------------------------------------------------------------------
# synthetic tri-gram matrix
# --------------------------------------------------------------------------------------


class SyntheticTrigram:
    """A fixed sparse tri-gram count matrix, materialised row by row on demand.

    Row (a, b) = bigram context; it holds m in [2, 8] distinct successor tokens drawn Zipf(1.1)
    with Zipf-distributed integer counts.  successors(a, b) returns (tokens, probabilities) with
    probabilities count / sum(count) as in Eq. (1), sorted by probability (ties: lower id first).
    """

    def __init__(self, vocab: int, seed: int = 0):
        self.vocab = vocab
        self.seed = seed
        self.zipf = ZipfVocab(vocab, seed)

    def successors(self, a: int, b: int) -> Tuple[np.ndarray, np.ndarray]:
        g = _rng(self.seed, _stream_id(20, a, b))
        m = int(g.integers(2, 9))
        toks: List[int] = []
        while len(toks) < m:
            for t in self.zipf.draw(g, m):
                if int(t) not in toks and len(toks) < m:
                    toks.append(int(t))
        counts = np.floor(1.0 / np.maximum(g.random(m), 1e-3) ** (1 / 1.1)).astype(np.int64) + 12
        order = sorted(range(m), key=lambda i: (-int(counts[i]), toks[i]))
        toks_s = np.array([toks[i] for i in order], dtype=np.int32)
        cnt_s = counts[order].astype(np.float64)
        return toks_s, cnt_s / cnt_s.sum()


# --------------------------------------------------------------------------------------
# trees
# --------------------------------------------------------------------------------------


def tree_depths(parent: Sequence[int]) -> np.ndarray:
    d = np.zeros(len(parent), dtype=np.int32)
    for i in range(1, len(parent)):
        d[i] = d[parent[i]] + 1
    return d


def chain_tree(n: int) -> np.ndarray:
    """parent array of a single chain 0 <- 1 <- ... <- n-1."""
    return np.arange(-1, n - 1, dtype=np.int32)


def all_trees(n: int) -> List[np.ndarray]:
    """Every parent array with parent[0] = -1 and 0 <= parent[i] < i ((n-1)! of them)."""
    out = []
    for combo in itertools.product(*[range(i) for i in range(1, n)]):
        out.append(np.array((-1,) + combo, dtype=np.int32))
    return out


def random_tree(n: int, depth: Optional[int], seed: int = 0) -> np.ndarray:
    """parent[i] ~ U{0..i-1}; redrawn with the next stream until the maximum depth equals `depth`."""
    for attempt in range(100000):
        g = _rng(seed, _stream_id(30, n, attempt))
        parent = np.full(n, -1, dtype=np.int32)
        for i in range(1, n):
            parent[i] = int(g.integers(0, i))
        if depth is None or int(tree_depths(parent).max()) == depth:
            return parent
    raise RuntimeError("no tree of the requested depth found")


def trigram_tree(tri: SyntheticTrigram, prev_token: int, root_token: int, n_nodes: int, depth: int,
                 topk: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """Draft tree of exactly n_nodes rows (root included) and maximum depth `depth`.

    Children of node v are the top-k[depth(v)] successors of the context (token[parent(v)], token[v])
    (the root's context is (prev_token, root_token)).  The greedy top-1 chain down to `depth` is
    always kept; the remaining rows are the candidates with the largest path probability.  Nodes are
    renumbered breadth-first so that parent[i] < i."""
    # candidate nodes: (path_prob, parent_candidate_index, token, depth, is_chain)
    cands = [(1.0, -1, int(root_token), 0, True)]
    ctx = [(int(prev_token), int(root_token))]
    frontier = [0]
    for dep in range(depth):
        k = topk[dep] if dep < len(topk) else topk[-1]
        nxt = []
        for ci in frontier:
            toks, probs = tri.successors(*ctx[ci])
            for j in range(min(k, len(toks))):
                cands.append((cands[ci][0] * float(probs[j]), ci, int(toks[j]), dep + 1,
                              cands[ci][4] and j == 0))
                ctx.append((ctx[ci][1], int(toks[j])))
                nxt.append(len(cands) - 1)
        frontier = nxt
    keep = {i for i, c in enumerate(cands) if c[4]}
    if len(keep) > n_nodes:
        raise ValueError("n_nodes smaller than the forced chain")
    # best-first: a candidate is eligible once its parent is kept
    order = sorted((i for i in range(len(cands)) if i not in keep), key=lambda i: (-cands[i][0], i))
    while len(keep) < n_nodes:
        for i in order:
            if i not in keep and cands[i][1] in keep:
                keep.add(i)
                break
        else:
            raise ValueError("tri-gram expansion too small for the requested n_nodes; raise topk")
    # breadth-first renumbering (by depth, then candidate index)
    kept = sorted(keep, key=lambda i: (cands[i][3], i))
    new_id = {old: new for new, old in enumerate(kept)}
    parent = np.array([-1 if cands[o][1] < 0 else new_id[cands[o][1]] for o in kept], dtype=np.int32)
    token = np.array([cands[o][2] for o in kept], dtype=np.int32)
    return parent, token


def workload_tree(wl: Workload, seed: int = 0, seq: int = 0) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(prefix_tokens, parent, token) for one sequence of a model workload (c1, c3, c4, c5)."""
    V = wl.model.vocab
    toks = zipf_tokens(V, wl.prefix_len + 1, seed, stream=seq)
    prefix, root = toks[:-1], int(toks[-1])
    tri = SyntheticTrigram(V, seed)
    prev = int(prefix[-1]) if wl.prefix_len else 0
    parent, token = trigram_tree(tri, prev, root, wl.n_nodes, wl.depth, wl.topk)
    return prefix.astype(np.int32), parent, token


# --------------------------------------------------------------------------------------
# attention-only inputs
# --------------------------------------------------------------------------------------


def attention_inputs(n_heads: int, n_kv_heads: int, head_dim: int, prefix_len: int, n_nodes: int,
                     seed: int = 0, dtype: str = "bf16") -> Dict[str, np.ndarray]:
    """q [N][H][hd], prefix K/V [Hkv][P][hd], tree K/V [Hkv][N][hd]; all N(0,1) in `dtype` storage."""
    def draw(stream, shape):
        return normal_matrix(seed, _stream_id(40, stream), shape, 1.0, dtype)
    return {
        "q": draw(0, (n_nodes, n_heads, head_dim)),
        "k_prefix": draw(1, (n_kv_heads, prefix_len, head_dim)),
        "v_prefix": draw(2, (n_kv_heads, prefix_len, head_dim)),
        "k_tree": draw(3, (n_kv_heads, n_nodes, head_dim)),
        "v_tree": draw(4, (n_kv_heads, n_nodes, head_dim)),
    }
