"""ctypes binding of libded_verify.so: argument marshalling only.

Module-level functions carry the names of the C entry points (include/ded_verify.h) and take raw
pointers / numpy arrays; `Verifier` is a convenience holder that allocates the device buffers with
torch (device memory and streams are all torch is used for) and keeps them alive.
The library is required: importing works without it, but every call raises if it is not built.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# DED_VERIFY_LIB names another build of the same library (the host-sanitizer build of the CPU test tier)
LIB_PATH = os.environ.get("DED_VERIFY_LIB") or os.path.join(_HERE, "libded_verify.so")

DED_OK, DED_EINVAL, DED_ETREE, DED_ETOKEN, DED_ECAP, DED_ESTATE, DED_EHIP, DED_ENOMEM, DED_ENONFINITE = 0, -1, -2, -3, -4, -5, -6, -7, -8
DED_F32, DED_BF16 = 0, 1

EXPORTS = [
    "ded_workspace_bytes", "ded_kv_layer_bytes", "ded_validate_tree", "ded_build_tree", "ded_verify_init", "ded_verify_free",
    "ded_verify_step", "ded_sample", "ded_accept", "ded_get_argmax", "ded_kv_store", "ded_kv_load", "ded_tree_attention",
    "ded_tree_attention_static", "ded_static_scratch_bytes", "ded_probe_stream_read",
    "ded_profile_enable", "ded_profile_read", "ded_strerror",
    "ded_trigram_create", "ded_trigram_free", "ded_trigram_count", "ded_trigram_finalize", "ded_trigram_adjust",
    "ded_trigram_lookup", "ded_trigram_size", "ded_draft_mcts",
]


class ded_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rope_base", C.c_float), ("rms_eps", C.c_float)] + \
               [(n, C.c_int32) for n in ("dtype", "max_batch", "kv_capacity", "max_nodes")]


class ded_weights(C.Structure):
    _fields_ = [("emb", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p),
                ("wqkv", C.POINTER(C.c_void_p)), ("wo", C.POINTER(C.c_void_p)),
                ("wgate_up", C.POINTER(C.c_void_p)), ("wdown", C.POINTER(C.c_void_p)),
                ("norm_attn", C.POINTER(C.c_void_p)), ("norm_ffn", C.POINTER(C.c_void_p))]


class ded_kv(C.Structure):
    _fields_ = [("k", C.POINTER(C.c_void_p)), ("v", C.POINTER(C.c_void_p))]


class DedError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {ded_strerror(code)} ({code})")


_lib = None


def lib() -> C.CDLL:
    """Loads the shared library (built in-tree by __graft_entry__.build()); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        # torch ships its own HIP runtime.  It has to be in the process before this library is, so that both use
        # the same one; loaded the other way round, device pointers allocated by torch are unknown to the runtime
        # this library would have pulled in, and every call that takes one fails.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = C.CDLL(LIB_PATH)
        i32p, vp = C.POINTER(C.c_int32), C.c_void_p
        L.ded_workspace_bytes.restype = C.c_size_t
        L.ded_workspace_bytes.argtypes = [C.POINTER(ded_config)]
        L.ded_kv_layer_bytes.restype = C.c_size_t
        L.ded_kv_layer_bytes.argtypes = [C.POINTER(ded_config)]
        L.ded_validate_tree.restype = C.c_int
        L.ded_validate_tree.argtypes = [C.POINTER(ded_config), C.c_int32, i32p, i32p, i32p, i32p]
        L.ded_sample.restype = C.c_int
        L.ded_sample.argtypes = [vp, C.c_float, C.c_float, C.POINTER(C.c_float)]
        L.ded_build_tree.restype = C.c_int
        L.ded_build_tree.argtypes = [C.c_int32, C.c_int32, i32p, i32p, C.c_int32, C.c_int32, i32p, i32p, i32p, i32p]
        f64p = C.POINTER(C.c_double)
        L.ded_trigram_create.restype = vp
        L.ded_trigram_create.argtypes = []
        L.ded_trigram_free.restype = None
        L.ded_trigram_free.argtypes = [vp]
        L.ded_trigram_count.restype = C.c_int
        L.ded_trigram_count.argtypes = [vp, i32p, C.c_int64, C.c_int64]
        L.ded_trigram_finalize.restype = C.c_int
        L.ded_trigram_finalize.argtypes = [vp, C.c_int32]
        L.ded_trigram_adjust.restype = C.c_int
        L.ded_trigram_adjust.argtypes = [vp, i32p, C.c_int64, C.c_int64, C.c_double, C.c_double]
        L.ded_trigram_lookup.restype = C.c_int
        L.ded_trigram_lookup.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, i32p, f64p, i32p]
        L.ded_trigram_size.restype = C.c_int64
        L.ded_trigram_size.argtypes = [vp]
        L.ded_draft_mcts.restype = C.c_int
        L.ded_draft_mcts.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_double, C.c_double,
                                     f64p, C.c_int64, i32p, i32p, f64p, i32p]
        L.ded_verify_init.restype = C.c_int
        L.ded_verify_init.argtypes = [C.POINTER(ded_config), C.POINTER(ded_weights), C.POINTER(ded_kv), vp,
                                      C.c_size_t, vp, C.POINTER(vp)]
        L.ded_verify_free.restype = None
        L.ded_verify_free.argtypes = [vp]
        L.ded_verify_step.restype = C.c_int
        L.ded_verify_step.argtypes = [vp, C.c_int32, i32p, i32p, i32p, i32p, vp]
        L.ded_accept.restype = C.c_int
        L.ded_accept.argtypes = [vp, C.c_int32, i32p, i32p, i32p, i32p]
        L.ded_get_argmax.restype = C.c_int
        L.ded_get_argmax.argtypes = [vp, i32p, C.POINTER(C.c_float)]
        for name in ("ded_kv_store", "ded_kv_load"):
            f = getattr(L, name)
            f.restype = C.c_int
            f.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp, vp]
        for name in ("ded_tree_attention", "ded_tree_attention_static"):
            f = getattr(L, name)
            f.restype = C.c_int
            f.argtypes = [vp, C.c_int32, C.c_int32, i32p, i32p, i32p, vp, vp, vp, vp]
        L.ded_static_scratch_bytes.restype = C.c_size_t
        L.ded_static_scratch_bytes.argtypes = []
        L.ded_probe_stream_read.restype = C.c_int
        L.ded_probe_stream_read.argtypes = [vp, C.c_size_t, vp, vp]
        L.ded_profile_enable.restype = C.c_int
        L.ded_profile_enable.argtypes = [vp, C.c_int32]
        L.ded_profile_read.restype = C.c_int
        L.ded_profile_read.argtypes = [vp, C.c_int32, C.POINTER(C.c_char_p), C.POINTER(C.c_double),
                                       C.POINTER(C.c_int64)]
        L.ded_strerror.restype = C.c_char_p
        L.ded_strerror.argtypes = [C.c_int]
        _lib = L
    return _lib


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p32(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.POINTER(C.c_int32))


def make_config(n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab, rope_base, rms_eps, dtype,
                max_batch, kv_capacity, max_nodes) -> ded_config:
    dt = {"fp32": DED_F32, "bf16": DED_BF16}.get(dtype, dtype)
    return ded_config(n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab, rope_base, rms_eps, dt,
                      max_batch, kv_capacity, max_nodes)


# ---- same-named wrappers -------------------------------------------------------------------


def ded_strerror(code: int) -> str:
    return lib().ded_strerror(int(code)).decode()


def ded_workspace_bytes(cfg: ded_config) -> int:
    return int(lib().ded_workspace_bytes(C.byref(cfg)))


def ded_kv_layer_bytes(cfg: ded_config) -> int:
    return int(lib().ded_kv_layer_bytes(C.byref(cfg)))


def ded_validate_tree(cfg: ded_config, prefix_len, n_nodes, parent, token) -> int:
    """parent / token: [batch][max_nodes] int arrays (or None to exercise the null check)."""
    pl, nn = _i32(prefix_len), _i32(n_nodes)
    par = None if parent is None else _i32(parent)
    tok = None if token is None else _i32(token)
    return int(lib().ded_validate_tree(C.byref(cfg), len(pl), _p32(pl), _p32(nn), _p32(par), _p32(tok)))


def ded_build_tree(root_token: int, candidates, max_nodes: int):
    """candidates: ranked sequences of token ids.  Returns (rc, parent, token, cand_end) with parent / token
    cut to the nodes written."""
    n = len(candidates)
    lens = _i32([len(c) for c in candidates]) if n else np.zeros(1, np.int32)
    max_len = int(max([len(c) for c in candidates], default=0))
    toks = np.zeros((max(n, 1), max(max_len, 1)), np.int32)
    for i, c in enumerate(candidates):
        toks[i, : len(c)] = np.asarray(c, dtype=np.int32)
    parent = np.zeros(max(max_nodes, 1), np.int32)
    token = np.zeros(max(max_nodes, 1), np.int32)
    end = np.zeros(max(n, 1), np.int32)
    nn = C.c_int32(0)
    rc = int(lib().ded_build_tree(int(root_token), n, _p32(lens), _p32(toks), max(max_len, 1) if n else 0, int(max_nodes),
                                  _p32(parent), _p32(token), _p32(end), C.byref(nn)))
    return rc, parent[: nn.value].copy(), token[: nn.value].copy(), end[:n].copy()


class Drafter:
    """The CPU draft maker behind the C-ABI: tri-gram matrix + tree search (argument marshalling only)."""

    def __init__(self):
        self._m = lib().ded_trigram_create()
        if not self._m:
            raise DedError(DED_ENOMEM, "ded_trigram_create")

    def close(self):
        if getattr(self, "_m", None):
            lib().ded_trigram_free(self._m)
            self._m = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @staticmethod
    def _check(rc, where):
        if rc != DED_OK:
            raise DedError(rc, where)

    def count(self, tokens, times: int = 1):
        t = _i32(tokens)
        self._check(lib().ded_trigram_count(self._m, _p32(t), len(t), int(times)), "ded_trigram_count")

    def finalize(self, t: int = 12):
        self._check(lib().ded_trigram_finalize(self._m, int(t)), "ded_trigram_finalize")

    def adjust(self, tokens, max_length: int, increment: float, max_prob: float):
        t = _i32(tokens)
        self._check(lib().ded_trigram_adjust(self._m, _p32(t), len(t), int(max_length), float(increment),
                                             float(max_prob)), "ded_trigram_adjust")

    def successors(self, w0: int, w1: int):
        n = C.c_int32(0)
        self._check(lib().ded_trigram_lookup(self._m, int(w0), int(w1), 0, None, None, C.byref(n)), "ded_trigram_lookup")
        words = np.zeros(max(n.value, 1), np.int32)
        probs = np.zeros(max(n.value, 1), np.float64)
        self._check(lib().ded_trigram_lookup(self._m, int(w0), int(w1), n.value, _p32(words),
                                             probs.ctypes.data_as(C.POINTER(C.c_double)), C.byref(n)), "ded_trigram_lookup")
        return [(int(w), float(p)) for w, p in zip(words[: n.value], probs[: n.value])]

    def size(self) -> int:
        return int(lib().ded_trigram_size(self._m))

    def mcts(self, w0: int, w1: int, uniform, iterations: int = 150, l: int = 4, n: int = 24, c1: float = 32.0,
             c2: float = 8.0):
        """Returns [(score, [words])], best first."""
        u = np.ascontiguousarray(uniform, dtype=np.float64)
        toks = np.zeros((max(n, 1), l), np.int32)
        lens = np.zeros(max(n, 1), np.int32)
        score = np.zeros(max(n, 1), np.float64)
        nc = C.c_int32(0)
        f64p = C.POINTER(C.c_double)
        self._check(lib().ded_draft_mcts(self._m, int(w0), int(w1), int(iterations), int(l), int(n), float(c1), float(c2),
                                         u.ctypes.data_as(f64p), len(u), _p32(toks), _p32(lens),
                                         score.ctypes.data_as(f64p), C.byref(nc)), "ded_draft_mcts")
        return [(float(score[i]), toks[i, : lens[i]].tolist()) for i in range(nc.value)]


def ded_verify_init(cfg: ded_config, weights: ded_weights, kv: ded_kv, workspace_ptr: int, workspace_bytes: int,
                    stream_ptr: int) -> int:
    out = C.c_void_p()
    rc = lib().ded_verify_init(C.byref(cfg), C.byref(weights) if weights is not None else None,
                               C.byref(kv) if kv is not None else None, workspace_ptr, workspace_bytes,
                               stream_ptr, C.byref(out))
    if rc != DED_OK:
        raise DedError(rc, "ded_verify_init")
    return out.value


def ded_verify_free(ctx: int) -> None:
    lib().ded_verify_free(ctx)


def ded_verify_step(ctx: int, prefix_len, n_nodes, parent, token, logits_ptr: Optional[int] = None) -> int:
    pl, nn, par, tok = _i32(prefix_len), _i32(n_nodes), _i32(parent), _i32(token)
    return int(lib().ded_verify_step(ctx, len(pl), _p32(pl), _p32(nn), _p32(par), _p32(tok), logits_ptr))


def ded_accept(ctx: int, mode: int, batch: int, max_nodes: int):
    stride = max_nodes + 1
    acc = np.zeros((batch, stride), np.int32)
    nacc = np.zeros(batch, np.int32)
    path = np.zeros((batch, stride), np.int32)
    newp = np.zeros(batch, np.int32)
    rc = int(lib().ded_accept(ctx, mode, _p32(acc), _p32(nacc), _p32(path), _p32(newp)))
    return rc, acc, nacc, path, newp


def ded_get_argmax(ctx: int, batch: int, max_nodes: int):
    a = np.full((batch, max_nodes), -1, np.int32)
    m = np.zeros((batch, max_nodes), np.float32)
    rc = int(lib().ded_get_argmax(ctx, _p32(a), m.ctypes.data_as(C.POINTER(C.c_float))))
    return rc, a, m


def ded_kv_store(ctx, layer, seq, first_slot, n, k_ptr, v_ptr) -> int:
    return int(lib().ded_kv_store(ctx, layer, seq, first_slot, n, k_ptr, v_ptr))


def ded_kv_load(ctx, layer, seq, first_slot, n, k_ptr, v_ptr) -> int:
    return int(lib().ded_kv_load(ctx, layer, seq, first_slot, n, k_ptr, v_ptr))


def ded_tree_attention(ctx, layer, prefix_len, n_nodes, parent, q_ptr, k_ptr, v_ptr, out_ptr) -> int:
    pl, nn, par = _i32(prefix_len), _i32(n_nodes), _i32(parent)
    return int(lib().ded_tree_attention(ctx, layer, len(pl), _p32(pl), _p32(nn), _p32(par), q_ptr, k_ptr, v_ptr,
                                        out_ptr))


def ded_tree_attention_static(ctx, layer, prefix_len, n_nodes, parent, q_ptr, k_ptr, v_ptr, out_ptr) -> int:
    pl, nn, par = _i32(prefix_len), _i32(n_nodes), _i32(parent)
    return int(lib().ded_tree_attention_static(ctx, layer, len(pl), _p32(pl), _p32(nn), _p32(par), q_ptr, k_ptr,
                                               v_ptr, out_ptr))


def ded_static_scratch_bytes() -> int:
    return int(lib().ded_static_scratch_bytes())


def ded_probe_stream_read(buffer_ptr: int, nbytes: int, sink_ptr: int, stream_ptr: int) -> int:
    return int(lib().ded_probe_stream_read(buffer_ptr, nbytes, sink_ptr, stream_ptr))


def ded_profile_enable(ctx, on: bool) -> int:
    return int(lib().ded_profile_enable(ctx, 1 if on else 0))


def ded_profile_read(ctx) -> dict:
    cap = 64
    names = (C.c_char_p * cap)()
    ms = (C.c_double * cap)()
    cnt = (C.c_int64 * cap)()
    n = int(lib().ded_profile_read(ctx, cap, names, ms, cnt))
    if n < 0:
        raise DedError(n, "ded_profile_read")
    return {names[i].decode(): (float(ms[i]), int(cnt[i])) for i in range(min(n, cap))}


# ---- device-buffer holder ---------------------------------------------------------------------


def _to_device(a, device, dtype: str):
    """numpy (fp32, or uint16 bf16 bit patterns) / torch tensor -> device tensor in storage dtype."""
    import torch
    if isinstance(a, np.ndarray):
        if a.dtype == np.uint16:
            t = torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
        else:
            t = torch.from_numpy(np.ascontiguousarray(a)).to(device)
    else:
        t = a.to(device)
    want = torch.bfloat16 if dtype == "bf16" else torch.float32
    if t.dtype != want:
        raise TypeError(f"tensor dtype {t.dtype} does not match the configured storage type {dtype}")
    return t.contiguous()


class Verifier:
    """Owns the device buffers of one context.  model_cfg: object with n_layers, d_model, n_heads,
    n_kv_heads, head_dim, d_ffn, vocab, rope_base, rms_eps, dtype ("fp32" | "bf16").
    weights: {"emb", "lm_head", "final_norm", "layers": [{wq, wk, wv, wo, wg, wu, wd, norm_attn,
    norm_ffn}]} (numpy or torch), each linear map [out][in]."""

    def __init__(self, model_cfg, weights, max_batch: int, kv_capacity: int, max_nodes: int, device="cuda:0"):
        import torch
        self.torch = torch
        self.device = torch.device(device)
        self.mc = model_cfg
        self.dtype = model_cfg.dtype
        self.max_batch, self.max_nodes = max_batch, max_nodes
        if self.dtype == "bf16":
            kv_capacity = (kv_capacity + 63) // 64 * 64
        self.kv_capacity = kv_capacity
        self.cfg = make_config(model_cfg.n_layers, model_cfg.d_model, model_cfg.n_heads, model_cfg.n_kv_heads,
                               model_cfg.head_dim, model_cfg.d_ffn, model_cfg.vocab, model_cfg.rope_base,
                               model_cfg.rms_eps, self.dtype, max_batch, kv_capacity, max_nodes)
        ws = ded_workspace_bytes(self.cfg)
        if ws == 0:
            raise DedError(DED_EINVAL, "ded_workspace_bytes")
        L = model_cfg.n_layers
        with torch.cuda.device(self.device):
            self.stream = torch.cuda.current_stream()
            self.workspace = torch.empty(ws, dtype=torch.uint8, device=self.device)
            kvb = ded_kv_layer_bytes(self.cfg)
            self.k_cache = [torch.empty(kvb, dtype=torch.uint8, device=self.device) for _ in range(L)]
            self.v_cache = [torch.empty(kvb, dtype=torch.uint8, device=self.device) for _ in range(L)]
            dev = lambda a, dt=self.dtype: _to_device(a, self.device, dt)
            keep = []  # plain weights, alive until init returns

            def cat(parts):
                ts = [dev(p) for p in parts]
                t = ts[0] if len(ts) == 1 else torch.cat(ts, dim=0)
                keep.append(t)
                return t.data_ptr()

            arr = lambda ptrs: (C.c_void_p * max(len(ptrs), 1))(*ptrs)
            lw = weights["layers"]
            W = ded_weights()
            W.emb, W.lm_head = cat([weights["emb"]]), cat([weights["lm_head"]])
            fn = dev(weights["final_norm"], "fp32"); keep.append(fn)
            W.final_norm = fn.data_ptr()
            a_qkv = arr([cat([l["wq"], l["wk"], l["wv"]]) for l in lw])
            a_o = arr([cat([l["wo"]]) for l in lw])
            a_gu = arr([cat([l["wg"], l["wu"]]) for l in lw])
            a_d = arr([cat([l["wd"]]) for l in lw])
            na = [dev(l["norm_attn"], "fp32") for l in lw]
            nf = [dev(l["norm_ffn"], "fp32") for l in lw]
            keep += na + nf
            a_na, a_nf = arr([t.data_ptr() for t in na]), arr([t.data_ptr() for t in nf])
            W.wqkv, W.wo, W.wgate_up, W.wdown, W.norm_attn, W.norm_ffn = a_qkv, a_o, a_gu, a_d, a_na, a_nf
            KV = ded_kv()
            a_k, a_v = arr([t.data_ptr() for t in self.k_cache]), arr([t.data_ptr() for t in self.v_cache])
            KV.k, KV.v = a_k, a_v
            torch.cuda.synchronize(self.device)
            self.ctx = ded_verify_init(self.cfg, W, KV, self.workspace.data_ptr(), ws, self.stream.cuda_stream)
            del keep
        self._batch = 0

    def close(self):
        if getattr(self, "ctx", None):
            ded_verify_free(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- helpers
    def _pad(self, rows: Sequence[Sequence[int]], fill: int) -> np.ndarray:
        out = np.full((len(rows), self.max_nodes), fill, np.int32)
        for b, r in enumerate(rows):
            out[b, : len(r)] = np.asarray(r, dtype=np.int32)
        return out

    def verify_step(self, prefix_len, parents, tokens, want_logits=False):
        """parents / tokens: one sequence of ints per batch entry.  Returns fp32 logits
        [batch][max_nodes][vocab] (device tensor) when want_logits."""
        B = len(parents)
        nn = [len(p) for p in parents]
        logits = None
        if want_logits:
            logits = self.torch.zeros((B, self.max_nodes, self.mc.vocab), dtype=self.torch.float32, device=self.device)
        rc = ded_verify_step(self.ctx, prefix_len, nn, self._pad(parents, -1), self._pad(tokens, 0),
                             logits.data_ptr() if want_logits else None)
        if rc != DED_OK:
            raise DedError(rc, "ded_verify_step")
        self._batch = B
        return logits

    def sample(self, temperature: float, top_p: float, uniform):
        """uniform: one sequence of floats in [0, 1) per batch entry (one per node)."""
        u = np.zeros((self._batch, self.max_nodes), np.float32)
        for b, r in enumerate(uniform):
            u[b, : len(r)] = np.asarray(r, dtype=np.float32)
        rc = int(lib().ded_sample(self.ctx, float(temperature), float(top_p),
                                  u.ctypes.data_as(C.POINTER(C.c_float))))
        if rc != DED_OK:
            raise DedError(rc, "ded_sample")

    def accept(self, mode=0):
        rc, acc, nacc, path, newp = ded_accept(self.ctx, mode, self._batch, self.max_nodes)
        if rc != DED_OK:
            raise DedError(rc, "ded_accept")
        return ([acc[b, : nacc[b]].tolist() for b in range(self._batch)],
                [path[b, : nacc[b]].tolist() for b in range(self._batch)], newp.tolist())

    def get_argmax(self):
        rc, a, m = ded_get_argmax(self.ctx, self._batch, self.max_nodes)
        if rc != DED_OK:
            raise DedError(rc, "ded_get_argmax")
        return a, m

    def kv_store(self, layer, seq, first_slot, k_plain=None, v_plain=None):
        """k_plain / v_plain: [Hkv][n][hd] numpy (fp32 or bf16 bits) or device tensors."""
        kt = None if k_plain is None else _to_device(k_plain, self.device, self.dtype)
        vt = None if v_plain is None else _to_device(v_plain, self.device, self.dtype)
        n = (kt if kt is not None else vt).shape[1]
        rc = ded_kv_store(self.ctx, layer, seq, first_slot, n, kt.data_ptr() if kt is not None else None,
                          vt.data_ptr() if vt is not None else None)
        if rc != DED_OK:
            raise DedError(rc, "ded_kv_store")
        self.torch.cuda.synchronize(self.device)

    def kv_load(self, layer, seq, first_slot, n):
        t = self.torch
        dt = t.bfloat16 if self.dtype == "bf16" else t.float32
        k = t.empty((self.mc.n_kv_heads, n, self.mc.head_dim), dtype=dt, device=self.device)
        v = t.empty_like(k)
        rc = ded_kv_load(self.ctx, layer, seq, first_slot, n, k.data_ptr(), v.data_ptr())
        if rc != DED_OK:
            raise DedError(rc, "ded_kv_load")
        t.cuda.synchronize(self.device)
        return k, v

    def tree_attention(self, layer, prefix_len, parents, q, k_tree, v_tree, out=None, static=False):
        """q [B][max_nodes][H][hd], k_tree / v_tree [B][Hkv][max_nodes][hd] device tensors in storage dtype.
        static=True goes through ded_tree_attention_static (the caller then passes `out`: nothing is allocated)."""
        if out is None:
            out = self.torch.zeros_like(q)
        nn = [len(p) for p in parents]
        fn = ded_tree_attention_static if static else ded_tree_attention
        rc = fn(self.ctx, layer, prefix_len, nn, self._pad(parents, -1), q.data_ptr(), k_tree.data_ptr(),
                v_tree.data_ptr(), out.data_ptr())
        if rc != DED_OK:
            raise DedError(rc, fn.__name__)
        return out

    def profile(self, on: bool):
        rc = ded_profile_enable(self.ctx, on)
        if rc != DED_OK:
            raise DedError(rc, "ded_profile_enable")

    def profile_read(self) -> dict:
        return ded_profile_read(self.ctx)
