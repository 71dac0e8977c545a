#!/usr/bin/env python3
"""Benchmark of the verification hot path on one MI355X.

A "step" = one whole verification pass: ded_verify_step (tree ingest, embedding, 32 decoder layers
with tree-masked attention, LM head, per-node argmax) + ded_accept (approval walk, KV compaction,
result download) on the Llama-2-7B shape with a 1024-token prefix and a 64-node draft tree
(synthetic random-init bf16 weights, Zipf prefix, tri-gram-seeded tree; everything resident in HBM).

Prints ONE JSON line.  `value` = verify steps/s = 1 / median step time, the median taken over at least 50
steps (and at least one second of them) after at least 10 warm-up steps, each step bracketed by HIP events on
the library's stream; the wall-clock median and mean per step are printed beside it.  Extra fields: verified
tokens/s (raw tri-gram trees and with planted acceptance), per-kernel-class times, the roofline of the dominant
kernel (the gate/up weight-streaming GEMM) and of all GEMMs, measured ceilings of the same run (a plain streaming
read, a large library GEMM) with every fraction also against them, tree attention on the attention-only
configuration (split-KV kernel plus merge kernel), the matrix-core-bound batched shapes, the batched
configurations c4 and c5 at their own depth, the paper's own tree shape (24 candidates of 4 tokens: up to 97
rows), and the CPU oracle timed on one whole step of the benchmark workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GEMM_CLASSES = ["gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down", "gemm_lm_head"]
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0  # f16 and bf16 dense MFMA peak
# HBM traffic per launch, KiB, as read by rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on `bench.py --profile-mode c3` and `--profile-mode c2`
# (summary and commands: profiles/c3_verify_step_hbm_traffic_pmc.md).  A plain 1 GiB device copy in the same
# run reads 0.5 GiB on FETCH_SIZE (wide coalesced loads are counted at half their size) and 1.0 GiB on
# WRITE_SIZE, hence the factors.
PMC_FETCH_FACTOR = 2.0
PMC_WRITE_FACTOR = 1.0
PMC_KIB = {  # class: (FETCH_SIZE, WRITE_SIZE) mean per launch
    "gemm_qkv": (63005.0, 14346.0),
    "gemm_o": (21083.0, 6282.0),
    "gemm_gate_up": (98621.0, 12395.0),
    "gemm_down": (52187.0, 6282.0),
    "gemm_lm_head": (136299.0, 16512.0),
    "tree_attention_c2": (33615.0 + 4249.0, 8320.0 + 2048.0),  # split-KV kernel + merge kernel
}


def pmc_bytes(cls):
    f, w = PMC_KIB[cls]
    return (f * PMC_FETCH_FACTOR + w * PMC_WRITE_FACTOR) * 1024.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def gemm_weight_elems(cfg):
    qkv = (cfg.n_heads + 2 * cfg.n_kv_heads) * cfg.head_dim * cfg.d_model
    per_layer = qkv + cfg.d_model * cfg.n_heads * cfg.head_dim + 3 * cfg.d_model * cfg.d_ffn
    return cfg.n_layers * per_layer + cfg.vocab * cfg.d_model


def planted_trees(di, ver, wl, prefix, parent, token, seed):
    """Draft trees whose first branch carries the model's own greedy continuation for m tokens
    (m ~ geometric, capped at the tree depth), so that acceptance lengths look like Table 1's
    2.2-2.8 tokens per forward.  The continuation comes from the library itself (single-node steps)."""
    import numpy as np
    P = len(prefix)
    cont, root, p = [], int(token[0]), P
    for _ in range(wl.depth):
        ver.verify_step([p], [[-1]], [[root]])
        acc, _, newp = ver.accept(mode=0)
        root, p = acc[0][0], newp[0]
        cont.append(root)
    depth = di.tree_depths(parent)
    # the greedy top-1 chain of the tri-gram tree: first child of each node, from the root down
    chain, v = [], 0
    for _ in range(wl.depth):
        kids = np.flatnonzero(parent == v)
        v = int(kids[0])
        chain.append(v)
    g = np.random.default_rng(seed)
    trees = []
    for _ in range(16):
        m = min(int(g.geometric(0.42)) - 1, wl.depth)  # mean ~1.4 accepted draft tokens + 1 bonus
        t = token.copy()
        for j in range(m):
            t[chain[j]] = cont[j]
        if m < wl.depth and t[chain[m]] == cont[m]:
            t[chain[m]] = (cont[m] + 1) % wl.model.vocab
        trees.append(t)
    return trees


def time_steps(step, min_steps, warmup, min_seconds=1.0, max_steps=2000):
    """step(i) runs one whole verification step (ded_verify_step + ded_accept, which synchronises) and returns the
    number of tokens it committed.  Every timed step sits between two HIP events recorded on the library's stream
    (torch's current stream) and between two host clock readings.  At least `min_steps` steps and `min_seconds`
    of them are timed after `warmup` untimed ones."""
    import statistics
    import torch
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ev_ms, wall_ms, n_tok, i = [], [], 0, 0
    while i < max_steps and (i < min_steps or sum(wall_ms) < 1e3 * min_seconds):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        n_tok += step(warmup + i)
        e1.record()
        e1.synchronize()
        wall_ms.append((time.perf_counter() - t0) * 1e3)
        ev_ms.append(e0.elapsed_time(e1))
        i += 1
    return {"steps": i, "tokens": n_tok, "event_ms_median": statistics.median(ev_ms),
            "wall_ms_median": statistics.median(wall_ms), "wall_ms_mean": sum(wall_ms) / i,
            "event_ms_p10": sorted(ev_ms)[i // 10], "event_ms_p90": sorted(ev_ms)[(9 * i) // 10]}


def measured_ceilings():
    """What this chip sustains in this run, by the simplest possible kernels: (1) a plain streaming read of 2 GiB
    (the library's probe kernel, 16 bytes per lane), (2) a large square bf16 GEMM from the vendor library
    (8192^3 through torch.matmul).  The streaming kernels are reported against (1), the matrix-core-bound ones
    against (2), beside the published peaks."""
    import statistics
    import torch
    from paper_2407_12021_amd import binding as B
    n = 2 << 30
    buf = torch.empty(n, dtype=torch.uint8, device="cuda")
    buf.random_(0, 255)
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    times = []
    for i in range(12):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        rc = B.ded_probe_stream_read(buf.data_ptr(), n, sink.data_ptr(), st)
        e1.record()
        e1.synchronize()
        assert rc == 0
        if i >= 2:
            times.append(e0.elapsed_time(e1))
    read_gbs = n / (statistics.median(times) * 1e-3) / 1e9
    del buf
    m = 8192
    a = torch.randn(m, m, device="cuda", dtype=torch.bfloat16)
    b = torch.randn(m, m, device="cuda", dtype=torch.bfloat16)
    times = []
    for i in range(12):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        c = a @ b
        e1.record()
        e1.synchronize()
        if i >= 2:
            times.append(e0.elapsed_time(e1))
    gemm_tflops = 2.0 * m ** 3 / (statistics.median(times) * 1e-3) / 1e12
    del a, b, c
    torch.cuda.empty_cache()
    return {"stream_read_gbs": read_gbs, "stream_read": "2 GiB, 16 B per lane, non-temporal loads, library probe kernel, median of 10",
            "library_gemm_tflops": gemm_tflops, "library_gemm": "bf16 8192 x 8192 x 8192 via torch.matmul, median of 10",
            "hbm_peak_gbs": HBM_PEAK_GBS, "mfma_peak_tflops": MFMA_BF16_PEAK_TFLOPS}


def decode_loop_bench(di, ver, wl, prefix, root, n_new=48, seed=2):
    """End-to-end decoding from the resident 1024-token prefix with the whole loop of the method: every step the
    C++ draft maker searches the tri-gram matrix (150 iterations, n = 24 candidates of l = 4 words, C1 = 32, C2 = 8,
    elimination threshold 12), ded_build_tree merges the candidates (budget = the context's 64 nodes), the tree is
    verified, the accepted tokens are committed and fed back through Adjust3Gram.
    A random-init model agrees with no corpus, so the synthetic corpus is made to resemble the model's output the
    way the paper's corpora resemble an LLM's: for every context of the model's own greedy continuation (from a
    plain one-token-per-step pass through the same library) it holds the true next token among that context's
    synthetic successors, with a share of the context's 200 occurrences drawn from {0.05, 0.2, 0.5} (0.05 falls
    under the threshold), and three levels of synthetic continuations of the wrong successors.  What is accepted
    is whatever the search finds.
    The output must equal the plain greedy continuation token for token."""
    import numpy as np
    from paper_2407_12021_amd import binding as B
    P = len(prefix)
    import torch
    ref, r, p = [], int(root), P
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while len(ref) < n_new + wl.depth + 8:  # plain greedy decoding, one token per step
        ver.verify_step([p], [[-1]], [[r]])
        acc, _, newp = ver.accept(mode=0)
        r, p = acc[0][0], newp[0]
        ref.append(r)
    plain_tokens_per_s = len(ref) / (time.perf_counter() - t0)
    tri = di.SyntheticTrigram(wl.model.vocab, seed=0)
    g = np.random.default_rng(seed)
    drafter = B.Drafter()

    def add_context(a, c, true, levels):
        """Counts for the context (a, c): its synthetic successors share 200 occurrences (minus the true token's
        share); successors frequent enough to survive the threshold get continuations of their own."""
        succ, prob = tri.successors(a, c)
        share = float(g.choice([0.05, 0.2, 0.5])) if true is not None else 0.0
        for x, px in zip(succ.tolist(), prob.tolist()):
            if x == true:
                continue
            k = int(round(200 * px * (1.0 - share)))
            drafter.count([a, c, x], k)
            if levels > 0 and k >= 12:
                add_context(c, x, None, levels - 1)
        if true is not None:
            drafter.count([a, c, true], int(round(200 * share)))

    seq = [int(prefix[-1]), int(root)] + ref
    for i in range(2, len(seq)):
        add_context(seq[i - 2], seq[i - 1], seq[i], 3)
    drafter.finalize(12)
    out, steps, nodes, n_cands = [], 0, 0, 0
    prev, r, p = int(prefix[-1]), int(root), P
    t_draft = t_tree = 0.0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while len(out) < n_new:
        tb = time.perf_counter()
        cands = [w for _, w in drafter.mcts(prev, r, g.random(600), iterations=150, l=4, n=24, c1=32.0, c2=8.0)]
        tc = time.perf_counter()
        rc, parent, token, _ = B.ded_build_tree(r, cands, wl.n_nodes)
        assert rc == B.DED_OK
        t_draft += tc - tb
        t_tree += time.perf_counter() - tc
        ver.verify_step([p], [parent], [token])
        acc, _, newp = ver.accept(mode=0)
        out += acc[0]
        tb = time.perf_counter()
        drafter.adjust(([prev, r] + acc[0])[-34:], 34, 0.1, 1.0)  # Adjust3Gram on what was just committed
        t_draft += time.perf_counter() - tb
        prev = acc[0][-2] if len(acc[0]) > 1 else r
        r, p = acc[0][-1], newp[0]
        steps += 1
        nodes += len(parent)
        n_cands += len(cands)
    dt = time.perf_counter() - t0
    lossless = out[:n_new] == ref[:n_new]
    trigrams = drafter.size()
    drafter.close()
    return {"tokens": len(out), "steps": steps, "tokens_per_s": len(out) / dt, "steps_per_s": steps / dt,
            "plain_greedy_tokens_per_s": plain_tokens_per_s, "speedup_vs_plain_greedy": len(out) / dt / plain_tokens_per_s,
            "mean_accepted_per_step": len(out) / steps, "mean_tree_nodes": nodes / steps,
            "mean_candidates": n_cands / steps, "trigrams_in_matrix": trigrams,
            "draft_maker_us_per_step": 1e6 * t_draft / steps, "tree_build_us_per_step": 1e6 * t_tree / steps,
            "host_draft_and_tree_build_share": (t_draft + t_tree) / dt, "lossless_vs_plain_greedy": bool(lossless)}


def attention_only_bench(di, iters=40):
    """Tree attention alone on the attention-only configuration; 8 layers act as rotating K/V buffer
    sets (8 x 68 MB > the 256 MB last-level cache) so that every launch streams from HBM."""
    import numpy as np
    import torch
    from paper_2407_12021_amd import Verifier
    from paper_2407_12021_amd.binding import _to_device
    wl = di.WORKLOADS["c2"]
    sets = 8
    cfg = di.ModelConfig("attn-only", sets, 128, 32, 32, 128, 128, 16)
    w = di.make_weights(cfg, seed=0)
    ver = Verifier(cfg, w, max_batch=1, kv_capacity=wl.prefix_len + wl.n_nodes, max_nodes=wl.n_nodes)
    parent = di.random_tree(wl.n_nodes, wl.depth, seed=0)
    qs, kts, vts = [], [], []
    for l in range(sets):
        x = di.attention_inputs(32, 32, 128, wl.prefix_len, wl.n_nodes, seed=100 + l)
        ver.kv_store(l, 0, 0, x["k_prefix"], x["v_prefix"])
        qs.append(_to_device(x["q"], ver.device, "bf16")[None])
        kts.append(_to_device(x["k_tree"], ver.device, "bf16")[None])
        vts.append(_to_device(x["v_tree"], ver.device, "bf16")[None])
    for l in range(sets):
        ver.tree_attention(l, [wl.prefix_len], [parent], qs[l], kts[l], vts[l])
    torch.cuda.synchronize()
    ver.profile(True)
    for i in range(iters):
        l = i % sets
        ver.tree_attention(l, [wl.prefix_len], [parent], qs[l], kts[l], vts[l])
    prof = ver.profile_read()
    ver.profile(False)
    ver.close()
    ms, n = prof["tree_attention"]  # one bracket around the whole operation: split-KV kernel + merge kernel
    keys = wl.prefix_len + wl.n_nodes
    kv_bytes = 2 * keys * 32 * 128 * 2            # K and V, 2 bytes each, every key of every kv head once
    q_o_bytes = 2 * wl.n_nodes * 32 * 128 * 2      # q in, o out
    alg = kv_bytes + q_o_bytes
    us = ms / n * 1e3
    whole = alg / (us * 1e-6) / 1e9
    return {"bound": "hbm", "kernel": "tree_attn_tiled_kernel + tree_attn_merge_kernel (the whole attention operation)",
            "workload": "c2 attention-only: 32 heads x 128, 4096-key prefix, 64-node tree of depth 8, 8 rotating K/V sets",
            "achieved": whole, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": whole / HBM_PEAK_GBS,
            "traffic": pmc_bytes("tree_attention_c2"),
            "time_base": "one HIP-event bracket around the two launches of the operation (ded_profile_*); per-kernel "
                         "durations: profiles/c2_tree_attention_kernel_stats_and_pmc.md",
            "us_per_launch": us, "algorithmic_bytes": alg}


def large_rows_bench(di, steps=8):
    """The projection GEMMs where they are matrix-core bound: batched trees give hundreds of rows per weight.
    7B-shape layers (2 of them), batch 8 x 256-node trees = 2048 rows, and the 13B shape with batch 4 x 128 =
    512 rows; empty prefixes (the attention share does not matter here).  Times are HIP-event brackets per
    kernel class.  'executed' counts the hi and lo activation planes (two matrix instructions per useful one in
    the QKV / gate-up GEMMs; the LM head reads the hi plane alone from 256 rows on, like the O and down
    projections), 'useful' counts 2 * rows * N * K once."""
    import numpy as np
    from paper_2407_12021_amd import Verifier
    out = []
    for label, base, batch, nodes in (("7B shape, 8 x 256-node trees", di.WORKLOADS["c3"].model, 8, 256),
                                      ("13B shape, 4 x 128-node trees", di.WORKLOADS["c4"].model, 4, 128)):
        cfg = base.with_layers(2)
        w = di.make_weights(cfg, seed=0, threads=16)
        ver = Verifier(cfg, w, max_batch=batch, kv_capacity=nodes + 64, max_nodes=nodes)
        del w
        parent = di.random_tree(nodes, None, seed=3)
        g = np.random.default_rng(5)
        toks = [g.integers(0, cfg.vocab, size=nodes) for _ in range(batch)]
        run = lambda: (ver.verify_step([0] * batch, [parent] * batch, toks), ver.accept(mode=0))
        for _ in range(2):
            run()
        ver.profile(True)
        for _ in range(steps):
            run()
        prof = ver.profile_read()
        ver.profile(False)
        ver.close()
        R = batch * nodes
        d, F, V, qkv_n = cfg.d_model, cfg.d_ffn, cfg.vocab, (cfg.n_heads + 2 * cfg.n_kv_heads) * cfg.head_dim
        shapes = {"gemm_qkv": (qkv_n, d, 2), "gemm_o": (d, cfg.n_heads * cfg.head_dim, 1), "gemm_gate_up": (2 * F, d, 2),
                  "gemm_down": (d, F, 1), "gemm_lm_head": (V, d, 1 if R >= 256 else 2)}
        per = {}
        useful = executed = ms_total = 0.0
        for c, (N, K, planes) in shapes.items():
            ms, n = prof[c]
            fl = 2.0 * R * N * K * n
            per[c] = {"us_per_launch": round(ms / n * 1e3, 1), "executed_tflops": round(planes * fl / (ms * 1e-3) / 1e12, 1)}
            useful += fl
            executed += planes * fl
            ms_total += ms
        out.append({"workload": label, "rows": R, "executed_tflops": executed / (ms_total * 1e-3) / 1e12,
                    "useful_tflops": useful / (ms_total * 1e-3) / 1e12, "by_class": per})
    best = max(out, key=lambda o: o["executed_tflops"])
    return {"bound": "mfma", "kernel": "gemm_large_kernel (256 features x 128 or 256 rows per workgroup), all projections of a step",
            "achieved": best["executed_tflops"], "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": best["executed_tflops"] / MFMA_BF16_PEAK_TFLOPS, "traffic": None, "cases": out}


def profile_workload(di, mode):
    """The launches that a rocprofv3 run of `--profile-mode` other than c3 should see (see the option's help)."""
    import numpy as np
    import torch
    from paper_2407_12021_amd import Verifier
    if mode == "c2":
        attention_only_bench(di, iters=16)
        return
    if mode == "large":
        cfg, batch, nodes, P = di.WORKLOADS["c3"].model.with_layers(2), 8, 256, 0
    else:
        cfg, batch, nodes, P = di.WORKLOADS["c5"].model.with_layers(2), 8, 256, 16384
    w = di.make_weights(cfg, seed=0, threads=16)
    ver = Verifier(cfg, w, max_batch=batch, kv_capacity=P + nodes + 64, max_nodes=nodes)
    del w
    g = np.random.default_rng(5)
    for s0 in range(0, P, nodes):
        ver.verify_step([s0] * batch, [di.chain_tree(nodes)] * batch, [g.integers(0, cfg.vocab, size=nodes) for _ in range(batch)])
        ver.accept(mode=1)
    parent = di.random_tree(nodes, None, seed=3)
    toks = [g.integers(0, cfg.vocab, size=nodes) for _ in range(batch)]
    for _ in range(4 if mode == "large" else 3):
        ver.verify_step([P] * batch, [parent] * batch, toks)
        ver.accept(mode=0)
    torch.cuda.synchronize()
    ver.close()


STEP_LOWER_BOUND_MS = {"c3": 1.72, "c4": 6.2, "c5": 19.4}  # weight / cache bytes at 8 TB/s or matrix flops at 2.5 PFLOP/s


def batched_config_bench(di, name, min_steps):
    """One of the batched configurations at its own depth and size (c4: 13B shape, 40 layers, batch 4, prefix 2048,
    128-node trees; c5: Llama-3-8B shape, 32 layers, batch 8, prefix 16384, 256-node trees): random-init weights,
    prefix computed by chunked prefill, then the tree step timed like the headline (event median)."""
    import torch
    from paper_2407_12021_amd import Verifier
    wl = di.WORKLOADS[name]
    cfg = wl.model
    t0 = time.perf_counter()
    w = di.make_weights(cfg, seed=0, threads=16)
    B, N = wl.batch, wl.n_nodes
    ver = Verifier(cfg, w, max_batch=B, kv_capacity=wl.prefix_len + N + wl.depth + 2, max_nodes=N)
    del w
    seqs = [di.workload_tree(wl, seed=0, seq=b) for b in range(B)]
    P = wl.prefix_len
    for s0 in range(0, P, N):
        n = min(N, P - s0)
        ver.verify_step([s0] * B, [di.chain_tree(n)] * B, [q[0][s0:s0 + n] for q in seqs])
        ver.accept(mode=1)
    torch.cuda.synchronize()
    log(f"{name}: weights, init and prefill {time.perf_counter() - t0:.1f} s")
    parents, tokens = [q[1] for q in seqs], [q[2] for q in seqs]

    def step(i):
        ver.verify_step([P] * B, parents, tokens)
        acc, _, _ = ver.accept(mode=0)
        return sum(len(a) for a in acc)

    r = time_steps(step, min_steps, 3, min_seconds=0.5)
    ver.profile(True)
    for i in range(3):
        step(i)
    prof = ver.profile_read()
    ver.profile(False)
    ver.close()
    ms = r["event_ms_median"]
    rows = B * N
    flops = 2.0 * rows * gemm_weight_elems(cfg)
    return {"workload": f"{name}: {cfg.name}, {cfg.n_layers} layers, batch {B}, prefix {P}, {N}-node trees",
            "steps_per_s": 1e3 / ms, "ms_per_step": ms, "wall_ms_per_step_median": r["wall_ms_median"],
            "timed_steps": r["steps"], "verified_tokens_per_s_raw_trees": r["tokens"] / r["steps"] * 1e3 / ms,
            "step_lower_bound_ms": STEP_LOWER_BOUND_MS[name], "frac_of_lower_bound": STEP_LOWER_BOUND_MS[name] / ms,
            "projection_useful_tflops": flops / (sum(prof[c][0] for c in GEMM_CLASSES) / 3 * 1e-3) / 1e12,
            "kernel_ms_per_step": {k: round(v[0] / 3, 3) for k, v in prof.items() if v[1]}}


def cpu_baseline(di, wl, parent, token):
    """The fp64 oracle as it stands, timed on one whole verification step of the benchmark workload (all 32 layers,
    64-row tree against a 1024-key prefix; random K/V stand in for the prefix: the oracle's time does not depend
    on values, and computing the prefix itself is not part of a step)."""
    import numpy as np
    import oracle
    cfg = wl.model
    w = di.make_weights(cfg, seed=0, threads=16)
    kv = [di.attention_inputs(cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, wl.prefix_len, 1, seed=7 + l)
          for l in range(cfg.n_layers)]
    pk = [x["k_prefix"].transpose(1, 0, 2) for x in kv]
    pv = [x["v_prefix"].transpose(1, 0, 2) for x in kv]
    t0 = time.perf_counter()
    oracle.verify_tree(cfg, w, parent, token, pk, pv)
    t_step = time.perf_counter() - t0
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count()
    try:
        from threadpoolctl import threadpool_info
        blas = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        blas = cores
    return {"value": 1.0 / t_step, "unit": "verify steps/s", "cores": int(min(cores, blas)), "kind": "oracle",
            "sample": f"fp64 numpy oracle, one whole step (64-row tree, 1024-key prefix, {cfg.n_layers} layers): {t_step:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--layers", type=int, default=0, help="debug: fewer layers (result is then not the headline metric)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-attn", action="store_true")
    ap.add_argument("--no-large-rows", action="store_true")
    ap.add_argument("--no-batched", action="store_true", help="skip the c4 / c5 step timings (26 GB and 15 GB of weights)")
    ap.add_argument("--profile-mode", choices=["c3", "c2", "large", "c5attn"],
                    help="a minimal workload for rocprofv3 runs (kernel trace or one --pmc counter set), no timing: "
                         "c3 = a 1 GiB device copy (counter calibration) + 4 verification steps of the benchmark workload; "
                         "c2 = 24 attention-only launches of configuration 2; large = 4 steps of a 2-layer 7B-shape model "
                         "on 8 x 256-node trees (2048 rows); c5attn = 3 steps of a 2-layer Llama-3-8B-shape model, batch 8, "
                         "prefix 16384, 256-node trees")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import ded_inputs as di
    from paper_2407_12021_amd import Verifier

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if args.profile_mode and args.profile_mode != "c3":
        profile_workload(di, args.profile_mode)
        print(json.dumps({"profile_mode": args.profile_mode}))
        return
    wl = di.WORKLOADS["c3"]
    cfg = wl.model if not args.layers else wl.model.with_layers(args.layers)
    t0 = time.perf_counter()
    w = di.make_weights(cfg, seed=0, threads=16)
    log(f"weights: {time.perf_counter() - t0:.1f} s")
    prefix, parent, token = di.workload_tree(wl, seed=0)
    t0 = time.perf_counter()
    # max_nodes 128: the same context also runs the 97-row tree of the paper's shape; a step's kernels are shaped
    # by the step's own node count (64 here), not by the maximum
    ver = Verifier(cfg, w, max_batch=1, kv_capacity=wl.prefix_len + 128 + wl.depth + 2, max_nodes=128)
    del w
    log(f"upload + init: {time.perf_counter() - t0:.1f} s")
    P = len(prefix)
    for s in range(0, P, wl.n_nodes):  # chunked prefill through chain trees
        n = min(wl.n_nodes, P - s)
        ver.verify_step([s], [di.chain_tree(n)], [prefix[s:s + n]])
        ver.accept(mode=1)
    if args.profile_mode == "c3":
        a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        b.copy_(a)  # counter calibration: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        for _ in range(4):
            ver.verify_step([P], [parent], [token])
            ver.accept(mode=0)
        ver.close()
        print(json.dumps({"profile_mode": "c3"}))
        return
    planted = planted_trees(di, ver, wl, prefix, parent, token, seed=1)

    def step_planted(i):
        ver.verify_step([P], [parent], [planted[i % len(planted)]])
        acc, _, _ = ver.accept(mode=0)
        return len(acc[0])

    def step_raw(i):
        ver.verify_step([P], [parent], [token])
        acc, _, _ = ver.accept(mode=0)
        return len(acc[0])

    # headline: planted acceptance (kernel time does not depend on the acceptance length)
    head = time_steps(step_planted, max(args.steps, 50), max(args.warmup, 10))
    raw = time_steps(step_raw, 20, 2, min_seconds=0.2)
    ms_step = head["event_ms_median"]

    # the paper's own tree shape (Appendix F.1: n = 24 candidates of l = 4 tokens): the pseudo-sequence has up to
    # 1 + 24 * 4 = 97 rows when no two candidates share a prefix; that worst case is timed here
    g = np.random.default_rng(4)
    cands = [[int(x) for x in g.choice(cfg.vocab, size=4, replace=False)] for _ in range(24)]
    firsts = g.choice(cfg.vocab, size=24, replace=False)
    for c, f in zip(cands, firsts):
        c[0] = int(f)
    from paper_2407_12021_amd import binding as B
    rc, parent97, token97, _ = B.ded_build_tree(int(token[0]), cands, 128)
    assert rc == 0 and len(parent97) == 97

    def step_paper(i):
        ver.verify_step([P], [parent97], [token97])
        acc, _, _ = ver.accept(mode=0)
        return len(acc[0])

    paper = time_steps(step_paper, 50, 5, min_seconds=0.3)
    paper_shape = {"candidates": 24, "tokens_per_candidate": 4, "nodes": 97, "ms_per_step": paper["event_ms_median"],
                   "steps_per_s": 1e3 / paper["event_ms_median"],
                   "ratio_to_64_node_step": paper["event_ms_median"] / ms_step,
                   "verified_tokens_per_s_at_paper_accept_2.4": 2.4 * 1e3 / paper["event_ms_median"]}

    decode = decode_loop_bench(di, ver, wl, prefix, int(token[0]))

    # stochastic approval (temperature 0.8, top-p 0.9): the extra cost of sampling the model's token at 64 nodes
    g = np.random.default_rng(3)

    def step_sampled(i):
        ver.verify_step([P], [parent], [planted[i % len(planted)]])
        ver.sample(0.8, 0.9, [g.random(len(parent)).astype(np.float32)])
        acc, _, _ = ver.accept(mode=0)
        return len(acc[0])

    # per-kernel-class times of the plain step first (separate pass: event brackets add ~2 us per launch); the
    # sampled steps come last because a context that has sampled keeps materialising its logits
    ver.profile(True)
    prof_steps = 5
    for i in range(prof_steps):
        step_planted(i)
    prof = ver.profile_read()
    ver.profile(False)
    st = time_steps(step_sampled, 20, 3, min_seconds=0.2)
    ver.profile(True)
    for i in range(3):
        step_sampled(i)
    prof_st = ver.profile_read()
    ver.profile(False)
    stochastic = {"temperature": 0.8, "top_p": 0.9, "steps_per_s": 1e3 / st["event_ms_median"],
                  "ms_per_step": st["event_ms_median"],
                  "sample_kernel_us": prof_st["sample_top_p"][0] / max(prof_st["sample_top_p"][1], 1) * 1e3}
    ver.close()
    del ver
    torch.cuda.empty_cache()
    ceil = measured_ceilings()

    gemm_ms = sum(prof[c][0] for c in GEMM_CLASSES) / prof_steps
    gemm_launches = sum(prof[c][1] for c in GEMM_CLASSES) // prof_steps
    w_bytes = 2.0 * gemm_weight_elems(cfg)
    gemm_gbs = w_bytes / (gemm_ms * 1e-3) / 1e9
    gemm_tflops = 2.0 * wl.n_nodes * gemm_weight_elems(cfg) / (gemm_ms * 1e-3) / 1e12
    kernels_ms = {k: round(v[0] / prof_steps, 4) for k, v in prof.items() if v[1]}
    # dominant kernel: the gate/up projection (largest share of the step); one launch streams 2F x d bf16 weights
    gu_us = prof["gemm_gate_up"][0] / max(prof["gemm_gate_up"][1], 1) * 1e3 if cfg.n_layers else float("nan")
    gu_bytes = 2.0 * 2 * cfg.d_ffn * cfg.d_model
    gu_gbs = gu_bytes / (gu_us * 1e-6) / 1e9
    full_model = cfg.n_layers == wl.model.n_layers
    per_launch = {c: prof[c][0] / max(prof[c][1], 1) * 1e3 for c in GEMM_CLASSES}
    gemm_traffic_step = (sum(pmc_bytes(c) for c in GEMM_CLASSES[:4]) * cfg.n_layers + pmc_bytes("gemm_lm_head")
                         if full_model else None)
    step_bytes = w_bytes + 2.0 * 2 * (P + wl.n_nodes) * cfg.n_kv_heads * cfg.head_dim * cfg.n_layers
    time_base = ("HIP-event brackets around each launch on the library's stream in a separate 5-step pass "
                 "(ded_profile_*; ~2 us of bracket per launch included); kernel-only durations: "
                 "profiles/c3_verify_step_kernel_stats.md")

    out = {
        "metric": "tree-verify steps/s at 7B shape (64-node tree, 1024-token prefix, batch 1)",
        "value": 1e3 / ms_step,
        "unit": "verify steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_step,
        "timing": {"what": "median over timed_steps steps, each between two HIP events on the library's stream, after "
                           "warmup_steps untimed steps", "timed_steps": head["steps"], "warmup_steps": max(args.warmup, 10),
                   "event_ms_p10": head["event_ms_p10"], "event_ms_p90": head["event_ms_p90"],
                   "wall_ms_per_step_median": head["wall_ms_median"], "wall_ms_per_step_mean": head["wall_ms_mean"]},
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 matrix-core operands (bf16 weights widened exactly, hi/lo activation pairs), fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": "c3: Llama-2-7B shape, bf16 random init N(0,0.02), prefix 1024 (Zipf 1.1), "
                               "64-node tri-gram-seeded tree of depth 6, batch 1"
                               + (f" [DEBUG: {args.layers} layers]" if args.layers else ""),
                   "n_layers": cfg.n_layers, "prefix_len": P, "n_nodes": wl.n_nodes, "batch": 1},
        "verified_tokens_per_s": head["tokens"] / head["steps"] * 1e3 / ms_step,
        "mean_accepted_per_step": head["tokens"] / head["steps"],
        "acceptance": "planted: one branch carries the model's own continuation for m~Geom tokens",
        "step_hbm": {"algorithmic_bytes_per_step": step_bytes, "achieved_gbs": step_bytes / (ms_step * 1e-3) / 1e9,
                     "frac_of_peak": step_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "frac_of_measured_stream_read": step_bytes / (ms_step * 1e-3) / 1e9 / ceil["stream_read_gbs"],
                     "step_lower_bound_ms": STEP_LOWER_BOUND_MS["c3"]},
        "raw_trigram_tree": {"steps_per_s": 1e3 / raw["event_ms_median"],
                             "verified_tokens_per_s": raw["tokens"] / raw["steps"] * 1e3 / raw["event_ms_median"],
                             "mean_accepted_per_step": raw["tokens"] / raw["steps"]},
        "paper_shape": paper_shape,
        "decode_loop": decode,
        "stochastic_approval": stochastic,
        "kernel_ms_per_step": kernels_ms,
        "ceilings": ceil,
        "roofline": {"bound": "hbm",
                     "kernel": "gate/up projection GEMM with SiLU*up epilogue (gemm_wide_kernel, 3 feature groups per "
                               "workgroup, 2 activation planes, split-K 2): 22016 x 4096 bf16 weights per launch",
                     "achieved": gu_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gu_gbs / HBM_PEAK_GBS,
                     "frac_of_measured_stream_read": gu_gbs / ceil["stream_read_gbs"],
                     "traffic": pmc_bytes("gemm_gate_up") if full_model else None,
                     "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of `bench.py --profile-mode c3` "
                                       "(profiles/c3_verify_step_hbm_traffic_pmc.md), not re-measured in this run",
                     "time_base": time_base,
                     "avg_launch_us": gu_us, "algorithmic_bytes_per_launch": gu_bytes,
                     "launches_per_step": cfg.n_layers, "share_of_step": gu_us * 1e-3 * cfg.n_layers / ms_step},
        "roofline_all_gemms": {"bound": "hbm", "kernel": "all projection GEMMs of a step (QKV, O, gate/up, down, LM head)",
                               "achieved": gemm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gemm_gbs / HBM_PEAK_GBS,
                               "frac_of_measured_stream_read": gemm_gbs / ceil["stream_read_gbs"],
                               "traffic_per_step": gemm_traffic_step, "launches_per_step": int(gemm_launches),
                               "avg_launch_us": gemm_ms * 1e3 / max(gemm_launches, 1),
                               "us_per_launch_by_class": {k: round(v, 2) for k, v in per_launch.items()},
                               "algorithmic_bytes_per_step": w_bytes, "mfma_tflops": gemm_tflops,
                               "mfma_frac": gemm_tflops / MFMA_BF16_PEAK_TFLOPS, "time_base": time_base},
    }
    if not args.no_attn:
        att = attention_only_bench(di)
        att["frac_of_measured_stream_read"] = att["achieved"] / ceil["stream_read_gbs"]
        out["roofline_tree_attention"] = att
    if not args.no_large_rows:
        lr = large_rows_bench(di)
        lr["frac_of_library_gemm"] = lr["achieved"] / ceil["library_gemm_tflops"]
        out["roofline_large_rows"] = lr
    if not args.no_batched:
        out["batched_configs"] = {"c4": batched_config_bench(di, "c4", 20), "c5": batched_config_bench(di, "c5", 10)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(di, wl, parent, token)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
