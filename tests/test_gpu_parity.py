"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest

import ded_inputs as di
import oracle

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-4, "bf16": 2e-2}  # max-abs logit error allowed per storage type
MARGIN = 0.05                       # token decisions are compared only above this top-1 margin


def _verifier(*a, **k):
    import torch
    assert torch.cuda.is_available()
    from paper_2407_12021_amd import Verifier
    return Verifier(*a, **k)


def gpu_prefill(ver, tokens, seq_count=1, chunk=None):
    """Chunked prefill through chain trees + force-accept; tokens: list of per-sequence arrays (equal length)."""
    chunk = chunk or ver.max_nodes
    P = len(tokens[0])
    done = 0
    while done < P:
        n = min(chunk, P - done)
        ver.verify_step([done] * seq_count, [di.chain_tree(n)] * seq_count, [t[done:done + n] for t in tokens])
        _, _, newp = ver.accept(mode=1)
        done += n
        assert newp == [done] * seq_count
    return P


def check_step(cfg, w, ver, prefix, parent, token, pk, pv, seq=0, batch_inputs=None):
    """One tree step on the GPU vs the oracle: logits, argmax, walk, compaction, cache contents."""
    P = len(prefix)
    N = len(parent)
    ref, kr, vr = oracle.verify_tree(cfg, w, parent, token, pk, pv)
    logits = ver.verify_step([P], [parent], [token], want_logits=True)[0, :N].cpu().numpy().astype(np.float64)
    err = np.abs(logits - ref).max()
    assert err <= TOL[cfg.dtype], f"max |logit error| {err:.3e}"
    a_ref, margin = oracle.argmax_margin(ref)
    a_gpu, m_gpu = ver.get_argmax()
    sure = margin > MARGIN
    assert (a_gpu[0, :N][sure] == a_ref[sure]).all()
    assert np.abs(m_gpu[0, :N] - margin).max() <= 2 * TOL[cfg.dtype]
    # the device-side argmax must agree with the device-side logits exactly (lowest id on ties)
    assert (a_gpu[0, :N] == np.argmax(logits, axis=1)).all()
    acc, path, newp = ver.accept(mode=0)
    # walk parity: feed the GPU's own tokens to the oracle walk (integer work -> bit exact) ...
    acc2, path2 = oracle.accept_walk(parent, token, a_gpu[0, :N])
    assert acc[0] == acc2 and path[0] == path2 and newp[0] == P + len(path2)
    # ... and the oracle's tokens wherever every decision on the walk is above the margin
    acc_ref, path_ref = oracle.accept_walk(parent, token, a_ref)
    if all(sure[v] for v in set(path_ref) | set(path[0])):
        assert acc[0] == acc_ref and path[0] == path_ref
    # cache after compaction == prefix K/V followed by the path rows
    L = cfg.n_layers
    for l in sorted({0, L - 1}) if L else []:
        k_gpu, v_gpu = ver.kv_load(l, seq, 0, newp[0])
        k_ref = oracle.compact_rows(oracle.widen(pk[l]) if P else kr[l][:0], kr[l], path[0])
        v_ref = oracle.compact_rows(oracle.widen(pv[l]) if P else vr[l][:0], vr[l], path[0])
        kerr = np.abs(k_gpu.float().cpu().numpy().transpose(1, 0, 2) - k_ref).max()
        verr = np.abs(v_gpu.float().cpu().numpy().transpose(1, 0, 2) - v_ref).max()
        scale = max(1.0, np.abs(k_ref).max(), np.abs(v_ref).max())
        lim = (1e-4 if cfg.dtype == "fp32" else 2e-2) * scale
        assert kerr <= lim and verr <= lim, (l, kerr, verr)
    return float(err), int((~sure).sum())


# ------------------------------------------------------------------------------------------ fp32


def test_c1_tiny_fp32_full_step():
    """Config 1: tiny fp32 decoder, 128-token Zipf prefix, 16-node tri-gram tree of depth 4."""
    wl = di.WORKLOADS["c1"]
    cfg = wl.model
    w = di.make_weights(cfg, seed=0)
    prefix, parent, token = di.workload_tree(wl, seed=0)
    ver = _verifier(cfg, w, max_batch=1, kv_capacity=wl.prefix_len + wl.n_nodes, max_nodes=wl.n_nodes)
    gpu_prefill(ver, [prefix])
    _, pk, pv = oracle.prefill(cfg, w, prefix)
    err, unsure = check_step(cfg, w, ver, prefix, parent, token, pk, pv)
    print(f"c1: max |logit error| {err:.2e}, nodes under the {MARGIN} margin: {unsure}/{wl.n_nodes}")
    ver.close()


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_small_model_trees_and_edge_cases(dtype):
    """Gains != 1, GQA, P = 0, single-node tree, ragged node counts, trees deeper than one mask word."""
    hd = 128 if dtype == "bf16" else 32
    cfg = di.ModelConfig("edge-" + dtype, 2, 128, 4, 2, hd, 256, 320, dtype=dtype)
    w = di.make_weights(cfg, seed=4, gain_jitter=0.1)
    ver = _verifier(cfg, w, max_batch=1, kv_capacity=512, max_nodes=80)
    # P = 0: the tree is the whole sequence
    parent = di.random_tree(9, None, seed=1)
    token = di.zipf_tokens(cfg.vocab, 9, seed=2)
    check_step(cfg, w, ver, np.zeros(0, np.int32), parent, token, None, None)
    # single node (plain autoregressive step) after a 70-token prefix (ragged tail inside a 64-key tile)
    prefix = di.zipf_tokens(cfg.vocab, 70, seed=3)
    _, pk, pv = oracle.prefill(cfg, w, prefix)
    ver2 = _verifier(cfg, w, max_batch=1, kv_capacity=512, max_nodes=80)
    gpu_prefill(ver2, [prefix], chunk=33)
    check_step(cfg, w, ver2, prefix, np.array([-1], np.int32), token[:1], pk, pv)
    # the accepted step moved the cache on: rebuild and run a 77-node tree (second mask word in use)
    ver3 = _verifier(cfg, w, max_batch=1, kv_capacity=512, max_nodes=80)
    gpu_prefill(ver3, [prefix], chunk=80)
    parent = di.random_tree(77, None, seed=5)
    token = di.zipf_tokens(cfg.vocab, 77, seed=6)
    check_step(cfg, w, ver3, prefix, parent, token, pk, pv)
    for v in (ver, ver2, ver3):
        v.close()


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_errors_leave_the_context_usable(dtype):
    """Every rejected call returns its documented code before anything is launched, and the step after the
    errors is as correct as any other."""
    from paper_2407_12021_amd import binding as B
    hd = 128 if dtype == "bf16" else 32
    cfg = di.ModelConfig("err-" + dtype, 2, 128, 2, 2, hd, 256, 512, dtype=dtype)
    w = di.make_weights(cfg, seed=3, gain_jitter=0.1, std=0.05)
    ver = _verifier(cfg, w, max_batch=2, kv_capacity=128, max_nodes=16)
    prefix = di.zipf_tokens(512, 20, seed=1)
    gpu_prefill(ver, [prefix])
    _, pk, pv = oracle.prefill(cfg, w, prefix)
    parent = di.random_tree(12, None, seed=2)
    token = di.zipf_tokens(512, 12, seed=3)

    def code(fn):
        try:
            fn()
            return B.DED_OK
        except B.DedError as e:
            return e.code

    bad_parent = parent.copy()
    bad_parent[5] = 7  # a parent that comes after its child
    bad_token = token.copy()
    bad_token[3] = 512  # outside the vocabulary
    assert code(lambda: ver.verify_step([20], [bad_parent], [token])) == B.DED_ETREE
    assert code(lambda: ver.verify_step([20], [parent], [bad_token])) == B.DED_ETOKEN
    assert code(lambda: ver.verify_step([120], [parent], [token])) == B.DED_ECAP
    assert code(lambda: ver.verify_step([20] * 3, [parent] * 3, [token] * 3)) == B.DED_EINVAL  # above max_batch
    assert code(lambda: ver.accept(mode=0)) == B.DED_ESTATE  # nothing pending
    check_step(cfg, w, ver, prefix, parent, token, pk, pv)
    ver.verify_step([21], [parent], [token])
    assert code(lambda: ver.accept(mode=1)) == B.DED_ETREE  # forced acceptance needs a chain
    ver.accept(mode=0)
    ver.close()


def test_random_shapes_prefixes_and_trees():
    """60 seeded random cases over model shape (0-3 layers, widths, head counts with grouped-query ratios 1 / 2 / 4,
    FFN widths, vocabularies that are not multiples of 64), prefix length (0, 1, around the 64-key tile edge, 200),
    node budget and tree size (1 .. 100 nodes, two mask words): each a full check_step against the oracle."""
    g = np.random.default_rng(20240717)
    worst = {"fp32": 0.0, "bf16": 0.0}
    for case in range(60):
        dtype = "bf16" if case % 2 else "fp32"
        Hkv = int(g.choice([1, 2, 3]))
        H = Hkv * int(g.choice([1, 2, 4]))
        if dtype == "bf16":
            hd, d, F, V = 128, int(g.choice([128, 256, 384])), int(g.choice([128, 384, 640])), int(g.choice([496, 512, 1008, 2064]))
        else:
            hd, d, F, V = int(g.choice([16, 32, 64, 128])), int(g.choice([48, 64, 96, 200])), int(g.choice([40, 96, 136])), int(g.choice([97, 500, 1000]))
        L = int(g.choice([0, 1, 2, 3]))
        max_nodes = int(g.choice([1, 5, 16, 33, 64, 100]))
        P = int(g.choice([0, 1, 7, 63, 64, 65, 130, 200]))
        n = int(g.integers(1, max_nodes + 1))
        cfg = di.ModelConfig(f"rnd{case}", L, d, H, Hkv, hd, F, V, dtype=dtype)
        w = di.make_weights(cfg, seed=100 + case, gain_jitter=0.1, std=0.04)
        prefix = di.zipf_tokens(V, P, seed=200 + case) if P else np.zeros(0, np.int32)
        parent = di.random_tree(n, None, seed=300 + case)
        token = di.zipf_tokens(V, n, seed=400 + case)
        print(f"case {case}: {dtype} L{L} d{d} H{H}/{Hkv} hd{hd} F{F} V{V} P{P} n{n}/{max_nodes}", flush=True)
        ver = _verifier(cfg, w, max_batch=1, kv_capacity=((P + max_nodes + 63) // 64) * 64, max_nodes=max_nodes)
        pk = pv = None
        if P:
            gpu_prefill(ver, [prefix])
            if L:
                _, pk, pv = oracle.prefill(cfg, w, prefix)
        err, _ = check_step(cfg, w, ver, prefix, parent, token, pk, pv)
        worst[dtype] = max(worst[dtype], err)
        ver.close()
    print(f"worst logit error: fp32 {worst['fp32']:.2e}, bf16 {worst['bf16']:.2e}")


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_batch_of_independent_trees(dtype):
    """Independent tree, prefix length and node count per sequence; no cross-sequence attention."""
    hd = 128 if dtype == "bf16" else 64
    cfg = di.ModelConfig("batch-" + dtype, 1, 128, 2, 2, hd, 128, 256, dtype=dtype)
    w = di.make_weights(cfg, seed=7, gain_jitter=0.05)
    B = 3
    ver = _verifier(cfg, w, max_batch=B, kv_capacity=192, max_nodes=24)
    plens = [40, 40, 40]
    prefixes = [di.zipf_tokens(cfg.vocab, 40, seed=8, stream=b) for b in range(B)]
    gpu_prefill(ver, prefixes, seq_count=B)
    nn = [24, 5, 17]
    parents = [di.random_tree(n, None, seed=10 + b) for b, n in enumerate(nn)]
    tokens = [di.zipf_tokens(cfg.vocab, n, seed=11, stream=b) for b, n in enumerate(nn)]
    logits = ver.verify_step(plens, parents, tokens, want_logits=True).cpu().numpy()
    a_gpu, _ = ver.get_argmax()
    acc, path, newp = ver.accept(mode=0)
    for b in range(B):
        _, pk, pv = oracle.prefill(cfg, w, prefixes[b])
        ref, kr, vr = oracle.verify_tree(cfg, w, parents[b], tokens[b], pk, pv)
        assert np.abs(logits[b, : nn[b]] - ref).max() <= TOL[dtype]
        acc2, path2 = oracle.accept_walk(parents[b], tokens[b], a_gpu[b, : nn[b]])
        assert acc[b] == acc2 and path[b] == path2 and newp[b] == 40 + len(path2)
        k_gpu, v_gpu = ver.kv_load(0, b, 0, newp[b])
        k_ref = oracle.compact_rows(pk[0], kr[0], path[b])
        assert np.abs(k_gpu.float().cpu().numpy().transpose(1, 0, 2) - k_ref).max() <= TOL[dtype] * 4
    ver.close()


def test_random_ragged_batches():
    """40 seeded random batches (2 / 3 / 5 sequences) with ragged prefix lengths and tree sizes: logits, decisions,
    walk, new prefix length and the compacted cache of every layer against the oracle, sequence by sequence."""
    g = np.random.default_rng(77)
    for case in range(40):
        dtype = "bf16" if case % 2 else "fp32"
        Hkv = int(g.choice([1, 2]))
        H = Hkv * int(g.choice([1, 2, 4]))
        if dtype == "bf16":
            hd, d, F, V = 128, int(g.choice([128, 256])), int(g.choice([128, 384])), int(g.choice([496, 512, 1008]))
        else:
            hd, d, F, V = int(g.choice([16, 64])), int(g.choice([48, 96])), int(g.choice([40, 136])), int(g.choice([97, 500]))
        L = int(g.choice([1, 2]))
        B = int(g.choice([2, 3, 5]))
        max_nodes = int(g.choice([4, 16, 40, 70]))
        Pc = int(g.choice([0, 7, 64, 130]))  # common part of the prefixes; each sequence then gets 1..16 tokens more
        ext = [int(g.integers(1, min(16, max_nodes) + 1)) for _ in range(B)]
        nn = [int(g.integers(1, max_nodes + 1)) for _ in range(B)]
        cfg = di.ModelConfig(f"rb{case}", L, d, H, Hkv, hd, F, V, dtype=dtype)
        w = di.make_weights(cfg, seed=500 + case, gain_jitter=0.1, std=0.04)
        prefixes = [di.zipf_tokens(V, Pc + ext[b], seed=600 + case, stream=b) for b in range(B)]
        print(f"case {case}: {dtype} L{L} d{d} H{H}/{Hkv} hd{hd} F{F} V{V} B{B} Pc{Pc} ext{ext} n{nn}/{max_nodes}", flush=True)
        ver = _verifier(cfg, w, max_batch=B, kv_capacity=((Pc + 16 + max_nodes + 63) // 64) * 64, max_nodes=max_nodes)
        if Pc:
            gpu_prefill(ver, [p[:Pc] for p in prefixes], seq_count=B)
        ver.verify_step([Pc] * B, [di.chain_tree(e) for e in ext], [prefixes[b][Pc:] for b in range(B)])
        _, _, newp = ver.accept(mode=1)
        plens = [Pc + e for e in ext]
        assert newp == plens
        parents = [di.random_tree(n, None, seed=700 + case + b) for b, n in enumerate(nn)]
        tokens = [di.zipf_tokens(V, n, seed=800 + case, stream=b) for b, n in enumerate(nn)]
        logits = ver.verify_step(plens, parents, tokens, want_logits=True).cpu().numpy()
        a_gpu, _ = ver.get_argmax()
        acc, path, newp = ver.accept(mode=0)
        for b in range(B):
            _, pk, pv = oracle.prefill(cfg, w, prefixes[b])
            ref, kr, vr = oracle.verify_tree(cfg, w, parents[b], tokens[b], pk, pv)
            assert np.abs(logits[b, : nn[b]] - ref).max() <= TOL[dtype]
            a_ref, margin = oracle.argmax_margin(ref)
            sure = margin > MARGIN
            assert (a_gpu[b, : nn[b]][sure] == a_ref[sure]).all()
            acc2, path2 = oracle.accept_walk(parents[b], tokens[b], a_gpu[b, : nn[b]])
            assert acc[b] == acc2 and path[b] == path2 and newp[b] == plens[b] + len(path2)
            for l in range(L):
                k_gpu, v_gpu = ver.kv_load(l, b, 0, newp[b])
                k_ref = oracle.compact_rows(pk[l], kr[l], path[b])
                v_ref = oracle.compact_rows(pv[l], vr[l], path[b])
                scale = max(1.0, np.abs(k_ref).max(), np.abs(v_ref).max())
                assert np.abs(k_gpu.float().cpu().numpy().transpose(1, 0, 2) - k_ref).max() <= TOL[dtype] * scale
                assert np.abs(v_gpu.float().cpu().numpy().transpose(1, 0, 2) - v_ref).max() <= TOL[dtype] * scale
        ver.close()


def test_random_planted_trees_over_three_steps():
    """30 seeded random cases, three steps each: random branched trees in which, level by level, a random subset of
    nodes is given the model's own token of its parent (so the walk goes several levels deep and has to choose among
    branches), verified, accepted and compacted; the next step runs on the compacted cache.  The oracle sees token ids
    only (its own prefill of everything committed so far): logits relative to their scale, the walk bit for bit on the
    GPU's tokens (and on the oracle's where margins allow), new prefix length, and every layer's cache rows."""
    g = np.random.default_rng(4242)
    lengths = {}
    for case in range(30):
        dtype = "bf16" if case % 2 else "fp32"
        Hkv = int(g.choice([1, 2]))
        H = Hkv * int(g.choice([1, 2]))
        if dtype == "bf16":
            hd, d, F, V = 128, int(g.choice([128, 256])), int(g.choice([128, 384])), int(g.choice([496, 512]))
        else:
            hd, d, F, V = int(g.choice([16, 64])), int(g.choice([48, 96])), int(g.choice([40, 136])), int(g.choice([97, 500]))
        L = int(g.choice([1, 2, 3]))
        max_nodes = int(g.choice([8, 24, 64, 90]))
        P0 = int(g.choice([0, 3, 60, 64, 129]))
        cfg = di.ModelConfig(f"pl{case}", L, d, H, Hkv, hd, F, V, dtype=dtype)
        w = di.make_weights(cfg, seed=1500 + case, gain_jitter=0.1, std=0.15)  # wide top-1 margins
        seq = di.zipf_tokens(V, P0 + 1, seed=1600 + case).tolist()  # committed tokens; the last one is the root
        print(f"case {case}: {dtype} L{L} d{d} H{H}/{Hkv} hd{hd} F{F} V{V} P0 {P0} max_nodes {max_nodes}", flush=True)
        ver = _verifier(cfg, w, max_batch=1, kv_capacity=((P0 + 4 * max_nodes + 63) // 64) * 64 + 64, max_nodes=max_nodes)
        if P0:
            gpu_prefill(ver, [np.array(seq[:P0], np.int32)])
        P = P0
        for step in range(3):
            n = int(g.integers(1, max_nodes + 1))
            parent = di.random_tree(n, None, seed=1700 + 10 * case + step)
            depth = oracle.node_depths(parent)
            token = di.zipf_tokens(V, n, seed=1800 + 10 * case + step).copy()
            token[0] = seq[-1]
            for lvl in range(1, int(depth.max()) + 1 if n > 1 else 1):
                ver.verify_step([P], [parent], [token])
                a, _ = ver.get_argmax()
                for i in np.flatnonzero(depth == lvl):
                    taken = any(parent[j] == parent[i] and j < i and token[j] == a[0, parent[i]] for j in range(n))
                    if g.random() < 0.6 and not taken:
                        token[i] = a[0, parent[i]]
            pk = pv = None
            if P:
                _, pk, pv = oracle.prefill(cfg, w, np.array(seq[:P], np.int32))
            ref, kr, vr = oracle.verify_tree(cfg, w, parent, token, pk, pv)
            logits = ver.verify_step([P], [parent], [token], want_logits=True)[0, :n].cpu().numpy().astype(np.float64)
            err = np.abs(logits - ref).max()
            # N(0, 0.15) weights give logits far wider than the benchmark's N(0, 0.02) (|logit| up to ~40): the bound
            # here is this test's own, relative to the logit scale (1 % of the largest logit), NOT the absolute 2e-2
            # of the benchmark configurations, which test_gpu_full_size / test_gpu_big_shapes assert as such
            assert err <= (1e-4 if dtype == "fp32" else 1e-2) * max(1.0, np.abs(ref).max()), (err, np.abs(ref).max())
            a_gpu, _ = ver.get_argmax()
            acc, path, newp = ver.accept(mode=0)
            acc2, path2 = oracle.accept_walk(parent, token, a_gpu[0, :n])
            assert acc[0] == acc2 and path[0] == path2 and newp[0] == P + len(path2)
            lengths[len(path2)] = lengths.get(len(path2), 0) + 1
            a_ref, margin = oracle.argmax_margin(ref)
            acc3, path3 = oracle.accept_walk(parent, token, a_ref)
            if all(margin[v] > MARGIN for v in set(path2) | set(path3)):
                assert acc2 == acc3 and path2 == path3
            for l in range(L):
                k_gpu, v_gpu = ver.kv_load(l, 0, 0, newp[0])
                k_ref = oracle.compact_rows(pk[l] if P else kr[l][:0], kr[l], path2)
                v_ref = oracle.compact_rows(pv[l] if P else vr[l][:0], vr[l], path2)
                scale = max(1.0, np.abs(k_ref).max(), np.abs(v_ref).max())
                assert np.abs(k_gpu.float().cpu().numpy().transpose(1, 0, 2) - k_ref).max() <= 2 * TOL[dtype] * scale
                assert np.abs(v_gpu.float().cpu().numpy().transpose(1, 0, 2) - v_ref).max() <= 2 * TOL[dtype] * scale
            seq = seq[:P] + [int(token[v]) for v in path2] + [int(acc2[-1])]
            P = newp[0]
            assert len(seq) == P + 1
        ver.close()
    print(f"accepted path lengths: {dict(sorted(lengths.items()))}")
    assert sum(c for k, c in lengths.items() if k >= 3) >= 20  # the walks did go deep


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_lossless_multi_step_decode(dtype):
    """Sec. 2.4: draft-verification decoding reproduces plain greedy autoregressive decoding.
    Drafts are random except for a planted branch; compared token by token while margins allow."""
    hd = 128 if dtype == "bf16" else 32
    cfg = di.ModelConfig("loss-" + dtype, 2, 128, 2, 2, hd, 256, 512, dtype=dtype)
    w = di.make_weights(cfg, seed=13, gain_jitter=0.1, std=0.3)  # seed / std chosen for wide oracle margins
    prompt = di.zipf_tokens(cfg.vocab, 9, seed=13).tolist()
    n_new = 24
    # oracle AR with margins
    seq = list(prompt)
    ar, margins = [], []
    for _ in range(n_new):
        lg = oracle.autoregressive_logits(cfg, w, seq)[-1]
        a, m = oracle.argmax_margin(lg[None])
        ar.append(int(a[0]))
        margins.append(float(m[0]))
        seq.append(int(a[0]))
    ver = _verifier(cfg, w, max_batch=1, kv_capacity=256, max_nodes=16)
    gpu_prefill(ver, [np.array(prompt[:-1], np.int32)])
    P, root, produced = len(prompt) - 1, prompt[-1], []
    g = np.random.default_rng(0)
    step = 0
    while len(produced) < n_new:
        m = step % 4
        known = ar[len(produced): len(produced) + m]
        parent = [-1] + list(range(len(known)))
        token = [root] + known
        for _ in range(6):
            parent.append(int(g.integers(0, len(token))))
            token.append(int(g.integers(0, cfg.vocab)))
        ver.verify_step([P], [parent], [token])
        acc, path, newp = ver.accept(mode=0)
        produced.extend(acc[0])
        P, root = newp[0], acc[0][-1]
        step += 1
    first_unsure = next((i for i, mg in enumerate(margins) if mg <= MARGIN), n_new)
    assert produced[:first_unsure] == ar[:first_unsure]
    assert first_unsure >= 12, "test model too flat to say anything"
    ver.close()


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_whole_loop_with_the_draft_maker_is_lossless(dtype):
    """The method end to end (Fig. 2 / Appendix H data flow): tri-gram matrix -> tree search -> pseudo-sequence ->
    verification -> approval -> Adjust3Gram, every part behind the C ABI.  The corpus holds the oracle's own greedy
    continuation among distractors, so some drafts are right and some are wrong; whatever is proposed, the output
    must be the oracle's plain autoregressive decoding (Sec. 2.4), and the matrix must have learnt the output."""
    from paper_2407_12021_amd import binding as B
    hd = 128 if dtype == "bf16" else 32
    cfg = di.ModelConfig("loop-" + dtype, 2, 128, 2, 2, hd, 256, 512, dtype=dtype)
    w = di.make_weights(cfg, seed=13, gain_jitter=0.1, std=0.3)
    prompt = di.zipf_tokens(cfg.vocab, 9, seed=13).tolist()
    n_new = 24
    seq, ar, margins = list(prompt), [], []
    for _ in range(n_new + 6):
        lg = oracle.autoregressive_logits(cfg, w, seq)[-1]
        a, m = oracle.argmax_margin(lg[None])
        ar.append(int(a[0]))
        margins.append(float(m[0]))
        seq.append(int(a[0]))
    g = np.random.default_rng(1)
    drafter = B.Drafter()
    for i in range(len(prompt), len(seq)):  # the true tri-gram among 3 wrong successors; weak every third position
        a, c, true = seq[i - 2], seq[i - 1], seq[i]
        for x in g.choice(cfg.vocab, size=3, replace=False).tolist():
            if x != true:
                drafter.count([a, c, x], 20)
                drafter.count([c, x, int(g.integers(0, cfg.vocab))], 15)
        drafter.count([a, c, true], 6 if i % 3 == 0 else 30)  # 6 < t: eliminated, the draft breaks there
    drafter.finalize(12)
    ver = _verifier(cfg, w, max_batch=1, kv_capacity=256, max_nodes=16)
    gpu_prefill(ver, [np.array(prompt[:-1], np.int32)])
    P, prev, root, produced, accepted_drafts, steps = len(prompt) - 1, prompt[-2], prompt[-1], [], 0, 0
    while len(produced) < n_new:
        cands = [wd for _, wd in drafter.mcts(prev, root, g.random(60 * 3), iterations=60, l=3, n=8)]
        rc, parent, token, _ = B.ded_build_tree(root, cands, 16)
        assert rc == B.DED_OK
        ver.verify_step([P], [parent], [token])
        acc, path, newp = ver.accept(mode=0)
        produced.extend(acc[0])
        accepted_drafts += len(acc[0]) - 1
        drafter.adjust([prev, root] + acc[0], 16, 0.25, 1.0)
        prev = acc[0][-2] if len(acc[0]) > 1 else root
        P, root = newp[0], acc[0][-1]
        steps += 1
    first_unsure = next((i for i, mg in enumerate(margins) if mg <= MARGIN), n_new)
    assert produced[:first_unsure] == ar[:first_unsure]
    assert first_unsure >= 12, "test model too flat to say anything"
    assert accepted_drafts >= 4 and steps < n_new, (accepted_drafts, steps)  # the search found real drafts
    # self-improvement: every tri-gram of the committed output is now in the matrix with at least the increment
    out = prompt[-2:] + produced
    for i in range(2, len(out)):
        p_i = dict(drafter.successors(out[i - 2], out[i - 1])).get(out[i], 0.0)
        assert p_i >= 0.25, (i, p_i)
    drafter.close()
    ver.close()


@pytest.mark.parametrize("dtype,P,N,H,Hkv", [
    ("fp32", 100, 20, 4, 2),
    ("bf16", 333, 50, 4, 2),     # 2 heads x 64 rows per kv head: the 128-row kernel shape, 3 key ranges
    ("bf16", 0, 16, 2, 2),       # no prefix at all: one ragged tile of tree keys
    ("bf16", 1500, 64, 2, 2),    # the 64-row shape, 8 key ranges, the last one holding the tree tile
    ("bf16", 130, 100, 4, 4),    # 112 padded rows: the 128-row shape with an empty row block, 2 mask words
    ("bf16", 700, 60, 8, 2),     # 4 heads x 64 rows per kv head: the 256-row shape, 3 key ranges
    ("bf16", 64, 200, 2, 1),     # 2 heads x 208 rows: two 256-row tiles (the second ragged), 4 mask words
    ("bf16", 2100, 256, 8, 2),   # 4 heads x 256 rows, 32 prefix tiles: the 256-row shape's pipelined prefix loop, in key
                                 # ranges that start inside the prefix, end inside it or hold the tree tiles
    ("bf16", 200, 128, 4, 1),    # 4 heads x 128 rows, one key range: 3 pipelined prefix tiles, then the masked tiles
])
def test_tree_attention_only(dtype, P, N, H, Hkv):
    """The attention layer on its own with injected q / K / V (config-2 style, small); the 16-bit cases walk through
    the kernel's workgroup shapes, with and without key ranges, ragged row tiles and 1 - 4 mask words."""
    import torch
    hd = 128 if dtype == "bf16" else 64
    cfg = di.ModelConfig("attn-" + dtype, 1, 128, H, Hkv, hd, 128, 64, dtype=dtype)
    w = di.make_weights(cfg, seed=1)
    ver = _verifier(cfg, w, max_batch=1, kv_capacity=P + N + 7, max_nodes=N)
    x = di.attention_inputs(H, Hkv, hd, P, N, seed=3, dtype=dtype)
    parent = di.random_tree(N, None, seed=4)
    if P:
        ver.kv_store(0, 0, 0, x["k_prefix"], x["v_prefix"])
    from paper_2407_12021_amd.binding import _to_device
    q = _to_device(x["q"], ver.device, dtype)[None]
    kt = _to_device(x["k_tree"], ver.device, dtype)[None]
    vt = _to_device(x["v_tree"], ver.device, dtype)[None]
    out = ver.tree_attention(0, [P], [parent], q, kt, vt)
    torch.cuda.synchronize()
    got = out[0].float().cpu().numpy()
    kk = np.concatenate([oracle.widen(x["k_prefix"]), oracle.widen(x["k_tree"])], axis=1).transpose(1, 0, 2)
    vv = np.concatenate([oracle.widen(x["v_prefix"]), oracle.widen(x["v_tree"])], axis=1).transpose(1, 0, 2)
    vis = np.concatenate([np.ones((N, P), bool), oracle.ancestor_mask(parent)], axis=1)
    ref = oracle.masked_attention(oracle.widen(x["q"]), kk, vv, vis)
    err = np.abs(got - ref).max()
    # outputs are O(1); bf16 output rounding alone is 2^-9 relative
    assert err <= (2e-5 if dtype == "fp32" else 2e-2), err
    # K/V round trip through the library layout: exact for every value of magnitude >= 2^-14; the 16-bit cache holds
    # f16, so a smaller bf16 value lands on the f16 subnormal grid (spacing 2^-24), at most 2^-25 away
    if P:
        k_back, v_back = ver.kv_load(0, 0, 0, P)
        for back, sent in ((k_back, x["k_prefix"]), (v_back, x["v_prefix"])):
            a, b = back.float().cpu().numpy(), oracle.widen(sent).astype(np.float32)
            big = np.abs(b) >= 2.0 ** -14
            assert np.array_equal(a[big], b[big])
            assert np.abs(a - b).max() <= (2.0 ** -25 if dtype == "bf16" else 0.0)
    ver.close()


def test_zero_layer_bf16_gemm_path():
    """L = 0: logits = lm_head . rmsnorm(emb[token]) -- isolates embedding, norm, the MFMA GEMM, argmax."""
    cfg = di.ModelConfig("L0-bf16", 0, 256, 2, 2, 128, 128, 1008, dtype="bf16")
    w = di.make_weights(cfg, seed=2, gain_jitter=0.2, std=0.3)
    ver = _verifier(cfg, w, max_batch=2, kv_capacity=64, max_nodes=40)
    parents = [di.random_tree(40, None, seed=1), di.random_tree(7, None, seed=2)]
    tokens = [di.zipf_tokens(cfg.vocab, 40, seed=3), di.zipf_tokens(cfg.vocab, 7, seed=4)]
    logits = ver.verify_step([0, 0], parents, tokens, want_logits=True).cpu().numpy()
    a_gpu, _ = ver.get_argmax()
    for b, n in enumerate((40, 7)):
        ref, _, _ = oracle.verify_tree(cfg, w, parents[b], tokens[b])
        # N(0, 0.3) LM-head weights: logits of width ~5; this test's own bound scales with them (see above)
        assert np.abs(logits[b, :n] - ref).max() <= 2e-2 * max(1.0, np.abs(ref).max() / 4)
        assert (a_gpu[b, :n] == np.argmax(logits[b, :n], axis=1)).all()
    ver.close()


@pytest.mark.parametrize("shape", ["ragged-vocab", "32000", "large-rows"])
def test_fused_argmax_equals_argmax_of_materialised_logits(shape):
    """Without a logits request the LM-head GEMM hands the argmax its per-tile candidates and the [rows][vocab]
    logits never reach memory; with one they are written and reduced by the stand-alone kernel.  Tokens and
    margins must be equal bit for bit (the merge rule is order-independent), on a vocabulary with a ragged last
    feature group, on the benchmark's vocabulary, and through the large-row GEMM (batched trees, split-K)."""
    if shape == "ragged-vocab":
        cfg, batch, nodes = di.ModelConfig("t2-a", 1, 256, 2, 2, 128, 128, 1008, dtype="bf16"), 2, 40
    elif shape == "32000":
        cfg, batch, nodes = di.ModelConfig("t2-b", 1, 512, 4, 4, 128, 256, 32000, dtype="bf16"), 1, 64
    else:
        cfg, batch, nodes = di.ModelConfig("t2-c", 1, 512, 4, 2, 128, 256, 4112, dtype="bf16"), 4, 128
    w = di.make_weights(cfg, seed=21, gain_jitter=0.1, std=0.05)
    # duplicate LM-head rows make exact ties (margin 0, lowest id must win) part of the comparison
    w["lm_head"][17] = w["lm_head"][3]
    w["lm_head"][cfg.vocab - 1] = w["lm_head"][cfg.vocab - 70]
    ver = _verifier(cfg, w, max_batch=batch, kv_capacity=64 + nodes, max_nodes=nodes)
    parents = [di.random_tree(nodes - 3 * b, None, seed=30 + b) for b in range(batch)]
    tokens = [di.zipf_tokens(cfg.vocab, nodes - 3 * b, seed=40 + b) for b in range(batch)]
    ver.verify_step([0] * batch, parents, tokens)  # fused
    a_f, m_f = ver.get_argmax()
    acc_f = ver.accept(mode=0)
    logits = ver.verify_step([0] * batch, parents, tokens, want_logits=True).cpu().numpy()  # materialised
    a_m, m_m = ver.get_argmax()
    acc_m = ver.accept(mode=0)
    assert np.array_equal(a_f, a_m) and np.array_equal(m_f, m_m) and acc_f == acc_m
    ties = 0
    for b in range(batch):
        n = len(parents[b])
        assert (a_f[b, :n] == np.argmax(logits[b, :n], axis=1)).all()
        top2 = np.partition(logits[b, :n], -2, axis=1)[:, -2:]
        assert np.array_equal(m_f[b, :n], top2[:, 1] - top2[:, 0])
        ties += int((m_f[b, :n] == 0).sum())
    print(f"fused argmax [{shape}]: equal to the materialised one on {sum(len(p) for p in parents)} nodes ({ties} exact ties)")
    ver.close()
    if shape != "ragged-vocab":
        return
    # exact ties at the top of EVERY row: the vocabulary's second half repeats the first (partners 504 ids apart,
    # i.e. in different feature groups and wavefronts), then neighbours repeat each other (partners inside one
    # lane's four features).  The lowest id must win and the margin must be exactly zero, fused and materialised.
    for variant in ("halves", "neighbours"):
        w2 = dict(w)
        lm = w["lm_head"].copy()
        if variant == "halves":
            lm[504:] = lm[:504]
        else:
            lm[1::2] = lm[0::2]
        w2["lm_head"] = lm
        ver = _verifier(cfg, w2, max_batch=batch, kv_capacity=64 + nodes, max_nodes=nodes)
        ver.verify_step([0] * batch, parents, tokens)
        a_f, m_f = ver.get_argmax()
        ver.accept(mode=0)
        ver.verify_step([0] * batch, parents, tokens, want_logits=True)
        a_m, m_m = ver.get_argmax()
        ver.accept(mode=0)
        assert np.array_equal(a_f, a_m) and np.array_equal(m_f, m_m)
        for b in range(batch):
            n = len(parents[b])
            assert (m_f[b, :n] == 0).all()
            assert (a_f[b, :n] < 504).all() if variant == "halves" else (a_f[b, :n] % 2 == 0).all()
        ver.close()


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_non_finite_logits_are_reported_not_walked(dtype):
    """A token whose embedding lies outside the half-precision operand range (bf16 storage holds it, the f16
    matrix-core operands do not) or is infinite (fp32) makes the logits of its node NaN: ded_get_argmax, ded_sample
    and ded_accept return DED_ENONFINITE instead of a token, nothing of that sequence is kept, and the next,
    finite step on the same context is as correct as any other."""
    from paper_2407_12021_amd import binding as B
    hd = 128 if dtype == "bf16" else 32
    cfg = di.ModelConfig("nf-" + dtype, 2, 128, 2, 1, hd, 128, 320, dtype=dtype)
    w = di.make_weights(cfg, seed=12, gain_jitter=0.1)
    poison = 77
    if dtype == "bf16":
        w["emb"][poison] = di.f32_to_bf16_bits(np.full(cfg.d_model, 3.0e38, np.float32))
    else:
        w["emb"][poison] = np.inf
    prefix = di.zipf_tokens(cfg.vocab, 40, seed=3)
    prefix = np.where(prefix == poison, poison + 1, prefix).astype(np.int32)
    ver = _verifier(cfg, w, max_batch=2, kv_capacity=192, max_nodes=24)
    gpu_prefill(ver, [prefix, prefix], seq_count=2)
    _, pk, pv = oracle.prefill(cfg, w, prefix)
    parent = di.random_tree(20, None, seed=5)
    clean = di.zipf_tokens(cfg.vocab, 20, seed=6)
    clean = np.where(clean == poison, poison + 1, clean).astype(np.int32)
    bad = clean.copy()
    bad[11] = poison
    P = len(prefix)
    for use_sample in (False, True):
        ver.verify_step([P, P], [parent, parent], [clean, bad])
        rc, _, _ = B.ded_get_argmax(ver.ctx, 2, ver.max_nodes)
        assert rc == B.DED_ENONFINITE
        if use_sample:
            with pytest.raises(B.DedError) as e:
                ver.sample(1.0, 0.9, [np.full(20, 0.5, np.float32)] * 2)
            assert e.value.code == B.DED_ENONFINITE
        rc, _, nacc, _, newp = B.ded_accept(ver.ctx, 0, 2, ver.max_nodes)
        assert rc == B.DED_ENONFINITE and nacc.tolist() == [0, 0] and newp.tolist() == [0, 0]  # nothing written
        rc, *_ = B.ded_accept(ver.ctx, 0, 2, ver.max_nodes)
        assert rc == B.DED_ESTATE  # the step was consumed
    # the poisoned step kept nothing of either sequence: a finite step from the same prefix is right in both.  Its
    # tree is SMALLER, so the slot that held the NaN key / value lies in the dead tail of the tile that the
    # attention kernel still fetches: it must have been zeroed.
    small, n2 = di.random_tree(9, None, seed=7), 9
    want = ver.verify_step([P, P], [small, small], [clean[:n2], clean[:n2]], want_logits=True).cpu().numpy()
    ref, _, _ = oracle.verify_tree(cfg, w_finite(w, poison), small, clean[:n2], pk, pv)
    for b in range(2):
        assert np.abs(want[b, :n2] - ref).max() <= TOL[dtype]
    a_gpu, _ = ver.get_argmax()
    acc, path, newp = ver.accept(mode=0)
    for b in range(2):
        acc2, path2 = oracle.accept_walk(small, clean[:n2], a_gpu[b, :n2])
        assert acc[b] == acc2 and path[b] == path2 and newp[b] == P + len(path2)
    ver.close()


def w_finite(w, row):
    """The same weights with the poisoned embedding row zeroed (the oracle widens whole matrices; the row is never
    looked up in the finite step)."""
    out = dict(w)
    emb = w["emb"].copy()
    emb[row] = 0
    out["emb"] = emb
    return out


SAMPLE_SLACK = 1e-4  # fp32 sums of up to 32000 weights against fp64: decisions closer than this to a boundary may flip


def _check_sampling(ver, logits_gpu, parents, tokens, combos, seed):
    """ded_sample against the oracle's sampler fed with the GPU's own fp32 logits (the decision is taken in the
    kernel's precision on both sides; logits parity is checked elsewhere).  Every decision is checked: the token
    must equal the oracle's when u is clear of every CDF step by SAMPLE_SLACK (counted as `exact`), and in any
    case u must lie inside the token's own CDF interval widened by SAMPLE_SLACK (with a 32000-token vocabulary
    the steps are ~3e-5 apart, so most decisions are of this second kind)."""
    g = np.random.default_rng(seed)
    exact = loose = 0
    for temperature, top_p in combos:
        us = [g.random(len(p)).astype(np.float32) for p in parents]
        ver.sample(temperature, top_p, us)
        a_gpu, _ = ver.get_argmax()
        for b, parent in enumerate(parents):
            n = len(parent)
            lg = logits_gpu[b, :n].astype(np.float64)
            ref, info = oracle.sample_rows(lg, temperature, top_p, us[b].astype(np.float64))
            for i in range(n):
                tok, u = int(a_gpu[b, i]), float(us[b][i])
                edge = info[i]["edge_mass"] if info[i]["nucleus_slack"] <= SAMPLE_SLACK else 0.0
                if info[i]["cdf_slack"] > SAMPLE_SLACK + edge:
                    assert tok == ref[i], (temperature, top_p, b, i)
                    exact += 1
                    continue
                x = lg[i] / temperature
                p = np.exp(x - x.max())
                p /= p.sum()
                keep = oracle.nucleus(p, top_p)
                if edge == 0.0:
                    assert keep[tok], (temperature, top_p, b, i)
                keep[tok] = True
                ids = np.flatnonzero(keep)
                cdf = np.cumsum(p[ids]) / p[ids].sum()
                pos = int(np.searchsorted(ids, tok))
                lo = cdf[pos - 1] if pos else 0.0
                assert lo - SAMPLE_SLACK - edge <= u <= cdf[pos] + SAMPLE_SLACK + edge, (temperature, top_p, b, i)
                loose += 1
    return exact, loose, a_gpu


@pytest.mark.parametrize("dtype", ["fp32", "bf16", "bf16-128k"])
def test_stochastic_approval(dtype):
    """Temperature / top-p sampling of the model's token and the walk that uses it.  The 128256-token vocabulary
    (Llama-3) does not fit the LDS-resident kernel and takes the one that works in global memory."""
    if dtype == "fp32":
        cfg = di.ModelConfig("samp-f32", 2, 64, 4, 2, 16, 96, 500, dtype="fp32")
    elif dtype == "bf16":
        cfg = di.ModelConfig("samp-bf16", 1, 256, 2, 2, 128, 128, 32000, dtype="bf16")  # full-size vocabulary
    else:
        cfg = di.ModelConfig("samp-bf16-128k", 1, 256, 2, 2, 128, 128, 128256, dtype="bf16")
    w = di.make_weights(cfg, seed=5, gain_jitter=0.1, std=0.3 if dtype == "fp32" else 0.08)
    ver = _verifier(cfg, w, max_batch=2, kv_capacity=128, max_nodes=40)
    prefixes = [di.zipf_tokens(cfg.vocab, 21, seed=7), di.zipf_tokens(cfg.vocab, 9, seed=8)]
    ver.verify_step([0, 0], [di.chain_tree(21), di.chain_tree(9)], prefixes)
    ver.accept(mode=1)
    parents = [di.random_tree(40, None, seed=1), di.random_tree(13, None, seed=2)]
    tokens = [di.zipf_tokens(cfg.vocab, 40, seed=3), di.zipf_tokens(cfg.vocab, 13, seed=4)]
    logits = ver.verify_step([21, 9], parents, tokens, want_logits=True).cpu().numpy()
    greedy, greedy_margin = ver.get_argmax()
    combos = [(1.0, 1.0), (0.7, 0.9), (1.5, 0.5), (1.0, 0.05), (0.3, 0.99), (2.0, 0.8)]
    exact, loose, _ = _check_sampling(ver, logits, parents, tokens, combos, seed=9)
    print(f"sampling [{dtype}], flat distributions: {exact} decisions equal to the oracle's, {loose} more within "
          f"{SAMPLE_SLACK} of a CDF step and inside their own CDF interval")
    # Peaked distributions (low temperature): a handful of tokens hold most of the mass, so the CDF steps that
    # matter are far wider than the slack and the decision itself is what is compared, also at the vocabulary
    # sizes whose flat distributions have steps of ~1e-5.
    peaked = [(0.05, 1.0), (0.1, 1.0), (0.1, 0.9), (0.15, 0.6), (0.2, 0.9), (0.2, 0.3), (0.25, 0.95), (0.08, 0.5),
              (0.12, 0.99), (0.3, 0.7)]
    if dtype == "fp32":
        peaked = [(3 * t, p) for t, p in peaked]  # 500 tokens with std 0.3 weights: the top logits lie ~3x further apart
    exact_pk, loose_pk, last = _check_sampling(ver, logits, parents, tokens, peaked, seed=10)
    print(f"sampling [{dtype}], peaked distributions: {exact_pk} equal to the oracle's, {loose_pk} near a CDF step")
    assert exact_pk >= 0.8 * (exact_pk + loose_pk)
    assert exact + exact_pk >= 0.5 * (exact + loose + exact_pk + loose_pk)
    # End to end: the oracle's OWN logits (fp64 forward from token ids) -> the oracle's sample, against the token the
    # library sampled, at every node where neither the logit error nor a CDF / nucleus boundary can flip the
    # decision: a logit error e moves every unnormalised weight by a factor within exp(+-e/T), so a CDF value
    # F = A / (A + B) moves by at most tanh(e/T) <= e/T (worst case: A up, B down, F = 1/2); the comparison asks
    # for twice that plus the summation slack on both sides of u, and likewise for the top-p boundary.
    pks, pvs, refs = [], [], []
    for b in range(2):
        _, pk, pv = oracle.prefill(cfg, w, prefixes[b])
        ref, _, _ = oracle.verify_tree(cfg, w, parents[b], tokens[b], pk, pv)
        refs.append(ref)
    err = max(np.abs(logits[b, :len(parents[b])] - refs[b]).max() for b in range(2))
    assert err <= TOL["fp32" if dtype == "fp32" else "bf16"], err
    g = np.random.default_rng(11)
    decided = total = 0
    for temperature, top_p in peaked + combos[:3]:
        us = [g.random(len(p)).astype(np.float32) for p in parents]
        ver.sample(temperature, top_p, us)
        a_gpu, _ = ver.get_argmax()
        need = 2.0 * err / temperature + 10 * SAMPLE_SLACK
        for b in range(2):
            ref_tok, info = oracle.sample_rows(refs[b], temperature, top_p, us[b].astype(np.float64))
            for i in range(len(parents[b])):
                total += 1
                edge = info[i]["edge_mass"] if info[i]["nucleus_slack"] <= need else 0.0
                if info[i]["cdf_slack"] > need + edge:
                    assert int(a_gpu[b, i]) == int(ref_tok[i]), (temperature, top_p, b, i)
                    decided += 1
        last = a_gpu
    print(f"sampling [{dtype}], from the oracle's own logits (max logit error {err:.2e}): {decided}/{total} decisions "
          f"clear of every boundary, all equal")
    assert decided >= 0.25 * total
    # the walk uses the sampled tokens
    acc, path, newp = ver.accept(mode=0)
    for b, (parent, token) in enumerate(zip(parents, tokens)):
        acc2, path2 = oracle.accept_walk(parent, token, last[b, :len(parent)])
        assert acc[b] == acc2 and path[b] == path2
    # a vanishing temperature is greedy decoding; errors
    ver.verify_step([21, 9], parents, tokens)
    ver.sample(1e-3, 1.0, [np.full(40, 0.5, np.float32), np.full(13, 0.999, np.float32)])
    cold, _ = ver.get_argmax()
    # at T = 1e-3 a runner-up closer than ~0.01 still holds visible mass: compare where the top-1 margin is clear
    clear = greedy_margin > 0.03
    assert clear.sum() >= 0.5 * clear.size and (cold[clear] == greedy[clear]).all()
    from paper_2407_12021_amd.binding import DedError
    for bad in ((0.0, 0.9, 0.5), (1.0, 0.0, 0.5), (1.0, 1.5, 0.5), (1.0, 0.9, 1.0), (1.0, 0.9, -0.1)):
        with pytest.raises(DedError):
            ver.sample(bad[0], bad[1], [np.full(40, bad[2], np.float32), np.full(13, 0.5, np.float32)])
    ver.accept(mode=0)
    with pytest.raises(DedError):  # no pending step
        ver.sample(1.0, 0.9, [np.full(40, 0.5, np.float32), np.full(13, 0.5, np.float32)])
    ver.close()


def test_sampler_when_the_running_sum_stops_short_of_the_target():
    """A case a random sweep found: a flat distribution over 36880 tokens (just above what the LDS-resident kernel
    holds) at T = 2.9, top-p 0.9, where for one node the scan places the target in a thread's chunk but that
    thread's own running sum, rounded in another order, ends just below it.  The token must still come from that
    chunk (an earlier version fell back to the last id of the whole nucleus)."""
    V = 36880
    cfg = di.ModelConfig("samp-edge", 1, 256, 2, 2, 128, 128, V, dtype="bf16")
    w = di.make_weights(cfg, seed=929, gain_jitter=0.1, std=0.1)
    nn = [28, 32]
    ver = _verifier(cfg, w, max_batch=2, kv_capacity=128, max_nodes=40)
    parents = [di.random_tree(n, None, seed=58 + b) for b, n in enumerate(nn)]
    tokens = [di.zipf_tokens(V, n, seed=79, stream=b) for b, n in enumerate(nn)]
    logits = ver.verify_step([0, 0], parents, tokens, want_logits=True).cpu().numpy()
    combos = [(0.2571029967541381, 1.0), (0.341189999444725, 0.5), (1.7843192694332748, 0.01), (2.909550738650948, 0.9)]
    exact, loose, _ = _check_sampling(ver, logits, parents, tokens, combos, seed=29)
    assert exact + loose == 4 * sum(nn)
    ver.accept(mode=0)
    ver.close()


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_maximum_tree_size_and_full_cache(dtype):
    """256 nodes (all four ancestor-mask words), once as a random tree and once as one 256-deep chain, with the
    cache filled to its last slot (prefix_len + n_nodes == kv_capacity)."""
    hd = 128 if dtype == "bf16" else 32
    cfg = di.ModelConfig("max-" + dtype, 1, 128, 2, 1, hd, 128, 192, dtype=dtype)
    w = di.make_weights(cfg, seed=8, gain_jitter=0.1)
    prefix = di.zipf_tokens(cfg.vocab, 64, seed=3)
    _, pk, pv = oracle.prefill(cfg, w, prefix)
    for parent in (di.random_tree(256, None, seed=5), di.chain_tree(256)):
        ver = _verifier(cfg, w, max_batch=1, kv_capacity=64 + 256, max_nodes=256)
        gpu_prefill(ver, [prefix], chunk=64)
        token = di.zipf_tokens(cfg.vocab, 256, seed=6)
        check_step(cfg, w, ver, prefix, parent, token, pk, pv)
        ver.close()
