"""The seeded input generators: determinism, shapes, tree validity (no GPU needed)."""
import numpy as np

import ded_inputs as di


def test_bf16_round_to_nearest_even():
    # 1 + 2^-8 lies halfway between bf16 neighbours 1.0 and 1 + 2^-7 -> ties to even (1.0)
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -0.3], dtype=np.float32)
    r = di.round_to_bf16(x)
    assert r[0] == 1.0 and r[1] == 1.0 + 2.0 ** -6 and r[2] == 1.0 + 2.0 ** -7
    assert abs(r[3] + 0.3) < 0.3 * 2.0 ** -8
    bits = di.f32_to_bf16_bits(x)
    assert np.array_equal(di.bf16_bits_to_f32(bits), r)


def test_weights_deterministic_and_scaled():
    cfg = di.ModelConfig("t", 2, 64, 4, 2, 16, 96, 128, dtype="bf16")
    a = di.make_weights(cfg, seed=5)
    b = di.make_weights(cfg, seed=5, threads=1)
    c = di.make_weights(cfg, seed=6)
    assert np.array_equal(a["layers"][1]["wd"], b["layers"][1]["wd"])
    assert not np.array_equal(a["layers"][1]["wd"], c["layers"][1]["wd"])
    assert a["layers"][0]["wq"].shape == (64, 64) and a["layers"][0]["wk"].shape == (32, 64)
    assert a["layers"][0]["wg"].shape == (96, 64) and a["layers"][0]["wd"].shape == (64, 96)
    std = di.bf16_bits_to_f32(a["emb"]).std()
    assert 0.018 < std < 0.022
    assert (a["final_norm"] == 1).all()


def test_zipf_tokens_are_skewed_and_in_range():
    t = di.zipf_tokens(4096, 20000, seed=0)
    assert t.min() >= 0 and t.max() < 4096 and t.dtype == np.int32
    counts = np.sort(np.bincount(t, minlength=4096))[::-1]
    assert counts[0] > 20 * max(1, counts[2000])
    assert np.array_equal(t, di.zipf_tokens(4096, 20000, seed=0))


def test_trigram_rows_are_probabilities():
    tri = di.SyntheticTrigram(4096, seed=0)
    for ctx in [(1, 2), (7, 7), (4000, 3)]:
        toks, p = tri.successors(*ctx)
        assert 2 <= len(toks) <= 8 and len(set(toks.tolist())) == len(toks)
        assert abs(p.sum() - 1) < 1e-12 and (np.diff(p) <= 1e-15).all()
        toks2, p2 = tri.successors(*ctx)
        assert np.array_equal(toks, toks2) and np.array_equal(p, p2)


def _check_tree(parent, n, depth):
    assert len(parent) == n and parent[0] == -1
    assert all(0 <= parent[i] < i for i in range(1, n))
    assert di.tree_depths(parent).max() == depth


def test_workload_trees_have_the_stated_shape():
    for name in ("c1", "c3"):
        wl = di.WORKLOADS[name]
        prefix, parent, token = di.workload_tree(wl, seed=0)
        assert len(prefix) == wl.prefix_len and len(token) == wl.n_nodes
        _check_tree(parent, wl.n_nodes, wl.depth)
        assert token.min() >= 0 and token.max() < wl.model.vocab
        # a trie: siblings carry distinct tokens
        for v in range(wl.n_nodes):
            kids = token[np.flatnonzero(parent == v)]
            assert len(set(kids.tolist())) == len(kids)
    wl = di.WORKLOADS["c2"]
    _check_tree(di.random_tree(wl.n_nodes, wl.depth, seed=0), 64, 8)


def test_all_trees_count():
    assert [len(di.all_trees(n)) for n in (1, 2, 3, 4)] == [1, 1, 2, 6]
