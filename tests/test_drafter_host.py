"""The C++ draft maker (host code behind the C ABI) against the oracle, bit for bit: same successors in the same
order, same probabilities, same candidates and scores.  No GPU calls."""
import os

import numpy as np
import pytest

import ded_inputs as di
from oracle import drafter as dr


@pytest.fixture(scope="module")
def b():
    from paper_2407_12021_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2407_12021_amd.build import build_library
        build_library()
    return binding


def _same_matrix(d, m, contexts):
    assert d.size() == sum(len(r) for r in m.matrix.values())
    for ctx in contexts:
        assert d.successors(*ctx) == m.successors(ctx), ctx


def _pair(docs, t, b):
    d, m = b.Drafter(), dr.TriGramMatrix()
    for doc in docs:
        d.count(doc)
        m.count(doc)
    d.finalize(t)
    m.finalize(t)
    return d, m


def test_matrix_hand_corpus(b):
    corpus = [1, 2, 3, 1, 2, 4, 1, 2, 3, 1, 2]
    for t in (0, 1, 2, 3):
        d, m = _pair([corpus], t, b)
        _same_matrix(d, m, [(1, 2), (2, 3), (3, 1), (2, 4), (4, 1), (7, 7)])
        d.close()


def test_document_multiplicity(b):
    docs = [[1, 2, 3, 4, 1, 2, 3], [1, 2, 5], [2, 3, 9]]
    d, m, d1 = b.Drafter(), dr.TriGramMatrix(), b.Drafter()
    for doc, k in zip(docs, (3, 0, 2)):
        d.count(doc, k)
        m.count(doc, k)
        for _ in range(k):
            d1.count(doc)
    for t in (1, 3, 4, 7):
        d.finalize(t), m.finalize(t), d1.finalize(t)
        for ctx in [(1, 2), (2, 3), (3, 4), (4, 1)]:
            assert d.successors(*ctx) == m.successors(ctx) == d1.successors(*ctx)
    d.close(), d1.close()


def test_matrix_counts_threshold_and_adjust_random(b):
    g = np.random.default_rng(11)
    for V, t in ((5, 1), (9, 3), (40, 2)):
        docs = [g.integers(0, V, size=int(n)).tolist() for n in (0, 1, 2, 3, 400, 1200)]
        d, m = _pair(docs, t, b)
        contexts = [(a, c) for a in range(V) for c in range(V)][:400]
        _same_matrix(d, m, contexts)
        for k in range(5):
            out = g.integers(0, V + 2, size=int(g.integers(0, 60))).tolist()
            ml = int(g.integers(0, 70))
            d.adjust(out, ml, 0.2, 0.85)
            m.adjust_3gram(out, ml, 0.2, 0.85)
            _same_matrix(d, m, contexts + [(V, V + 1), (V + 1, V)])
        d.finalize(t)  # rebuilding from the counts forgets the updates
        m.finalize(t)
        _same_matrix(d, m, contexts)
        d.close()


def _zipf_docs(V, n_docs, length, seed):
    tri = di.SyntheticTrigram(V, seed=seed)
    g = np.random.default_rng(seed + 1)
    docs = []
    for _ in range(n_docs):
        a, c = int(g.integers(0, V)), int(g.integers(0, V))
        doc = [a, c]
        for _ in range(length):
            succ, prob = tri.successors(a, c)
            w = int(succ[g.choice(len(succ), p=prob)])
            doc.append(w)
            a, c = c, w
        docs.append(doc)
    return docs


@pytest.mark.parametrize("params", [dict(iterations=1, l=1, n=1), dict(iterations=7, l=2, n=5),
                                    dict(iterations=150, l=4, n=24), dict(iterations=150, l=4, n=24, c1=2.414),
                                    dict(iterations=400, l=6, n=64, c1=0.5, c2=2.0), dict(iterations=0, l=4, n=24)])
def test_mcts_candidates_and_scores_equal_the_oracle(b, params):
    g = np.random.default_rng(3)
    for V, t, adjust in ((6, 1, False), (12, 2, True), (300, 1, True)):
        docs = [g.integers(0, V, size=3000).tolist()] if V < 100 else _zipf_docs(V, 30, 300, seed=V)
        d, m = _pair(docs, t, b)
        if adjust:
            out = docs[0][100:160]
            d.adjust(out, 48, 0.3, 0.9)
            m.adjust_3gram(out, 48, 0.3, 0.9)
        roots = [tuple(doc[5:7]) for doc in docs[:3]] + [(docs[0][50], docs[0][51]), (V + 5, V + 6)]
        for w0, w1 in roots:
            u = g.random(params["iterations"] * params["l"])
            got = d.mcts(w0, w1, u, **params)
            ref = dr.run_mcts(m, w0, w1, u, **params)
            assert [w for _, w in got] == [w for _, w in ref], (V, w0, w1)
            assert [s for s, _ in got] == [s for s, _ in ref]  # same operations in the same order: bit equal
        d.close()


def test_mcts_argument_errors(b):
    d = b.Drafter()
    d.count([1, 2, 3, 4])
    d.finalize(1)
    with pytest.raises(b.DedError):
        d.mcts(1, 2, [0.5] * 3, iterations=1, l=4)          # too few uniform numbers
    with pytest.raises(b.DedError):
        d.mcts(1, 2, [0.5] * 8, iterations=2, l=4, c2=0.0)  # log of a ratio with C2 = 0
    with pytest.raises(b.DedError):
        d.mcts(1, 2, [0.5] * 8, iterations=2, l=0)
    # iteration 0 creates word 3 and simulates 4, iteration 1 creates the leaf 4: one pass of score 1 + 1 + 1
    assert d.mcts(1, 2, [0.5] * 8, iterations=2, l=4) == [(3.0, [3, 4])]
    assert b.lib().ded_trigram_count(None, None, 0, 1) == b.DED_EINVAL
    assert b.lib().ded_trigram_size(None) < 0
    b.lib().ded_trigram_free(None)
    d.close()


def test_paper_shape_candidates_feed_the_tree_builder(b):
    """150 iterations, l = 4, n = 24 on a Zipf tri-gram corpus: candidates -> pseudo-sequence within the 64-node budget."""
    docs = _zipf_docs(2000, 40, 500, seed=9)
    d, m = _pair(docs, 1, b)
    g = np.random.default_rng(0)
    w0, w1 = docs[0][10], docs[0][11]
    cands = d.mcts(w0, w1, g.random(600))
    assert 1 <= len(cands) <= 24 and all(1 <= len(w) <= 4 for _, w in cands)
    rc, parent, token, end = b.ded_build_tree(w1, [w for _, w in cands], 64)
    assert rc == b.DED_OK and 2 <= len(parent) <= 64
    import oracle
    p2, t2, e2 = oracle.build_trie(w1, [w for _, w in cands], 64)
    assert parent.tolist() == p2 and token.tolist() == t2 and end.tolist() == e2
    d.close()
