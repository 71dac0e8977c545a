"""The CPU draft maker: tri-gram LLM representative, its self-improvement update and the tree search
that proposes candidate continuations (test infrastructure, not product code).

Sec. 2.2, Eq. (1): P(w_i | w_{i-2}, w_{i-1}) = C(w_{i-2}, w_{i-1}, w_i) / C(w_{i-2}, w_{i-1}) counted over a
corpus.  Sec. 2.3, Eq. (2), (3) (= Appendix E, Eq. (E.6), (E.7)): the draft search score.  Appendix G, Alg. 1: the
tree search; Alg. 2: Adjust3Gram.  Appendix F.1: t = 12, 150 iterations, C1 = 32, C2 = 8, l = 4, n = 24.

Readings (the paper is silent or its listing is garbled; each is stated where it is used):
  T1  C(w_{i-2}, w_{i-1}) counts the bi-gram as the start of a tri-gram (so the probabilities of a context sum to
      one before elimination); a document's last bi-gram, which no token follows, is not counted.
  T2  The threshold t eliminates tri-grams whose count is below t; the survivors keep their Eq. (1) value (no
      re-normalisation).  A context whose tri-grams are all eliminated disappears.
  T3  The successors of a context are kept in order of first appearance (corpus order, then Adjust3Gram insertions).
  M1  A search node stands for a word reached after a given previous word, i.e. for a bigram context; the root is
      the last two tokens of the input.  The words that may follow a node and have no child yet (`pending`) are
      the successors of its context in the tri-gram matrix.
  M2  Selection walks down while the node has no pending words, has children and the sentence is not full (the text
      of Appendix G; the listing's condition has a stray negation).  The step down takes the child of highest score
      Eq. (2) with Q(s,a) = child.score / child.visits (0 for an unvisited child), P(s,a) = the child's tri-gram
      probability, N(s,a) = child.visits and the sum over the node's children; the first child wins a tie.
  M3  Expansion creates a child for every pending word at once (as listed), empties the pending list, and
      continues with the child created last.
  M4  sentence_length = l + 1: the root pair plus l words.
  M5  Simulation draws the next word of the pair last reached by inverse CDF over that pair's successors in their
      stored order, weights = their probabilities divided by their sum (after elimination or Adjust3Gram they need
      not sum to one), with the uniform number u[iteration * l + (number of words already in the sentence)] that
      the caller supplies: the first j with  cumulative_j > u * sum  (the last one if rounding leaves none).
  M6  The score of an iteration is 1 + the sum of the tri-gram probabilities of all transitions of the sentence
      (tree part and simulated part alike); it is added to every node from the deepest tree node up to the root.
  M7  Sentences are the root-to-leaf paths of the search tree (leaf = node without children), a sentence's score is
      its leaf's accumulated score; they are sorted by descending score, depth-first order (children in creation
      order) among equals; the first n are returned, the root pair left out.
  A1  Adjust3Gram: every tri-gram that lies inside the window is updated, i.e. the third-word index runs over
      2 .. len(window) - 1 (0-based; the listing's upper limit is the length).
      A new tri-gram is appended to its context's successors (a new context is created if needed).
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

Pair = Tuple[int, int]


class TriGramMatrix:
    """matrix[(w_{i-2}, w_{i-1})] = {w_i: probability}, insertion-ordered (T3)."""

    def __init__(self) -> None:
        self.c3: Dict[Pair, Dict[int, int]] = {}   # C(w_{i-2}, w_{i-1}, w_i)
        self.c2: Dict[Pair, int] = {}              # C(w_{i-2}, w_{i-1})
        self.matrix: Dict[Pair, Dict[int, float]] = {}

    def count(self, tokens: Sequence[int], times: int = 1) -> None:
        """Adds one document's tri-grams to the counts (T1), as if the document occurred `times` times."""
        if times <= 0:
            return
        for i in range(2, len(tokens)):
            ctx = (int(tokens[i - 2]), int(tokens[i - 1]))
            row = self.c3.setdefault(ctx, {})
            row[int(tokens[i])] = row.get(int(tokens[i]), 0) + times
            self.c2[ctx] = self.c2.get(ctx, 0) + times

    def finalize(self, t: int = 12) -> None:
        """Eq. (1) for every counted tri-gram, then the elimination threshold (T2)."""
        self.matrix = {}
        for ctx, row in self.c3.items():
            kept = {w: c / self.c2[ctx] for w, c in row.items() if c >= t}
            if kept:
                self.matrix[ctx] = kept

    def successors(self, ctx: Pair) -> List[Tuple[int, float]]:
        return list(self.matrix.get((int(ctx[0]), int(ctx[1])), {}).items())

    def prob(self, ctx: Pair, w: int) -> float:
        return self.matrix.get((int(ctx[0]), int(ctx[1])), {}).get(int(w), 0.0)

    def adjust_3gram(self, tokens: Sequence[int], max_length: int, increment: float, max_prob: float) -> None:
        """Alg. 2 (A1): reinforce every tri-gram inside the last `max_length` tokens."""
        window = [int(x) for x in tokens[max(0, len(tokens) - max_length):]]
        for a, b, w in zip(window, window[1:], window[2:]):
            row = self.matrix.setdefault((a, b), {})
            row[w] = min(row[w] + increment, max_prob) if w in row else increment


def exploration_factor(sum_n: float, c1: float, c2: float) -> float:
    """Eq. (3): E = C1 + log((sum_b N(s,b) + C2 + 1) / C2)."""
    return c1 + math.log((sum_n + c2 + 1.0) / c2)


def puct(q: float, p: float, n_sa: float, sum_n: float, c1: float, c2: float) -> float:
    """Eq. (2): Q(s,a) + E * P(s,a) * sqrt(sum_b N(s,b)) / (1 + N(s,a))."""
    return q + exploration_factor(sum_n, c1, c2) * p * math.sqrt(sum_n) / (1.0 + n_sa)


class SearchNode:
    """One word of a candidate sentence, reached after `context[0]` (M1)."""

    def __init__(self, context: Pair, prior: float, pending: List[Tuple[int, float]],
                 parent: Optional["SearchNode"]) -> None:
        self.context = context    # (previous word, this node's word)
        self.prior = prior        # P(s,a) of the step that leads here
        self.pending = pending    # successors of `context` that have no child yet: [(word, probability)]
        self.children: List[SearchNode] = []
        self.parent = parent
        self.visits = 0
        self.score = 0.0

    @property
    def token(self) -> int:
        return self.context[1]


def _best_child(node: SearchNode, c1: float, c2: float) -> SearchNode:
    """The child of highest Eq. (2) score; the first one among equals (M2)."""
    sum_n = float(sum(ch.visits for ch in node.children))
    values = [puct(ch.score / ch.visits if ch.visits > 0 else 0.0, ch.prior, float(ch.visits), sum_n, c1, c2)
              for ch in node.children]
    return node.children[values.index(max(values))]


def _descend(root: SearchNode, sentence: List[int], full: int, c1: float, c2: float) -> SearchNode:
    """Selection (M2): follow best children while everything below the node is already expanded; the words passed
    are appended to `sentence` (a token list that starts with the root's two tokens)."""
    node = root
    while not node.pending and node.children and len(sentence) < full:
        node = _best_child(node, c1, c2)
        sentence.append(node.token)
    return node


def _expand(matrix: TriGramMatrix, node: SearchNode) -> SearchNode:
    """Expansion (M3): one child per pending word, in stored order; the search goes on with the last one."""
    for word, prior in node.pending:
        ctx = (node.token, word)
        node.children.append(SearchNode(ctx, prior, matrix.successors(ctx), node))
    node.pending = []
    return node.children[-1]


def _rollout(matrix: TriGramMatrix, sentence: List[int], full: int, uniform: Sequence[float], base: int) -> None:
    """Simulation (M5): extend `sentence` to `full` tokens by inverse-CDF draws; the draw that adds the j-th word
    after the root pair (j counted from 0) uses uniform[base + j]."""
    while len(sentence) < full:
        options = matrix.successors((sentence[-2], sentence[-1]))
        if not options:
            return
        total = 0.0
        for _, p in options:
            total += p
        target = float(uniform[base + len(sentence) - 2]) * total
        running, pick = 0.0, options[-1][0]
        for w, p in options:
            running += p
            if running > target:
                pick = w
                break
        sentence.append(pick)


def _sentence_score(matrix: TriGramMatrix, sentence: Sequence[int]) -> float:
    """1 + the tri-gram probabilities of all transitions, added left to right (M6)."""
    score = 1.0
    for a, b, w in zip(sentence, sentence[1:], sentence[2:]):
        score = score + matrix.prob((a, b), w)
    return score


def _backup(node: Optional[SearchNode], score: float) -> None:
    while node is not None:
        node.visits += 1
        node.score += score
        node = node.parent


def _ranked_leaf_paths(root: SearchNode, n: int) -> List[Tuple[float, List[int]]]:
    """Root-to-leaf word lists with the leaf's accumulated score, best first, depth-first order among equals (M7)."""
    found: List[Tuple[float, List[int]]] = []
    stack: List[Tuple[SearchNode, List[int]]] = [(root, [])]
    while stack:
        node, words = stack.pop()
        if not node.children:
            if words:
                found.append((node.score, words))
            continue
        for ch in reversed(node.children):  # popped in creation order
            stack.append((ch, words + [ch.token]))
    found.sort(key=lambda item: -item[0])  # stable
    return found[:n]


def run_mcts(matrix: TriGramMatrix, w0: int, w1: int, uniform: Sequence[float], iterations: int = 150, l: int = 4,
             n: int = 24, c1: float = 32.0, c2: float = 8.0, return_root: bool = False):
    """Alg. 1.  Returns [(score, [words])] best first (M7); with return_root also the search tree's root."""
    full = l + 2  # the root's two tokens plus l words (M4)
    assert len(uniform) >= iterations * l
    root = SearchNode((int(w0), int(w1)), 1.0, matrix.successors((w0, w1)), None)
    for it in range(iterations):
        sentence = [int(w0), int(w1)]
        node = _descend(root, sentence, full, c1, c2)
        if node.pending and len(sentence) < full:
            node = _expand(matrix, node)
            sentence.append(node.token)
        _rollout(matrix, sentence, full, uniform, it * l)
        _backup(node, _sentence_score(matrix, sentence))
    ranked = _ranked_leaf_paths(root, n)
    return (ranked, root) if return_root else ranked
