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
  M1  A tree node's `word` is the pair (previous word, word); the root holds the last two tokens of the input.  The
      words a node may be followed by ("untried words") are the successors of its pair in the tri-gram matrix.
  M2  Selection walks down while the node has no untried words, has children and the sentence is not full (the text
      of Appendix G; the listing's condition has a stray negation).  select_child takes the child of highest score
      Eq. (2) with Q(s,a) = child.score / child.visits (0 for an unvisited child), P(s,a) = the child's tri-gram
      probability, N(s,a) = child.visits and the sum over the node's children; the first child wins a tie.
  M3  Expansion creates a child for every untried word at once (as listed), empties the untried list, and
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
  A1  Adjust3Gram: i runs over 2 .. len(subTokens) - 1 (0-based indices; the listing's upper limit is the length).
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
        """Alg. 2 (A1)."""
        n = len(tokens)
        start_index = max(0, n - max_length)
        sub_tokens = [int(x) for x in tokens[start_index:n]]
        for i in range(2, len(sub_tokens)):
            ctx, w = (sub_tokens[i - 2], sub_tokens[i - 1]), sub_tokens[i]
            row = self.matrix.setdefault(ctx, {})
            if w in row:
                row[w] = min(row[w] + increment, max_prob)
            else:
                row[w] = increment


def exploration_factor(sum_n: float, c1: float, c2: float) -> float:
    """Eq. (3): E = C1 + log((sum_b N(s,b) + C2 + 1) / C2)."""
    return c1 + math.log((sum_n + c2 + 1.0) / c2)


def puct(q: float, p: float, n_sa: float, sum_n: float, c1: float, c2: float) -> float:
    """Eq. (2): Q(s,a) + E * P(s,a) * sqrt(sum_b N(s,b)) / (1 + N(s,a))."""
    return q + exploration_factor(sum_n, c1, c2) * p * math.sqrt(sum_n) / (1.0 + n_sa)


class Node:
    def __init__(self, p_word: int, word: int, prior: float, untried_words: List[Tuple[int, float]],
                 parent: Optional["Node"]) -> None:
        self.word: Pair = (p_word, word)
        self.prior = prior                  # P(s,a) of the action that leads here
        self.untried_words = untried_words  # [(word, probability)]
        self.children: List[Node] = []
        self.parent = parent
        self.visits = 0
        self.score = 0.0

    def select_child(self, c1: float, c2: float) -> "Node":
        sum_n = float(sum(ch.visits for ch in self.children))
        best, best_val = None, None
        for ch in self.children:
            q = ch.score / ch.visits if ch.visits > 0 else 0.0
            val = puct(q, ch.prior, float(ch.visits), sum_n, c1, c2)
            if best is None or val > best_val:
                best, best_val = ch, val
        return best


def run_mcts(matrix: TriGramMatrix, w0: int, w1: int, uniform: Sequence[float], iterations: int = 150, l: int = 4,
             n: int = 24, c1: float = 32.0, c2: float = 8.0, return_root: bool = False):
    """Alg. 1.  Returns [(score, [words])] best first (M7); with return_root also the search tree's root."""
    sentence_length = l + 1  # M4
    assert len(uniform) >= iterations * l
    root = Node(int(w0), int(w1), 1.0, matrix.successors((w0, w1)), None)
    for it in range(iterations):
        node = root
        state = [node.word]
        end = False
        # Selection (M2)
        while not node.untried_words and node.children and not end:
            selected_child = node.select_child(c1, c2)
            state.append(selected_child.word)
            node = selected_child
            if len(state) == sentence_length:
                end = True
        # Expansion (M3)
        if node.untried_words and not end:
            untried_words = node.untried_words
            p_word = node.word[1]
            for word, prior in untried_words:
                tmp_untried_words = matrix.successors((p_word, word))
                node.children.append(Node(p_word, word, prior, tmp_untried_words, node))
            node.untried_words = []
            node = node.children[-1]
            state.append(node.word)
        # Simulation (M5)
        while len(state) < sentence_length:
            last_word = state[-1]
            next_words = matrix.successors(last_word)
            if not next_words:
                break
            total = 0.0
            for _, p in next_words:
                total += p
            target = float(uniform[it * l + (len(state) - 1)]) * total
            cumulative, pick = 0.0, next_words[-1][0]
            for w, p in next_words:
                cumulative += p
                if cumulative > target:
                    pick = w
                    break
            state.append((last_word[1], pick))
        # Backpropagation (M6)
        score = 1.0
        for i in range(1, len(state)):
            score = score + matrix.prob(state[i - 1], state[i][1])
        current_node = node
        while current_node is not None:
            current_node.visits += 1
            current_node.score += score
            current_node = current_node.parent
    # Extract and sort (M7)
    sentences: List[Tuple[float, List[int]]] = []

    def walk(nd: Node, words: List[int]) -> None:
        if not nd.children:
            if words:
                sentences.append((nd.score, list(words)))
            return
        for ch in nd.children:
            words.append(ch.word[1])
            walk(ch, words)
            words.pop()

    walk(root, [])
    sentences.sort(key=lambda s: -s[0])  # stable: depth-first order among equal scores
    sentences = sentences[:n]
    return (sentences, root) if return_root else sentences
