// Host-side draft maker: the tri-gram LLM representative (Sec. 2.2, Eq. (1)), its self-improvement update
// (Appendix G, Alg. 2) and the tree search that proposes candidate continuations (Sec. 2.3, Eq. (2), (3);
// Appendix G, Alg. 1).  No device work: the paper runs this part on the CPU next to the verification step.
//
// Layout: a context (w_{i-2}, w_{i-1}) maps to a row; a row is a vector of (word, probability) in order of
// first appearance.  The search tree lives in one arena per call; the children of a node are created together
// and therefore sit in one contiguous index range.  All arithmetic is double precision, evaluated in the order
// the equations are written (no contraction), so that decisions taken on scores are reproducible.
#include <math.h>
#include <stdint.h>

#include <algorithm>
#include <new>
#include <unordered_map>
#include <vector>

#include "../../include/ded_verify.h"

#pragma STDC FP_CONTRACT OFF

namespace {

struct Successor {
  int32_t word;
  double prob;
};

struct CountRow {
  std::vector<int32_t> word;   // in order of first appearance
  std::vector<int64_t> count;  // C(w_{i-2}, w_{i-1}, w_i)
  int64_t total = 0;           // C(w_{i-2}, w_{i-1}): tri-grams that start with the pair
};

inline uint64_t pair_key(int32_t a, int32_t b) { return ((uint64_t)(uint32_t)a << 32) | (uint32_t)b; }

struct SearchNode {
  int32_t parent;
  int32_t p_word, word;
  int32_t first_child, n_children;  // valid once expanded
  int32_t row;                      // row of the pair (p_word, word) in the matrix, -1 if it has no successors
  bool expanded;
  double prior;
  int64_t visits;
  double score;
};

}  // namespace

struct ded_trigram {
  std::unordered_map<uint64_t, int32_t> count_index, index;  // pair -> row
  std::unordered_map<uint64_t, int32_t> count_pos;           // (count row, word) -> position in that row
  std::vector<uint64_t> count_key;                             // rows in order of first appearance
  std::vector<CountRow> counts;
  std::vector<std::vector<Successor>> rows;

  const std::vector<Successor>* find(int32_t a, int32_t b, int32_t* row_out = nullptr) const {
    auto it = index.find(pair_key(a, b));
    if (it == index.end()) return nullptr;
    if (row_out) *row_out = it->second;
    return &rows[(size_t)it->second];
  }
};

extern "C" ded_trigram* ded_trigram_create(void) { return new (std::nothrow) ded_trigram(); }

extern "C" void ded_trigram_free(ded_trigram* m) { delete m; }

extern "C" int ded_trigram_count(ded_trigram* m, const int32_t* tokens, int64_t n, int64_t times) {
  if (!m || n < 0 || (n > 0 && !tokens) || times < 0) return DED_EINVAL;
  if (times == 0) return DED_OK;
  try {
    for (int64_t i = 2; i < n; ++i) {
      const uint64_t key = pair_key(tokens[i - 2], tokens[i - 1]);
      auto it = m->count_index.find(key);
      if (it == m->count_index.end()) {
        it = m->count_index.emplace(key, (int32_t)m->counts.size()).first;
        m->counts.emplace_back();
        m->count_key.push_back(key);
      }
      CountRow& r = m->counts[(size_t)it->second];
      // frequent contexts of a real corpus have thousands of successors: look the word up, do not scan the row
      auto pos = m->count_pos.find(pair_key(it->second, tokens[i]));
      if (pos == m->count_pos.end()) {
        pos = m->count_pos.emplace(pair_key(it->second, tokens[i]), (int32_t)r.word.size()).first;
        r.word.push_back(tokens[i]);
        r.count.push_back(0);
      }
      r.count[(size_t)pos->second] += times;
      r.total += times;
    }
  } catch (const std::bad_alloc&) {
    return DED_ENOMEM;
  }
  return DED_OK;
}

extern "C" int ded_trigram_finalize(ded_trigram* m, int32_t t) {
  if (!m || t < 0) return DED_EINVAL;
  try {
    m->index.clear();
    m->rows.clear();
    for (size_t r = 0; r < m->counts.size(); ++r) {
      const CountRow& cr = m->counts[r];
      std::vector<Successor> row;
      for (size_t j = 0; j < cr.word.size(); ++j)
        if (cr.count[j] >= t) row.push_back({cr.word[j], (double)cr.count[j] / (double)cr.total});
      if (row.empty()) continue;
      m->index.emplace(m->count_key[r], (int32_t)m->rows.size());
      m->rows.push_back(std::move(row));
    }
  } catch (const std::bad_alloc&) {
    return DED_ENOMEM;
  }
  return DED_OK;
}

extern "C" int ded_trigram_adjust(ded_trigram* m, const int32_t* tokens, int64_t n, int64_t max_length,
                                  double increment, double max_prob) {
  if (!m || n < 0 || (n > 0 && !tokens) || max_length < 0) return DED_EINVAL;
  if (!(increment >= 0.0) || !(max_prob >= 0.0)) return DED_EINVAL;
  const int64_t start = std::max<int64_t>(0, n - max_length);
  try {
    for (int64_t i = start + 2; i < n; ++i) {
      const uint64_t key = pair_key(tokens[i - 2], tokens[i - 1]);
      auto it = m->index.find(key);
      if (it == m->index.end()) {
        it = m->index.emplace(key, (int32_t)m->rows.size()).first;
        m->rows.emplace_back();
      }
      std::vector<Successor>& row = m->rows[(size_t)it->second];
      size_t j = 0;
      while (j < row.size() && row[j].word != tokens[i]) ++j;
      if (j == row.size())
        row.push_back({tokens[i], increment});
      else
        row[j].prob = std::min(row[j].prob + increment, max_prob);
    }
  } catch (const std::bad_alloc&) {
    return DED_ENOMEM;
  }
  return DED_OK;
}

extern "C" int ded_trigram_lookup(const ded_trigram* m, int32_t w0, int32_t w1, int32_t cap, int32_t* words,
                                  double* probs, int32_t* n_out) {
  if (!m || !n_out || cap < 0 || (cap > 0 && (!words || !probs))) return DED_EINVAL;
  const std::vector<Successor>* row = m->find(w0, w1);
  const int32_t n = row ? (int32_t)row->size() : 0;
  *n_out = n;
  for (int32_t j = 0; j < std::min(n, cap); ++j) {
    words[j] = (*row)[(size_t)j].word;
    probs[j] = (*row)[(size_t)j].prob;
  }
  return DED_OK;
}

extern "C" int64_t ded_trigram_size(const ded_trigram* m) {
  if (!m) return DED_EINVAL;
  int64_t n = 0;
  for (const auto& r : m->rows) n += (int64_t)r.size();
  return n;
}

extern "C" int ded_draft_mcts(const ded_trigram* m, int32_t w0, int32_t w1, int32_t iterations, int32_t l, int32_t n,
                              double c1, double c2, const double* uniform, int64_t n_uniform, int32_t* cand_tokens,
                              int32_t* cand_len, double* cand_score, int32_t* n_cand) {
  if (!m || !n_cand || iterations < 0 || l < 1 || n < 0 || !(c2 > 0.0)) return DED_EINVAL;
  if (n > 0 && (!cand_tokens || !cand_len)) return DED_EINVAL;
  if ((int64_t)iterations * l > n_uniform || (iterations > 0 && !uniform)) return DED_EINVAL;
  const int sentence_length = l + 1;  // the root pair plus l words
  try {
    std::vector<SearchNode> tree;
    tree.reserve(1024);
    auto make_node = [&](int32_t parent, int32_t p_word, int32_t word, double prior) {
      SearchNode nd;
      nd.parent = parent, nd.p_word = p_word, nd.word = word;
      nd.first_child = 0, nd.n_children = 0, nd.row = -1;
      nd.expanded = false, nd.prior = prior, nd.visits = 0, nd.score = 0.0;
      m->find(p_word, word, &nd.row);
      tree.push_back(nd);
    };
    auto untried = [&](const SearchNode& nd) { return !nd.expanded && nd.row >= 0; };
    make_node(-1, w0, w1, 1.0);
    std::vector<int32_t> state_word;  // second word of every pair of the sentence
    std::vector<double> state_prob;   // tri-gram probability of the transition into that pair
    for (int32_t it = 0; it < iterations; ++it) {
      int32_t node = 0;
      state_word.assign(1, w1);
      state_prob.assign(1, 0.0);
      int32_t state_prev = w0;  // first word of the sentence's last pair
      bool end = false;
      // Selection: down the tree by Eq. (2) while the node is fully expanded, has children and the sentence is short
      while (!untried(tree[(size_t)node]) && tree[(size_t)node].n_children > 0 && !end) {
        const SearchNode& nd = tree[(size_t)node];
        int64_t visits = 0;
        for (int32_t c = 0; c < nd.n_children; ++c) visits += tree[(size_t)(nd.first_child + c)].visits;
        const double sum_n = (double)visits;
        const double e = c1 + log((sum_n + c2 + 1.0) / c2);  // Eq. (3)
        const double root_n = sqrt(sum_n);
        int32_t best = nd.first_child;
        double best_val = 0.0;
        for (int32_t c = 0; c < nd.n_children; ++c) {
          const SearchNode& ch = tree[(size_t)(nd.first_child + c)];
          const double q = ch.visits > 0 ? ch.score / (double)ch.visits : 0.0;
          const double val = q + e * ch.prior * root_n / (1.0 + (double)ch.visits);  // Eq. (2)
          if (c == 0 || val > best_val) best = nd.first_child + c, best_val = val;
        }
        state_prev = state_word.back();
        state_word.push_back(tree[(size_t)best].word);
        state_prob.push_back(tree[(size_t)best].prior);
        node = best;
        if ((int)state_word.size() == sentence_length) end = true;
      }
      // Expansion: a child for every successor at once; go on with the child created last
      if (untried(tree[(size_t)node]) && !end) {
        const std::vector<Successor>& row = m->rows[(size_t)tree[(size_t)node].row];
        const int32_t first = (int32_t)tree.size(), p_word = tree[(size_t)node].word;
        for (const Successor& s : row) make_node(node, p_word, s.word, s.prob);
        tree[(size_t)node].first_child = first;
        tree[(size_t)node].n_children = (int32_t)row.size();
        tree[(size_t)node].expanded = true;
        node = first + (int32_t)row.size() - 1;
        state_prev = state_word.back();
        state_word.push_back(tree[(size_t)node].word);
        state_prob.push_back(tree[(size_t)node].prior);
      }
      // Simulation: inverse CDF over the successors of the last pair with the caller's uniform numbers
      while ((int)state_word.size() < sentence_length) {
        const std::vector<Successor>* row = m->find(state_prev, state_word.back());
        if (!row || row->empty()) break;
        double total = 0.0;
        for (const Successor& s : *row) total += s.prob;
        const double target = uniform[(int64_t)it * l + ((int64_t)state_word.size() - 1)] * total;
        double cumulative = 0.0;
        const Successor* pick = &row->back();
        for (const Successor& s : *row) {
          cumulative += s.prob;
          if (cumulative > target) {
            pick = &s;
            break;
          }
        }
        state_prev = state_word.back();
        state_word.push_back(pick->word);
        state_prob.push_back(pick->prob);
      }
      // Backpropagation: 1 + the tri-gram probabilities of all transitions, added along the tree path
      double score = 1.0;
      for (size_t i = 1; i < state_word.size(); ++i) score = score + state_prob[i];
      for (int32_t cur = node; cur >= 0; cur = tree[(size_t)cur].parent) {
        tree[(size_t)cur].visits += 1;
        tree[(size_t)cur].score += score;
      }
    }
    // Sentences = root-to-leaf paths in depth-first order (children in creation order), ranked by the leaf's
    // accumulated score; equal scores keep depth-first order
    std::vector<int32_t> leaves;
    if (tree[0].n_children > 0) {
      std::vector<int32_t> stack(1, 0);
      while (!stack.empty()) {
        const int32_t v = stack.back();
        stack.pop_back();
        const SearchNode& nd = tree[(size_t)v];
        if (nd.n_children == 0) {
          leaves.push_back(v);
          continue;
        }
        for (int32_t c = nd.n_children - 1; c >= 0; --c) stack.push_back(nd.first_child + c);
      }
    }
    std::stable_sort(leaves.begin(), leaves.end(),
                     [&](int32_t a, int32_t b) { return tree[(size_t)a].score > tree[(size_t)b].score; });
    const int32_t out = (int32_t)std::min<size_t>(leaves.size(), (size_t)n);
    for (int32_t s = 0; s < out; ++s) {
      int32_t len = 0;
      for (int32_t cur = leaves[(size_t)s]; cur > 0; cur = tree[(size_t)cur].parent) ++len;
      cand_len[s] = len;
      int32_t pos = len;
      for (int32_t cur = leaves[(size_t)s]; cur > 0; cur = tree[(size_t)cur].parent)
        cand_tokens[(int64_t)s * l + --pos] = tree[(size_t)cur].word;
      if (cand_score) cand_score[s] = tree[(size_t)leaves[(size_t)s]].score;
    }
    *n_cand = out;
  } catch (const std::bad_alloc&) {
    return DED_ENOMEM;
  }
  return DED_OK;
}
