// Host-side construction of the pseudo-sequence (draft tree) from ranked candidate continuations
// (Sec. 2.4: every candidate is a sub-sequence, every common prefix appears only once).  No device work.
#include <stdint.h>

#include <unordered_map>

#include "../../include/ded_verify.h"

extern "C" int ded_build_tree(int32_t root_token, int32_t n_cand, const int32_t* cand_len, const int32_t* cand_tokens,
                              int32_t max_len, int32_t max_nodes, int32_t* parent, int32_t* token, int32_t* cand_end,
                              int32_t* n_nodes) {
  if (n_cand < 0 || max_len < 0 || max_nodes < 1 || !parent || !token || !n_nodes) return DED_EINVAL;
  if (n_cand > 0 && (!cand_len || (max_len > 0 && !cand_tokens))) return DED_EINVAL;
  for (int32_t c = 0; c < n_cand; ++c)
    if (cand_len[c] < 0 || cand_len[c] > max_len) return DED_EINVAL;
  // child lookup: (parent node, token) -> node
  std::unordered_map<uint64_t, int32_t> child;
  child.reserve((size_t)max_nodes * 2);
  parent[0] = -1;
  token[0] = root_token;
  int32_t n = 1;
  for (int32_t c = 0; c < n_cand; ++c) {
    const int32_t* seq = cand_tokens + (int64_t)c * max_len;
    int32_t v = 0;
    for (int32_t j = 0; j < cand_len[c]; ++j) {
      const uint64_t key = ((uint64_t)(uint32_t)v << 32) | (uint32_t)seq[j];
      auto it = child.find(key);
      if (it != child.end()) {
        v = it->second;
        continue;
      }
      if (n >= max_nodes) break;  // budget exhausted: this candidate is cut here, later ones still re-use nodes
      parent[n] = v;
      token[n] = seq[j];
      child.emplace(key, n);
      v = n++;
    }
    if (cand_end) cand_end[c] = v;
  }
  *n_nodes = n;
  return DED_OK;
}
