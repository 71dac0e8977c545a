/* The host-only part of the C ABI used from plain C: tri-gram matrix -> tree search -> pseudo-sequence -> validation.
 * Prints one line per check; exit status 0 when all hold. */
#include <stdio.h>
#include <stdlib.h>

#include "ded_verify.h"

#define CHECK(cond)                                      \
  do {                                                   \
    if (!(cond)) {                                       \
      printf("FAILED line %d: %s\n", __LINE__, #cond);   \
      return 1;                                          \
    }                                                    \
  } while (0)

int main(void) {
  /* corpus 1 2 3 1 2 4 1 2 3 1 2: P(3 | 1 2) = 2/3, P(4 | 1 2) = 1/3 (Eq. (1)) */
  const int32_t corpus[] = {1, 2, 3, 1, 2, 4, 1, 2, 3, 1, 2};
  ded_trigram *m = ded_trigram_create();
  CHECK(m != NULL);
  CHECK(ded_trigram_count(m, corpus, 11, 1) == DED_OK);
  CHECK(ded_trigram_finalize(m, 1) == DED_OK);
  int32_t words[4], n = 0;
  double probs[4];
  CHECK(ded_trigram_lookup(m, 1, 2, 4, words, probs, &n) == DED_OK);
  CHECK(n == 2 && words[0] == 3 && words[1] == 4);
  CHECK(probs[0] == 2.0 / 3.0 && probs[1] == 1.0 / 3.0);
  CHECK(ded_trigram_size(m) == 6);

  /* draft search from the context (1, 2): 20 iterations, l = 3 words, up to 4 candidates */
  enum { ITER = 20, L = 3, NC = 4 };
  double u[ITER * L];
  for (int i = 0; i < ITER * L; ++i) u[i] = (i * 37 % 100) / 100.0;
  int32_t cand[NC * L], len[NC], n_cand = 0;
  double score[NC];
  CHECK(ded_draft_mcts(m, 1, 2, ITER, L, NC, 32.0, 8.0, u, ITER * L, cand, len, score, &n_cand) == DED_OK);
  CHECK(n_cand >= 2 && n_cand <= NC);
  for (int c = 0; c < n_cand; ++c) {
    CHECK(len[c] >= 1 && len[c] <= L);
    CHECK(c == 0 || score[c] <= score[c - 1]);
    CHECK(cand[c * L] == 3 || cand[c * L] == 4); /* a successor of (1, 2) */
  }
  printf("draft search: %d candidates, best score %.3f\n", n_cand, score[0]);

  /* candidates -> pseudo-sequence under the root token 2 */
  int32_t parent[16], token[16], end[NC], n_nodes = 0;
  CHECK(ded_build_tree(2, n_cand, len, cand, L, 16, parent, token, end, &n_nodes) == DED_OK);
  CHECK(n_nodes >= 2 && parent[0] == -1 && token[0] == 2);
  for (int i = 1; i < n_nodes; ++i) CHECK(parent[i] >= 0 && parent[i] < i);
  printf("pseudo-sequence: %d nodes\n", n_nodes);

  /* the tree passes the step validation of a small configuration */
  ded_config cfg;
  cfg.n_layers = 2, cfg.d_model = 256, cfg.n_heads = 4, cfg.n_kv_heads = 4, cfg.head_dim = 64, cfg.d_ffn = 688;
  cfg.vocab = 4096, cfg.rope_base = 10000.0f, cfg.rms_eps = 1e-5f, cfg.dtype = DED_F32;
  cfg.max_batch = 1, cfg.kv_capacity = 64, cfg.max_nodes = 16;
  int32_t prefix_len = 10;
  CHECK(ded_workspace_bytes(&cfg) > 0);
  CHECK(ded_validate_tree(&cfg, 1, &prefix_len, &n_nodes, parent, token) == DED_OK);
  token[1] = 4096; /* outside the vocabulary */
  CHECK(ded_validate_tree(&cfg, 1, &prefix_len, &n_nodes, parent, token) == DED_ETOKEN);

  /* Adjust3Gram: a new tri-gram enters with the increment, an old one is capped */
  const int32_t out[] = {1, 2, 3, 9};
  CHECK(ded_trigram_adjust(m, out, 4, 8, 0.5, 0.9) == DED_OK);
  CHECK(ded_trigram_lookup(m, 1, 2, 4, words, probs, &n) == DED_OK && probs[0] == 0.9);
  CHECK(ded_trigram_lookup(m, 2, 3, 4, words, probs, &n) == DED_OK && n == 2 && words[1] == 9 && probs[1] == 0.5);
  ded_trigram_free(m);
  printf("ok\n");
  return 0;
}
