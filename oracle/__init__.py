"""CPU oracle for draft-tree verification.  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 numpy.  It defines what the GPU library must compute and shares no code with it.
Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this package; the
product path never does.

Pinned parts (see tests/test_oracle_pins.py): every function below is pinned by closed forms,
library special cases, brute force on tiny trees or the chain == autoregressive invariant; the
pseudo-sequence builder by the set of root-to-node paths, hand-worked cases and the equality of a
candidate's logits in the merged tree and in its own chain; the temperature / top-p sampler by brute
force over subsets on tiny vocabularies, its limits (argmax, plain soft-max frequencies) and monotonicity;
the draft maker (tri-gram matrix, Adjust3Gram, search score, tree search) by a hand-worked corpus, hand-evaluated
score values, a hand-traced first and second iteration, the closed form on a deterministic chain and the
conservation of visits and scores over the search tree.
Parity unpinned: none.
"""
from .decoder import (  # noqa: F401
    widen, rmsnorm, rope, silu, masked_attention, ancestor_mask, node_depths,
    forward_rows, prefill, verify_tree, autoregressive_logits, autoregressive_decode,
)
from .accept import argmax_margin, accept_walk, compact_rows  # noqa: F401
from .trie import build_trie  # noqa: F401
from .sample import nucleus, sample_top_p, sample_rows  # noqa: F401
from .drafter import TriGramMatrix, exploration_factor, puct, run_mcts  # noqa: F401
