"""Pseudo-sequence construction (test infrastructure, not product code).

Sec. 2.4 (Draft Construction and Verification): the draft maker returns several candidate
continuations that often start alike; they are merged into one pseudo-sequence in which every
candidate is a sub-sequence and every common prefix appears only once.  With the last committed token
as the root this is the trie of the candidates: a node per distinct non-empty prefix, its parent the
node of the prefix without its last token.

Readings (the paper fixes neither): nodes are numbered in order of first appearance while the
candidates are inserted in rank order, so a parent always precedes its children and higher-ranked
candidates get the lower indices; when a node budget is given, a candidate is cut where the budget
runs out and later candidates still re-use what exists.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple


def build_trie(root_token: int, candidates: Sequence[Sequence[int]],
               max_nodes: Optional[int] = None) -> Tuple[List[int], List[int], List[int]]:
    """Returns (parent, token, end): node 0 is the root (parent -1, token root_token); end[c] is the
    node at which candidate c stops (its last token's node, or the node where the budget cut it)."""
    parent, token = [-1], [int(root_token)]
    end = []
    for cand in candidates:
        v = 0
        for t in cand:
            t = int(t)
            kids = [i for i in range(len(parent)) if parent[i] == v and token[i] == t]
            if kids:
                v = kids[0]
                continue
            if max_nodes is not None and len(parent) >= max_nodes:
                break
            parent.append(v)
            token.append(t)
            v = len(parent) - 1
        end.append(v)
    return parent, token, end
