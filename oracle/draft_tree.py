"""CPU oracle for building the draft tree from recorded drafter candidates.
TEST INFRASTRUCTURE ONLY (same rules as verify_oracle.py: tests, smoke check and the
benchmark's CPU-baseline leg may import it; the product never does).

What the paper says (Sec. 4.1): the top-K predictions of the draft model are recorded
and form a tree with several paths, following the dynamic draft tree of Eagle-2; the
experiments use the top 8 tokens, a maximum of 50 nodes and a depth of 4 (Sec. 5.1;
App. A lists depth 5).  The paper gives no more than that.  Reading taken here, the
final selection step of that published strategy, restated:

  * every recorded candidate c has a parent candidate (or the root), a token and the
    log-probability the drafter gave it; its score is the sum of the log-probabilities
    on the path root..c (a joint log-probability), accumulated in float32 from the root
    down, one addition per edge - the precision is part of the definition because the
    score decides an integer (which nodes are kept);
  * the tree keeps the n_keep candidates of highest score, the lower candidate index
    winning ties.  Log-probabilities are <= 0, so a parent never scores below its child
    and, being listed first, wins a tie: the kept set is closed under "parent of";
  * kept nodes are numbered breadth first (by depth, then by candidate index) after the
    root, which is node 0 - the order the verification pass expects (parent[i] < i).

Parity unpinned by the paper (it states the idea in one sentence).  Pinned in
tests/test_oracle_draft_tree.py by what the definition implies: the kept set has the
largest total score among all parent-closed sets of its size (brute force on small
forests), closure, the hand-checkable chain / star cases, and agreement of the emitted
depth / ancestor arrays with verify_oracle.tree_structure.
"""
from __future__ import annotations

from typing import Dict, Sequence

import numpy as np


def candidate_scores(cand_parent: Sequence[int], cand_logp: Sequence[float]) -> np.ndarray:
    """Joint log-probability of every candidate, float32, accumulated root to node.
    cand_parent[c] = index of the parent candidate (< c) or -1 for a child of the root."""
    par = np.asarray(cand_parent, dtype=np.int64)
    lp = np.asarray(cand_logp, dtype=np.float32)
    score = np.zeros(len(par), dtype=np.float32)
    for c in range(len(par)):
        if not (-1 <= par[c] < c):
            raise ValueError("a candidate's parent must be listed before it")
        base = np.float32(0.0) if par[c] < 0 else score[par[c]]
        score[c] = np.float32(base + lp[c])
    return score


def build_draft_tree(cand_parent: Sequence[int], cand_logp: Sequence[float],
                     cand_token: Sequence[int], root_token: int, n_nodes: int) -> Dict[str, np.ndarray]:
    """Tree of n_nodes nodes (root + the n_nodes - 1 best candidates).

    Returns parent int32 [T], depth int32 [T], token int32 [T] (token[0] = root_token),
    cand int32 [T] (candidate index of each node, -1 for the root)."""
    par = np.asarray(cand_parent, dtype=np.int64)
    n_cand = len(par)
    n_keep = n_nodes - 1
    if n_keep < 0 or n_keep > n_cand:
        raise ValueError("need 0 <= n_nodes - 1 <= number of candidates")
    score = candidate_scores(par, cand_logp)
    order = sorted(range(n_cand), key=lambda c: (-float(score[c]), c))
    keep = sorted(order[:n_keep])
    cdepth = np.zeros(n_cand, dtype=np.int64)
    for c in range(n_cand):
        cdepth[c] = 1 if par[c] < 0 else cdepth[par[c]] + 1
    bfs = sorted(keep, key=lambda c: (cdepth[c], c))
    node_of = {c: i + 1 for i, c in enumerate(bfs)}
    parent = np.full(n_nodes, -1, dtype=np.int32)
    depth = np.zeros(n_nodes, dtype=np.int32)
    token = np.zeros(n_nodes, dtype=np.int32)
    cand = np.full(n_nodes, -1, dtype=np.int32)
    token[0] = root_token
    for c in bfs:
        i = node_of[c]
        if par[c] >= 0 and par[c] not in node_of:
            raise AssertionError("kept set is not closed under parent-of")
        parent[i] = 0 if par[c] < 0 else node_of[int(par[c])]
        depth[i] = cdepth[c]
        token[i] = int(np.asarray(cand_token)[c])
        cand[i] = c
    return {"parent": parent, "depth": depth, "token": token, "cand": cand}
