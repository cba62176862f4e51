"""Pins of oracle/draft_tree.py (CPU only): what the stated definition implies, checked by
means that do not reuse the oracle's own code path."""
import itertools

import numpy as np
import pytest

from oracle import draft_tree as dt
from oracle import verify_oracle as vo
from paper_2507_22424_amd import workload as wl


def _random_forest(rng, n, max_kids=3):
    par, kids = [], {}
    for c in range(n):
        choices = [-1] + [p for p in range(c) if kids.get(p, 0) < max_kids]
        p = int(choices[rng.integers(len(choices))])
        par.append(p)
        kids[p] = kids.get(p, 0) + 1
    lp = -rng.random(n).astype(np.float32) * 3
    return np.array(par), lp


def test_scores_are_joint_log_probabilities_of_the_path():
    par = np.array([-1, -1, 0, 2, 1])
    lp = np.array([-0.5, -1.0, -0.25, -2.0, -0.125], dtype=np.float32)   # exact in binary
    s = dt.candidate_scores(par, lp)
    assert s.dtype == np.float32
    assert s.tolist() == [-0.5, -1.0, -0.75, -2.75, -1.125]


@pytest.mark.parametrize("seed", range(12))
def test_kept_set_is_the_best_parent_closed_set(seed):
    """Brute force: among all parent-closed candidate sets of the same size none has a larger
    total score (float64 sum of the float32 scores); the oracle's set attains the maximum."""
    rng = np.random.default_rng(seed)
    n = int(rng.integers(4, 11))
    par, lp = _random_forest(rng, n)
    score = dt.candidate_scores(par, lp).astype(np.float64)
    for n_keep in range(0, n + 1):
        out = dt.build_draft_tree(par, lp, np.arange(n), 7, n_keep + 1)
        kept = set(int(c) for c in out["cand"][1:])
        assert len(kept) == n_keep
        best = -np.inf
        for sub in itertools.combinations(range(n), n_keep):
            ss = set(sub)
            if all(par[c] < 0 or par[c] in ss for c in sub):
                best = max(best, sum(score[c] for c in sub))
        assert np.isclose(sum(score[c] for c in kept), best, rtol=0, atol=1e-9)
        assert all(par[c] < 0 or int(par[c]) in kept for c in kept)


def test_chain_and_star():
    # a chain: the best k candidates are its first k links, the tree is a path
    n = 6
    par = np.arange(-1, n - 1)
    lp = np.full(n, -0.5, dtype=np.float32)
    out = dt.build_draft_tree(par, lp, 100 + np.arange(n), 9, 4)
    assert out["parent"].tolist() == [-1, 0, 1, 2]
    assert out["depth"].tolist() == [0, 1, 2, 3]
    assert out["token"].tolist() == [9, 100, 101, 102]
    # a star: the children of the root with the highest log-probabilities, in candidate order
    par = np.full(5, -1)
    lp = np.array([-3, -1, -2, -0.5, -4], dtype=np.float32)
    out = dt.build_draft_tree(par, lp, np.arange(5), 0, 4)
    assert out["cand"].tolist() == [-1, 1, 2, 3]
    assert out["parent"].tolist() == [-1, 0, 0, 0]


def test_ties_go_to_the_lower_candidate_index_and_keep_parents():
    par = np.array([-1, 0, -1, 2])
    lp = np.array([-1.0, 0.0, -1.0, 0.0], dtype=np.float32)     # all four scores equal
    out = dt.build_draft_tree(par, lp, np.arange(4), 0, 3)
    assert out["cand"].tolist() == [-1, 0, 1]                     # 0 and its child 1, not 2


@pytest.mark.parametrize("seed", range(6))
def test_output_is_a_breadth_first_tree_consistent_with_the_verifier_oracle(seed):
    cfg = wl.C3
    f = wl.candidate_forest(top_k=8, depth=5, seed=seed, n_bins=cfg.n_bins, action_lo=cfg.action_lo)
    out = dt.build_draft_tree(f["parent"], f["logp"], f["token"], cfg.action_lo + 3, 50)
    parent, depth = out["parent"], out["depth"]
    assert parent[0] == -1 and all(0 <= parent[i] < i for i in range(1, 50))
    assert all(depth[i] <= depth[i + 1] for i in range(49))      # breadth first
    d2, _ = vo.tree_structure(parent)
    assert d2.tolist() == depth.tolist() and depth.max() <= 5
    # tokens and depths are those of the candidates kept
    for i in range(1, 50):
        assert out["token"][i] == f["token"][out["cand"][i]]
    # nothing left out scores higher than something kept
    s = dt.candidate_scores(f["parent"], f["logp"])
    kept = set(out["cand"][1:].tolist())
    worst_kept = min(s[c] for c in kept)
    assert all(s[c] <= worst_kept for c in range(len(s)) if c not in kept)
