"""Pins of the oracle's acceptance rule and path selection (CPU only).

Held against: the strict rule (Eq. 3) at r = 0, the size of the acceptance window
(Sec. 4.3), monotonicity in r (Eq. 5), the chain scan of Alg. 1 run on every
root-to-leaf path (oracle/sequential_decode.py, separate code) over ALL trees of up to
six nodes, a closed form for the expected accepted length on chains, the token lists
of the paper's case study, and greedy decoding (Eq. 1) for r = 0.
"""
import itertools
import os

import numpy as np
import pytest
import torch

from oracle import sequential_decode as seq
from oracle import verify_oracle as vo
from paper_2507_22424_amd import workload as wl

LO, NB = 31744, 256           # action tokens = top 256 ids of a 32000-token vocabulary


def accept(parent, draft, target, r, lo=LO, nb=NB):
    return vo.relaxed_accept(parent, draft, target, lo, nb, r)


def test_r0_is_strict_matching():
    rng = np.random.default_rng(0)
    for _ in range(200):
        d = int(rng.integers(1, 8))
        parent = np.arange(-1, d)
        target = LO + rng.integers(0, 4, size=d + 1)
        draft = LO + rng.integers(0, 4, size=d + 1)
        res = accept(parent, draft, target, 0)
        n = 0
        while n < d and draft[n + 1] == target[n]:
            n += 1
        assert res["length"] == n
        assert res["mask"].tolist() == [True] * (n + 1) + [False] * (d - n)


@pytest.mark.parametrize("r", [0, 1, 4, 9, 300])
def test_window_holds_2r_plus_1_bins_clipped_to_the_bin_range(r):
    for b in (0, 1, 3, 100, 250, 255):
        n_ok = 0
        for bd in range(NB):
            res = accept([-1, 0], [LO, LO + bd], [LO + b, LO], r)
            n_ok += res["length"]
        assert n_ok == min(b + r, NB - 1) - max(b - r, 0) + 1


def test_tokens_outside_the_action_range_are_never_accepted():
    for bad in (LO - 1, LO + NB, 0):
        assert accept([-1, 0], [LO, bad], [LO, LO], 400)["length"] == 0
        assert accept([-1, 0], [LO, LO], [bad, LO], 400)["length"] == 0


def test_monotone_in_r_and_everything_accepted_at_r_255():
    cfg = wl.C3
    rng = np.random.default_rng(3)
    for ep in range(20):
        parent = wl.draft_tree(cfg.tree_nodes, cfg.max_depth, cfg.max_children, 7, rng)
        target = LO + rng.integers(0, NB, size=cfg.tree_nodes)
        draft = wl.noisy_draft_tokens(cfg.scaled(index=ep), 0, parent, target, spread=12)
        prev_mask, prev_len = None, -1
        for r in range(0, 14):
            res = accept(parent, draft, target, r)
            if prev_mask is not None:
                assert np.all(res["mask"] >= prev_mask)
            assert res["length"] >= prev_len
            prev_mask, prev_len = res["mask"], res["length"]
        res = accept(parent, draft, target, 255)
        assert res["mask"].all() and res["length"] == 7


def all_parent_arrays(T):
    for tail in itertools.product(*[range(i) for i in range(1, T)]):
        yield np.array((-1,) + tail)


@pytest.mark.parametrize("T", [1, 2, 3, 4, 5, 6])
def test_every_small_tree_against_the_per_path_chain_scan(T):
    rng = np.random.default_rng(T)
    for parent in all_parent_arrays(T):
        for _ in range(4):
            target = 10 + rng.integers(0, 5, size=T)
            draft = 10 + rng.integers(0, 5, size=T)
            for r in (0, 1, 2):
                res = vo.relaxed_accept(parent, draft, target, 10, 5, r)
                best, nodes, per_path = seq.accept_over_paths(parent, draft, target, 10, 5, r)
                assert res["length"] == best
                assert set(np.flatnonzero(res["mask"]).tolist()) == nodes
                # the emitted tokens are those of a path reaching the best length, and a
                # step always emits accepted + 1 tokens (Sec. 6)
                assert len(res["tokens"]) == res["length"] + 1
                assert any(n == best and em == res["tokens"] for n, em in per_path) or \
                    any(n == best and em[:best] == res["tokens"][:best] for n, em in per_path)
                assert res["path"][0] == 0 and res["path"][-1] == res["best"]
                assert res["tokens"][:-1] == [int(draft[n]) for n in res["path"][1:]]
                assert res["tokens"][-1] == int(target[res["best"]])


def test_best_node_is_the_lowest_index_among_the_deepest_accepted():
    #      0
    #    1   2        draft bins equal the target bins everywhere: all accepted
    #   3 4   5       deepest level holds 3, 4, 5 -> node 3
    parent = [-1, 0, 0, 1, 1, 2]
    tok = [LO + 7] * 6
    res = accept(parent, tok, tok, 0)
    assert res["best"] == 3 and res["path"] == [0, 1, 3] and res["length"] == 2
    # reject node 3 only: now 4
    draft = list(tok); draft[3] = LO + 9
    assert accept(parent, draft, tok, 1)["best"] == 4


@pytest.mark.parametrize("r", [0, 2, 8])
def test_expected_length_on_chains_matches_the_geometric_closed_form(r):
    """Chain of depth 7, draft bin = target bin + uniform offset in [-8, 8], no clipping:
    each edge passes independently with p = (2r+1)/17, so E[len] = sum_k p^k."""
    rng = np.random.default_rng(11 + r)
    n_trees, d = 20000, 7
    parent = np.arange(-1, d)
    total = 0
    for _ in range(n_trees):
        target = LO + rng.integers(8, NB - 8, size=d + 1)
        draft = np.empty(d + 1, dtype=np.int64)
        draft[0] = LO
        draft[1:] = target[:-1] + rng.integers(-8, 9, size=d)
        total += accept(parent, draft, target, r)["length"]
    p = (2 * r + 1) / 17.0
    expect = sum(p ** k for k in range(1, d + 1))
    var_bound = d * d / 4.0
    assert abs(total / n_trees - expect) < 5 * np.sqrt(var_bound / n_trees)
    if r == 8:
        assert total == n_trees * d


def test_paper_case_study_token_lists():
    path = os.path.join(os.path.dirname(__file__), "golden", "case_study_action1.txt")
    rows = {}
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        rows[key] = [int(v) for v in vals]
    strict, relaxed, r = rows["strict"], rows["relaxed"], rows["threshold"][0]
    d = len(strict) - 1
    parent = np.arange(-1, d)
    # bins 1..256 <-> tokens 1..256; target[i] = the strict run's token after position i
    target = strict[1:] + [strict[-1]]
    res = vo.relaxed_accept(parent, relaxed, target, 1, 256, r)
    assert res["length"] == d and res["tokens"][:-1] == relaxed[1:]
    # the largest distance on the list is exactly the threshold: one less rejects at once
    assert vo.relaxed_accept(parent, relaxed, target, 1, 256, r - 1)["length"] == 0
    # strict acceptance takes nothing here (first drafted token differs)
    assert vo.relaxed_accept(parent, relaxed, target, 1, 256, 0)["length"] == 0
    assert vo.relaxed_accept(parent, relaxed, target, 1, 256, 0)["tokens"] == [strict[1]]


def test_strict_acceptance_reproduces_greedy_decoding():
    """r = 0: whatever the tree, the emitted tokens are the first len+1 tokens that greedy
    autoregressive decoding produces after the root token; with the greedy sequence planted
    on a path the whole planted part is accepted."""
    cfg = wl.C1.scaled(name="greedy", index=9, hidden=32, n_heads=2, head_dim=16, mlp_dim=48,
                       vocab=80, n_bins=16, n_layers=2, prefix_lo=4, prefix_hi=4,
                       tree_nodes=12, max_depth=5, max_children=3, spine_lo=5)
    f64 = lambda t: t.to(torch.float64).numpy()
    layers = [{k: f64(v) for k, v in wl.layer_weights(cfg, l).items()} for l in range(2)]
    kv = [tuple(f64(t) for t in wl.prefix_kv(cfg, 0, l, 4)) for l in range(2)]
    head = {k: f64(v) for k, v in wl.head_weights(cfg).items()}
    E = f64(wl.embedding_table(cfg))
    lo = cfg.action_lo
    args = (cfg.n_heads, cfg.rms_eps, cfg.rope_theta)
    n_checked_planted = 0
    for trial in range(6):
        rng = np.random.default_rng(100 + trial)
        root_tok = lo + int(rng.integers(cfg.n_bins))
        greedy = seq.greedy_decode(E, root_tok, cfg.max_depth + 1, layers, kv, head["g_final"],
                                   head["w_lm"], lo, *args)
        parent = wl.draft_tree(cfg.tree_nodes, cfg.max_depth, cfg.max_children, 5, rng)
        depth, _ = vo.tree_structure(parent)
        draft = lo + rng.integers(0, cfg.n_bins, size=cfg.tree_nodes)
        draft[0] = root_tok
        planted = int(rng.integers(0, cfg.max_depth + 1))
        # node i (1..5) is the spine node of depth i after BFS relabelling? not guaranteed:
        # walk down from the root taking the first child each time
        node, on_path = 0, []
        for _ in range(planted):
            kids = [c for c in range(cfg.tree_nodes) if parent[c] == node]
            if not kids:
                break
            node = kids[0]
            on_path.append(node)
        for j, n in enumerate(on_path):
            draft[n] = greedy[j]
        x = E[draft]
        out = vo.verify_step(x, layers, kv, head["g_final"], head["w_lm"], lo, parent, *args)
        res = vo.relaxed_accept(parent, draft, out["token"], lo, cfg.n_bins, 0)
        assert res["tokens"] == greedy[:res["length"] + 1]
        assert res["length"] >= len(on_path)
        n_checked_planted += len(on_path)
    assert n_checked_planted > 5
