"""Brute-force references for tiny inputs.  TEST INFRASTRUCTURE ONLY.

Written on purpose without importing verify_oracle.py (and nothing from the
product): the two files are compared with each other in the tests, so a mistake
in the tree mask, the positions, the rotary pairing or the acceptance scan of
one of them shows up as a disagreement.

  * `decode_token`  - an ordinary one-token Llama decode step against a private
    KV cache (no tree, no mask): the sequential decoding that tree verification
    reorganises (Eq. 1).
  * `decode_paths`  - every root-to-leaf path of a tree decoded that way, one
    token at a time, each path with its own cache.
  * `chain_scan`    - the acceptance loop of Alg. 1 on a single chain of draft
    tokens: accept while the bin distance is at most r, stop at the first
    rejection keeping the verifier's token, add the extra token if all passed.
  * `accept_over_paths` - that scan applied to every root-to-leaf path.
  * `greedy_decode` - greedy autoregressive decoding (Eq. 1) with an embedding
    table, the output that strict acceptance (r = 0) has to reproduce.

Python loops throughout; meant for hidden sizes of a few hundred at most.
"""
from __future__ import annotations

import math
from typing import Dict, List, Sequence

import numpy as np


def _norm(vec, gain, eps):
    total = 0.0
    for t in vec:
        total += float(t) * float(t)
    scale = 1.0 / math.sqrt(total / len(vec) + eps)
    return np.array([float(vec[i]) * scale * float(gain[i]) for i in range(len(vec))])


def _rotate(vec, position, theta):
    """Rotary embedding of one head vector at an integer position."""
    d = len(vec)
    out = np.array(vec, dtype=np.float64)
    for j in range(d // 2):
        angle = position / (theta ** (2.0 * j / d))
        a, b = float(vec[j]), float(vec[j + d // 2])
        out[j] = a * math.cos(angle) - b * math.sin(angle)
        out[j + d // 2] = a * math.sin(angle) + b * math.cos(angle)
    return out


def new_cache(prefix_kv):
    """Private cache: per layer, per head, a list of key rows and of value rows."""
    cache = []
    for kp, vp in prefix_kv:
        cache.append(([list(kp[h]) for h in range(kp.shape[0])],
                      [list(vp[h]) for h in range(vp.shape[0])]))
    return cache


def decode_token(x_row, position, layers, cache, n_heads, eps, theta):
    """Feed one token row through all layers, appending to `cache`; returns the
    final residual row."""
    x = np.array(x_row, dtype=np.float64)
    for w, (kc, vc) in zip(layers, cache):
        d = w["wq"].shape[0] // n_heads
        xn = _norm(x, w["g1"], eps)
        q_all, k_all, v_all = w["wq"] @ xn, w["wk"] @ xn, w["wv"] @ xn
        heads_out = []
        for h in range(n_heads):
            q = _rotate(q_all[h * d:(h + 1) * d], position, theta)
            k = _rotate(k_all[h * d:(h + 1) * d], position, theta)
            kc[h].append(k)
            vc[h].append(v_all[h * d:(h + 1) * d])
            scores = [float(np.dot(q, kk)) / math.sqrt(d) for kk in kc[h]]
            top = max(scores)
            weights = [math.exp(s - top) for s in scores]
            z = sum(weights)
            o = np.zeros(d)
            for wt, vv in zip(weights, vc[h]):
                o += (wt / z) * np.asarray(vv, dtype=np.float64)
            heads_out.append(o)
        x = x + w["wo"] @ np.concatenate(heads_out)
        xn = _norm(x, w["g2"], eps)
        gate, up = w["wg"] @ xn, w["wu"] @ xn
        act = np.array([g / (1.0 + math.exp(-g)) for g in gate]) * up
        x = x + w["wd"] @ act
    return x


def head_logits(x_row, g_final, w_rows, eps):
    return w_rows @ _norm(x_row, g_final, eps)


def leaf_paths(parent: Sequence[int]) -> List[List[int]]:
    T = len(parent)
    has_child = [False] * T
    for c in range(1, T):
        has_child[parent[c]] = True
    paths = []
    for leaf in range(T):
        if has_child[leaf]:
            continue
        p, n = [], leaf
        while n != -1:
            p.append(n)
            n = int(parent[n])
        paths.append(p[::-1])
    return paths


def decode_paths(x, layers, prefix_kv, g_final, w_rows, parent, n_heads, eps, theta):
    """Sequentially decode every root-to-leaf path.  Returns {node: [logits from
    each path that contains the node]} and the same for the final residual rows."""
    P = prefix_kv[0][0].shape[1]
    logits: Dict[int, list] = {}
    finals: Dict[int, list] = {}
    for path in leaf_paths(parent):
        cache = new_cache(prefix_kv)
        for step, node in enumerate(path):
            out = decode_token(x[node], P + step, layers, cache, n_heads, eps, theta)
            finals.setdefault(node, []).append(out)
            logits.setdefault(node, []).append(head_logits(out, g_final, w_rows, eps))
    return logits, finals


def chain_scan(draft_chain: Sequence[int], target_chain: Sequence[int], action_lo: int,
               n_bins: int, r: int):
    """Alg. 1's loop on one chain.  draft_chain[i] (i >= 1) was drafted for the
    position whose verifier token is target_chain[i-1]; entry 0 of draft_chain
    is the committed root token.  Returns (accepted count, emitted tokens)."""
    emitted = []
    n_acc = 0
    for i in range(1, len(draft_chain)):
        a_hat, a = int(draft_chain[i]), int(target_chain[i - 1])
        in_range = (action_lo <= a_hat < action_lo + n_bins) and (action_lo <= a < action_lo + n_bins)
        if in_range and abs(a_hat - a) <= r:
            emitted.append(a_hat)
            n_acc += 1
        else:
            emitted.append(a)
            return n_acc, emitted
    emitted.append(int(target_chain[len(draft_chain) - 1]))   # the extra token
    return n_acc, emitted


def accept_over_paths(parent, draft_token, target_token, action_lo, n_bins, r):
    """Scan every root-to-leaf path; returns (best length, set of nodes accepted
    on some path (root included), list of (length, emitted tokens) per path)."""
    accepted = {0}
    best = 0
    per_path = []
    for path in leaf_paths(parent):
        n_acc, emitted = chain_scan([draft_token[n] for n in path],
                                    [target_token[n] for n in path], action_lo, n_bins, r)
        accepted.update(path[1:1 + n_acc])
        best = max(best, n_acc)
        per_path.append((n_acc, emitted))
    return best, accepted, per_path


def greedy_decode(embed, first_token, n_tokens, layers, prefix_kv, g_final, w_rows,
                  token_lo, n_heads, eps, theta):
    """Greedy autoregressive decoding (Eq. 1) of n_tokens tokens after first_token,
    the argmax running over ids token_lo .. token_lo + len(w_rows) - 1."""
    P = prefix_kv[0][0].shape[1]
    cache = new_cache(prefix_kv)
    out = []
    tok = int(first_token)
    for step in range(n_tokens):
        h = decode_token(embed[tok], P + step, layers, cache, n_heads, eps, theta)
        lg = head_logits(h, g_final, w_rows, eps)
        tok = token_lo + int(np.argmax(lg))
        out.append(tok)
    return out
