"""CPU oracle for one Spec-VLA tree-verification step.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the CPU-baseline leg of the benchmark may
import this file; the product path (the HIP library and its binding) never
does, and this file imports nothing from the product.  Everything is float64
numpy, written as the plain definition of what the step computes, in the
paper's order, with no blocking, fusion or reordering:

  * the verifier scores every draft position in one pass (Alg. 1, the "compute
    the reference token set in parallel" step; Sec. 4.1: the draft tokens form
    a tree whose paths are verified in parallel).  For a node i of the tree that
    means: the logits of node i are those an ordinary causal Llama forward gives
    at the last position of  prefix + tokens on the path root..i.  Hence node i
    attends to every prefix key and to the tree nodes that are its ancestors or
    itself, and sits at position  P + depth(i).
  * the verifier's choice is the greedy argmax (Eq. 1), here over the action
    tokens, the lowest id winning exact ties.
  * a draft token is accepted when the distance between its bin and the bin of
    the verifier's choice is at most r (Eq. 5; Sec. 4.3: distance = absolute
    difference of bin ids, 256 bins); r = 0 is the strict rule (Eq. 3).  Tokens
    after the first rejected one on a path are dropped (Sec. 3.2, Alg. 1).
  * accepted positions keep the draft's token; the verifier's own token follows
    at the first rejected position, or as the extra token when the whole path
    was accepted (Alg. 1), so a step always emits accepted_len + 1 tokens
    (Sec. 6: the verifier always contributes a length of 1).

Conventions the paper does not fix (RMSNorm epsilon, rotate-half RoPE pairing,
tie-breaks among equally long accepted paths) are parameters or are stated at
the function that takes them; the pairing and epsilon are checked in the tests
against the Llama decoder layer of the `transformers` library.

Pins (tests/test_oracle_*.py): per-path sequential decoding (sequential_decode.py,
no shared code), transformers' LlamaDecoderLayer, torch's rms_norm / silu /
scaled_dot_product_attention, brute force over all small trees, closed forms for
the acceptance length, the r = 0 = greedy decoding invariant, and the token lists
of the paper's case study.  Parity unpinned: none of the functions below; the
tie-break rule of `relaxed_accept` for the *path* (not mask or length) is a
convention and is only checked for self-consistency.
"""
from __future__ import annotations

from typing import Dict, Iterable, Optional, Sequence

import numpy as np


def tree_structure(parent: Sequence[int]):
    """Depth of every node and the ancestor-or-self relation of a draft tree.

    `parent[0]` must be -1 (root) and 0 <= parent[i] < i otherwise.  Returns
    (depth int64 [T], anc bool [T, T]) with anc[i, j] true iff j lies on the path
    root..i (i itself included)."""
    parent = np.asarray(parent, dtype=np.int64)
    T = parent.shape[0]
    if T < 1 or parent[0] != -1:
        raise ValueError("node 0 must be the root with parent -1")
    depth = np.zeros(T, dtype=np.int64)
    anc = np.zeros((T, T), dtype=bool)
    anc[0, 0] = True
    for i in range(1, T):
        p = int(parent[i])
        if not (0 <= p < i):
            raise ValueError(f"parent[{i}] = {p} is not an earlier node")
        depth[i] = depth[p] + 1
        anc[i] = anc[p]
        anc[i, i] = True
    return depth, anc


def rms_norm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """Llama RMSNorm over the last axis: x / sqrt(mean(x^2) + eps) * gain."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(v: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing.

    v [T, n_heads, d]; pos [T] integer positions.  Component j < d/2 is paired
    with j + d/2 and the pair is rotated by the angle pos * theta^(-2j/d)."""
    d = v.shape[-1]
    half = d // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]   # [T, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    lo, hi = v[..., :half], v[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def verify_layer(x: np.ndarray, w: Dict[str, np.ndarray], k_prefix: np.ndarray,
                 v_prefix: np.ndarray, parent: Sequence[int], n_heads: int,
                 eps: float, theta: float) -> Dict[str, np.ndarray]:
    """One Llama decoder layer over the T rows of a draft tree.

    x [T, H] residual stream; w: g1, wq, wk, wv, wo, g2, wg, wu, wd with the
    matrices stored [out, in]; k_prefix / v_prefix [n_heads, P, d] are used as
    given (prefix keys are already rotated).  Returns the new residual stream
    "x", the attention output before the output projection "attn" [T, H] and
    the tree's own rotated keys / values "k_tree", "v_tree" [T, n_heads, d]."""
    T, H = x.shape
    P = k_prefix.shape[1]
    d = k_prefix.shape[2]
    depth, anc = tree_structure(parent)

    xh = rms_norm(x, w["g1"], eps)
    q = (xh @ w["wq"].T).reshape(T, n_heads, d)
    k = (xh @ w["wk"].T).reshape(T, n_heads, d)
    v = (xh @ w["wv"].T).reshape(T, n_heads, d)
    pos = P + depth
    q = rope(q, pos, theta)
    k = rope(k, pos, theta)

    attn = np.zeros((T, n_heads, d), dtype=np.float64)
    for h in range(n_heads):
        for i in range(T):
            keys = np.concatenate([k_prefix[h], k[anc[i], h]], axis=0)
            vals = np.concatenate([v_prefix[h], v[anc[i], h]], axis=0)
            s = keys @ q[i, h] / np.sqrt(d)
            p = np.exp(s - s.max())
            p /= p.sum()
            attn[i, h] = p @ vals
    attn = attn.reshape(T, n_heads * d)

    x1 = x + attn @ w["wo"].T
    xh2 = rms_norm(x1, w["g2"], eps)
    mlp = (silu(xh2 @ w["wg"].T) * (xh2 @ w["wu"].T)) @ w["wd"].T
    return {"x": x1 + mlp, "attn": attn, "k_tree": k, "v_tree": v}


def action_head(x: np.ndarray, g_final: np.ndarray, w_rows: np.ndarray,
                token_lo: int, eps: float):
    """Final RMSNorm, logits of the scored vocabulary rows, greedy choice (Eq. 1).

    w_rows [n_scored, H] are the LM-head rows of token ids token_lo ..
    token_lo + n_scored - 1.  Returns (logits [T, n_scored], token int64 [T]);
    the lowest id wins exact ties."""
    z = rms_norm(x, g_final, eps)
    logits = z @ w_rows.T
    return logits, token_lo + np.argmax(logits, axis=-1).astype(np.int64)


def relaxed_accept(parent: Sequence[int], draft_token: Sequence[int],
                   target_token: Sequence[int], action_lo: int, n_bins: int, r: int):
    """Relaxed acceptance over a draft tree and the longest accepted path.

    draft_token[c] is the token the drafter put at node c (entry 0, the root, is
    the last committed token and is never tested); target_token[j] is the
    verifier's greedy choice for the position after node j.  bin(t) = t -
    action_lo.  Node c >= 1 passes its own test when |bin(draft[c]) -
    bin(target[parent[c]])| <= r (Eq. 5); a token outside the action range never
    passes.  A node is accepted when it and all nodes above it pass (everything
    after the first rejection on a path is dropped).  Among the accepted nodes
    the deepest is taken, the lowest index among equally deep ones.

    Returns dict: mask bool [T] (root true), length (= depth of the best node),
    best, path (root..best), tokens (accepted draft tokens, then the verifier's
    token at the best node: length + 1 entries)."""
    parent = np.asarray(parent, dtype=np.int64)
    draft = np.asarray(draft_token, dtype=np.int64)
    target = np.asarray(target_token, dtype=np.int64)
    depth, _ = tree_structure(parent)
    T = parent.shape[0]

    def bin_of(t):
        b = int(t) - action_lo
        return b if 0 <= b < n_bins else None

    acc = np.zeros(T, dtype=bool)
    acc[0] = True
    for c in range(1, T):
        bd, bt = bin_of(draft[c]), bin_of(target[parent[c]])
        ok = bd is not None and bt is not None and abs(bd - bt) <= r
        acc[c] = ok and acc[parent[c]]
    best = 0
    for c in range(1, T):
        if acc[c] and depth[c] > depth[best]:
            best = c
    path = []
    n = best
    while n != -1:
        path.append(n)
        n = int(parent[n])
    path.reverse()
    tokens = [int(draft[n]) for n in path[1:]] + [int(target[best])]
    return {"mask": acc, "length": int(depth[best]), "best": int(best),
            "path": path, "tokens": tokens}


def verify_step(x: np.ndarray, layers: Iterable[Dict[str, np.ndarray]],
                prefix_kv: Iterable, g_final: np.ndarray, w_rows: np.ndarray,
                token_lo: int, parent: Sequence[int], n_heads: int, eps: float,
                theta: float, keep_layers: bool = False):
    """All layers, then the action head, for one episode.

    `layers` and `prefix_kv` are iterated in step (one dict of float64 weights and
    one (k_prefix, v_prefix) pair per layer), so a caller can stream a large
    model layer by layer.  Returns dict with "x" (final residual stream),
    "logits", "token" and, if asked, the per-layer outputs of `verify_layer`."""
    per_layer = []
    for w, (kp, vp) in zip(layers, prefix_kv):
        out = verify_layer(x, w, kp, vp, parent, n_heads, eps, theta)
        x = out["x"]
        if keep_layers:
            per_layer.append(out)
    logits, token = action_head(x, g_final, w_rows, token_lo, eps)
    return {"x": x, "logits": logits, "token": token, "layers": per_layer}
