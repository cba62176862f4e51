"""Seeded synthetic inputs for the Spec-VLA tree-verification pass.

This module only draws random inputs (weights, hidden rows, prefix KV, draft
trees, draft ids).  It holds none of the method's arithmetic: no norm, no
attention, no acceptance rule, and it imports neither the HIP binding nor the
CPU oracle.  Both sides of every parity test are fed from here, so they see the
identical values, already rounded once to the configuration's storage type.

The shapes stand in for the paper's workload (Sec. 5.1: a Llama-2-7B backbone
as verifier, one camera image plus an instruction as prefix, 256 action bins,
7-token actions, Eagle-2 style draft trees); the LIBERO data and the trained
weights themselves are not used anywhere.

Recipe
------
* base seed S0 = 20250722; configuration k, episode b, layer l use
  ``S0 + 100000*k + 1000*b + l`` (trees and ids use l = 999, the LM head l = 900,
  hidden rows l = 998); tensor number i inside one of those draws from
  ``torch.Generator`` (CPU, mt19937) seeded with ``16*seed + i``.
* matrices ~ N(0, std 0.02); RMSNorm gains 1 + N(0, 0.02); hidden rows and
  prefix K/V ~ N(0, 1); everything rounded once to the storage dtype.
* trees: node 0 is the root; a spine 0-1-..-D is laid first so the depth is
  reached, every further node picks its parent uniformly among nodes that are
  not at the maximum depth and still have room for a child; the nodes are then
  relabelled in breadth-first order so that parent[i] < i and depth never
  decreases with the index.  Integer draws use numpy's PCG64.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

S0 = 20250722

LAYER_TENSORS = ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")


@dataclasses.dataclass(frozen=True)
class VerifyConfig:
    """One row of the workload table (shapes only)."""

    name: str
    index: int              # k in the seed recipe
    dtype: str              # "f32" or "bf16" (storage type of weights / KV)
    n_layers: int
    hidden: int
    n_heads: int
    head_dim: int
    mlp_dim: int
    vocab: int
    n_bins: int             # action bins = the top n_bins ids of the vocabulary
    n_episodes: int
    prefix_lo: int          # prefix length is uniform in [prefix_lo, prefix_hi]
    prefix_hi: int
    tree_nodes: int         # T, root included
    max_depth: int
    max_children: int
    spine_lo: int           # spine length is uniform in [spine_lo, max_depth]
    r_values: Tuple[int, ...]
    rms_eps: float = 1e-5
    rope_theta: float = 1e4

    @property
    def action_lo(self) -> int:
        return self.vocab - self.n_bins

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    def scaled(self, **kw) -> "VerifyConfig":
        return dataclasses.replace(self, **kw)


def _llama7b(name, index, **kw) -> VerifyConfig:
    base = dict(dtype="bf16", n_layers=32, hidden=4096, n_heads=32, head_dim=128,
                mlp_dim=11008, vocab=32000, n_bins=256, n_episodes=1,
                prefix_lo=280, prefix_hi=280, tree_nodes=60, max_depth=7,
                max_children=4, spine_lo=7, r_values=(0, 1, 4, 8))
    base.update(kw)
    return VerifyConfig(name=name, index=index, **base)


C1 = VerifyConfig(name="C1-tiny-f32", index=0, dtype="f32", n_layers=1, hidden=256,
                  n_heads=4, head_dim=64, mlp_dim=688, vocab=512, n_bins=256,
                  n_episodes=1, prefix_lo=64, prefix_hi=64, tree_nodes=15,
                  max_depth=7, max_children=3, spine_lo=3, r_values=(0, 2))
C2 = _llama7b("C2-one-layer-bf16", 1, n_layers=1, tree_nodes=26, r_values=())
C3 = _llama7b("C3-full-bf16", 2)
C4 = _llama7b("C4-batched-bf16", 3, n_episodes=16, prefix_lo=260, prefix_hi=300,
              r_values=(4,))
C5 = _llama7b("C5-long-bf16", 4, prefix_lo=2048, prefix_hi=2048, tree_nodes=128,
              max_children=6, r_values=(0, 8))
CONFIGS = (C1, C2, C3, C4, C5)


def seed_for(cfg: VerifyConfig, episode: int, layer: int) -> int:
    return S0 + 100000 * cfg.index + 1000 * episode + layer


def _gen(seed: int, i: int) -> torch.Generator:
    return torch.Generator(device="cpu").manual_seed(16 * seed + i)


def _normal(shape, seed, i, dtype, std=1.0, mean=0.0) -> torch.Tensor:
    t = torch.randn(shape, generator=_gen(seed, i), dtype=torch.float32)
    if std != 1.0:
        t.mul_(std)
    if mean != 0.0:
        t.add_(mean)
    return t.to(dtype)


def layer_weights(cfg: VerifyConfig, layer: int) -> Dict[str, torch.Tensor]:
    """The nine tensors of decoder layer `layer`, matrices stored [out, in]."""
    H, F, D = cfg.hidden, cfg.mlp_dim, cfg.n_heads * cfg.head_dim
    shapes = {"g1": (H,), "wq": (D, H), "wk": (D, H), "wv": (D, H), "wo": (H, D),
              "g2": (H,), "wg": (F, H), "wu": (F, H), "wd": (H, F)}
    seed = seed_for(cfg, 0, layer)
    out = {}
    for i, name in enumerate(LAYER_TENSORS):
        if name.startswith("g"):
            out[name] = _normal(shapes[name], seed, i, cfg.torch_dtype, 0.02, 1.0)
        else:
            out[name] = _normal(shapes[name], seed, i, cfg.torch_dtype, 0.02)
    return out


def layer_weights_w8(cfg: VerifyConfig, layer: int) -> Dict[str, torch.Tensor]:
    """Decoder layer `layer` with 8-bit matrices: gains as in layer_weights; every matrix `w*` as
    uint8 E4M3 codes [out, in] (a standard normal draw converted by torch's float8_e4m3fn type)
    plus `w*_scale`, float32 [out], about 0.02 with a spread of a few tens of percent per row - so
    the dequantised matrix looks like the bf16 one."""
    H, F, D = cfg.hidden, cfg.mlp_dim, cfg.n_heads * cfg.head_dim
    shapes = {"g1": (H,), "wq": (D, H), "wk": (D, H), "wv": (D, H), "wo": (H, D),
              "g2": (H,), "wg": (F, H), "wu": (F, H), "wd": (H, F)}
    seed = seed_for(cfg, 0, layer) + 7777
    out = {}
    for i, name in enumerate(LAYER_TENSORS):
        if name.startswith("g"):
            out[name] = _normal(shapes[name], seed, i, torch.bfloat16, 0.02, 1.0)
        else:
            z = _normal(shapes[name], seed, i, torch.float32, 1.0)
            out[name] = z.to(torch.float8_e4m3fn).view(torch.uint8)
            u = torch.rand(shapes[name][0], generator=_gen(seed, 100 + i), dtype=torch.float32)
            out[name + "_scale"] = 0.02 * (0.75 + 0.5 * u)
    return out


def layer_weights_w4(cfg: VerifyConfig, layer: int) -> Dict[str, torch.Tensor]:
    """Decoder layer `layer` with 4-bit integer matrices: gains as in layer_weights; every matrix
    `w*` as uint8 [out, in / 2] holding two codes per byte (the code of the even k in the low four
    bits; a code c in 0 .. 15 stands for the integer c - 8: a normal draw of standard deviation 2.5,
    rounded and clipped to -8 .. 7) plus `w*_scale`, float32 [out], about 0.008 with a spread of a
    few tens of percent per row - so the dequantised matrix has the scale of the bf16 one."""
    H, F, D = cfg.hidden, cfg.mlp_dim, cfg.n_heads * cfg.head_dim
    shapes = {"g1": (H,), "wq": (D, H), "wk": (D, H), "wv": (D, H), "wo": (H, D),
              "g2": (H,), "wg": (F, H), "wu": (F, H), "wd": (H, F)}
    seed = seed_for(cfg, 0, layer) + 4444
    out = {}
    for i, name in enumerate(LAYER_TENSORS):
        if name.startswith("g"):
            out[name] = _normal(shapes[name], seed, i, torch.bfloat16, 0.02, 1.0)
        else:
            z = _normal(shapes[name], seed, i, torch.float32, 2.5)
            code = (torch.clamp(torch.round(z), -8, 7) + 8).to(torch.uint8)
            out[name] = (code[:, 0::2] | (code[:, 1::2] << 4)).contiguous()
            u = torch.rand(shapes[name][0], generator=_gen(seed, 100 + i), dtype=torch.float32)
            out[name + "_scale"] = 0.008 * (0.75 + 0.5 * u)
    return out


def all_layer_weights(cfg: VerifyConfig, workers: int = 8) -> List[Dict[str, torch.Tensor]]:
    """All layers; the draws are independent per layer so they run in threads."""
    with ThreadPoolExecutor(max_workers=max(1, workers)) as ex:
        return list(ex.map(lambda l: layer_weights(cfg, l), range(cfg.n_layers)))


def head_weights(cfg: VerifyConfig, full_vocab: bool = False) -> Dict[str, torch.Tensor]:
    """Final RMSNorm gain and the LM head.

    With ``full_vocab=False`` only the action rows [vocab - n_bins, vocab) are
    drawn (shape [n_bins, hidden]); those rows have the same values as the tail
    of nothing else - the full matrix uses its own tensor number.
    """
    seed = seed_for(cfg, 0, 900)
    g = _normal((cfg.hidden,), seed, 0, cfg.torch_dtype, 0.02, 1.0)
    if full_vocab:
        w = _normal((cfg.vocab, cfg.hidden), seed, 2, cfg.torch_dtype, 0.02)
    else:
        w = _normal((cfg.n_bins, cfg.hidden), seed, 1, cfg.torch_dtype, 0.02)
    return {"g_final": g, "w_lm": w}


def hidden_rows(cfg: VerifyConfig, episode: int) -> torch.Tensor:
    """Input rows of the tree nodes of one episode, [T, hidden] ~ N(0,1)."""
    return _normal((cfg.tree_nodes, cfg.hidden), seed_for(cfg, episode, 998), 0,
                   cfg.torch_dtype)


def row_magnitudes(cfg: VerifyConfig, episode: int, decades: float) -> torch.Tensor:
    """One positive factor per tree node, 10^u with u uniform in [-decades, decades]: input rows of
    very different size inside one batch (an outlier token, episodes at different scales)."""
    rng = np.random.Generator(np.random.PCG64(seed_for(cfg, episode, 996)))
    u = rng.uniform(-decades, decades, size=cfg.tree_nodes)
    return torch.from_numpy((10.0 ** u).astype(np.float32))


def prefix_lengths(cfg: VerifyConfig) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed_for(cfg, 0, 997)))
    return rng.integers(cfg.prefix_lo, cfg.prefix_hi + 1, size=cfg.n_episodes).astype(np.int32)


def prefix_kv(cfg: VerifyConfig, episode: int, layer: int, prefix_len: int
              ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Prefix keys and values of one layer, each [n_heads, prefix_len, head_dim].

    They are used as they are: keys count as already rotated."""
    seed = seed_for(cfg, episode, layer)
    shape = (cfg.n_heads, prefix_len, cfg.head_dim)
    return (_normal(shape, seed, 12, cfg.torch_dtype),
            _normal(shape, seed, 13, cfg.torch_dtype))


def draft_tree(n_nodes: int, max_depth: int, max_children: int, spine: int,
               rng: np.random.Generator) -> np.ndarray:
    """Parent array of a random tree (root = 0, parent[0] = -1, parent[i] < i)."""
    if n_nodes < 1:
        raise ValueError("a tree has at least its root")
    spine = min(spine, max_depth, n_nodes - 1)
    parent = [-1]
    depth = [0]
    kids = [0]
    for i in range(1, spine + 1):
        parent.append(i - 1); depth.append(i); kids.append(0); kids[i - 1] += 1
    while len(parent) < n_nodes:
        open_ = [j for j in range(len(parent))
                 if depth[j] < max_depth and kids[j] < max_children]
        if not open_:
            raise ValueError("tree shape cannot hold that many nodes")
        p = open_[int(rng.integers(len(open_)))]
        parent.append(p); depth.append(depth[p] + 1); kids.append(0); kids[p] += 1
    # breadth-first relabelling (stable in the old index inside one level)
    order = sorted(range(n_nodes), key=lambda j: (depth[j], j))
    new_of = {old: new for new, old in enumerate(order)}
    out = np.full(n_nodes, -1, dtype=np.int32)
    for old in range(n_nodes):
        if parent[old] >= 0:
            out[new_of[old]] = new_of[parent[old]]
    return out


def episode_tree(cfg: VerifyConfig, episode: int) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(seed_for(cfg, episode, 999)))
    spine = int(rng.integers(cfg.spine_lo, cfg.max_depth + 1))
    return draft_tree(cfg.tree_nodes, cfg.max_depth, cfg.max_children, spine, rng)


def candidate_forest(top_k: int, depth: int, seed: int, n_bins: int = 256, action_lo: int = 0):
    """Synthetic record of a drafter's top-K predictions, level by level, shaped like a
    dynamic draft tree's candidates (Sec. 4.1, Sec. 5.1: top 8, depth 4-5): level 1 holds
    top_k children of the root; at every further level the top_k candidates of the level
    above with the highest joint log-probability are expanded, each into top_k children.
    Log-probabilities are the top_k entries of a log-softmax over random logits.
    Returns dict(parent int32 [n] (-1 = child of the root, else an earlier candidate),
    logp float32 [n], token int32 [n]); n = top_k + (depth - 1) * top_k**2."""
    rng = np.random.Generator(np.random.PCG64(S0 + 7919 * seed + 17))
    parent, logp, token, joint = [], [], [], []

    def children(of: int, base: float):
        logits = rng.standard_normal(n_bins) * 2.0
        lsm = logits - np.log(np.sum(np.exp(logits)))
        top = np.argsort(-lsm, kind="stable")[:top_k]
        for t in top:
            parent.append(of); logp.append(np.float32(lsm[t])); token.append(action_lo + int(t))
            joint.append(base + float(np.float32(lsm[t])))

    children(-1, 0.0)
    level = list(range(top_k))
    for _ in range(depth - 1):
        expand = sorted(level, key=lambda c: (-joint[c], c))[:top_k]
        first = len(parent)
        for c in sorted(expand):
            children(c, joint[c])
        level = list(range(first, len(parent)))
    return {"parent": np.asarray(parent, dtype=np.int32), "logp": np.asarray(logp, dtype=np.float32),
            "token": np.asarray(token, dtype=np.int32)}


def uniform_draft_tokens(cfg: VerifyConfig, episode: int) -> np.ndarray:
    """Draft ids uniform over the action tokens (entry 0, the root, is unused)."""
    rng = np.random.Generator(np.random.PCG64(seed_for(cfg, episode, 996)))
    return (cfg.action_lo + rng.integers(0, cfg.n_bins, size=cfg.tree_nodes)).astype(np.int32)


def noisy_draft_tokens(cfg: VerifyConfig, episode: int, parent: np.ndarray,
                       target_token: np.ndarray, spread: int = 8) -> np.ndarray:
    """Draft ids within +-spread bins of a given target token of the parent node.

    `target_token[j]` is whatever the caller takes as the verifier's choice after
    node j (the oracle's argmax in the parity tests, a seeded stand-in in
    accept-only runs).  draft[c] = clip(bin(target[parent[c]]) + delta_c) with
    delta_c uniform in [-spread, spread]."""
    rng = np.random.Generator(np.random.PCG64(seed_for(cfg, episode, 995)))
    delta = rng.integers(-spread, spread + 1, size=cfg.tree_nodes)
    out = np.empty(cfg.tree_nodes, dtype=np.int32)
    out[0] = cfg.action_lo
    for c in range(1, cfg.tree_nodes):
        b = int(target_token[parent[c]]) - cfg.action_lo + int(delta[c])
        out[c] = cfg.action_lo + min(max(b, 0), cfg.n_bins - 1)
    return out


def seeded_target_tokens(cfg: VerifyConfig, episode: int) -> np.ndarray:
    """A stand-in target token per node, uniform over the action tokens."""
    rng = np.random.Generator(np.random.PCG64(seed_for(cfg, episode, 994)))
    return (cfg.action_lo + rng.integers(0, cfg.n_bins, size=cfg.tree_nodes)).astype(np.int32)


def embedding_table(cfg: VerifyConfig) -> torch.Tensor:
    """Token embeddings [vocab, hidden] ~ N(0,1) for the greedy-decoding tests."""
    return _normal((cfg.vocab, cfg.hidden), seed_for(cfg, 0, 993), 0, cfg.torch_dtype)
