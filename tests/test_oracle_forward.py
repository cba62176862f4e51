"""Pins of the oracle's forward pass (CPU only).

The one-pass tree verification of oracle/verify_oracle.py is held against
 (a) per-path sequential decoding written separately (oracle/sequential_decode.py),
 (b) the Llama decoder layer of the `transformers` library (RMSNorm epsilon,
     [out, in] weight layout, rotate-half RoPE, softmax scale, SwiGLU, residuals,
     and - through an explicit mask built here by walking parent links - the tree
     mask and the position rule),
 (c) torch's rms_norm / silu / scaled_dot_product_attention on special cases,
 (d) closed forms (rotation in 2-D, relative-position property, planted argmax).
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import sequential_decode as seq
from oracle import verify_oracle as vo
from paper_2507_22424_amd import workload as wl

TINY = wl.C1.scaled(name="unit", index=7, hidden=32, n_heads=2, head_dim=16, mlp_dim=48,
                    vocab=96, n_bins=64, n_layers=2, prefix_lo=5, prefix_hi=5,
                    tree_nodes=9, max_depth=4, max_children=3, spine_lo=2,
                    n_episodes=3)


def f64(t):
    return t.to(torch.float64).numpy()


def make_inputs(cfg, episode=0):
    layers = [{k: f64(v) for k, v in wl.layer_weights(cfg, l).items()}
              for l in range(cfg.n_layers)]
    P = int(wl.prefix_lengths(cfg)[episode])
    kv = [tuple(f64(t) for t in wl.prefix_kv(cfg, episode, l, P)) for l in range(cfg.n_layers)]
    head = {k: f64(v) for k, v in wl.head_weights(cfg).items()}
    x = f64(wl.hidden_rows(cfg, episode))
    parent = wl.episode_tree(cfg, episode)
    return layers, kv, head, x, parent


def rel_err(a, b):
    return np.max(np.abs(a - b)) / np.max(np.abs(b))


@pytest.mark.parametrize("episode", [0, 1, 2])
def test_tree_pass_equals_per_path_sequential_decoding(episode):
    cfg = TINY
    layers, kv, head, x, parent = make_inputs(cfg, episode)
    one_pass = vo.verify_step(x, layers, kv, head["g_final"], head["w_lm"], cfg.action_lo,
                              parent, cfg.n_heads, cfg.rms_eps, cfg.rope_theta)
    logits, finals = seq.decode_paths(x, layers, kv, head["g_final"], head["w_lm"], parent,
                                      cfg.n_heads, cfg.rms_eps, cfg.rope_theta)
    assert sorted(logits) == list(range(cfg.tree_nodes))
    for node, copies in logits.items():
        for lg in copies:                      # a node shared by paths gets the same logits
            assert rel_err(lg, one_pass["logits"][node]) < 1e-11
        for fx in finals[node]:
            assert rel_err(fx, one_pass["x"][node]) < 1e-11


def test_star_and_chain_trees_against_sequential_decoding():
    cfg = TINY
    layers, kv, head, x, _ = make_inputs(cfg)
    T = cfg.tree_nodes
    for parent in (np.array([-1] + [0] * (T - 1)), np.arange(-1, T - 1)):
        one_pass = vo.verify_step(x, layers, kv, head["g_final"], head["w_lm"], cfg.action_lo,
                                  parent, cfg.n_heads, cfg.rms_eps, cfg.rope_theta)
        logits, _ = seq.decode_paths(x, layers, kv, head["g_final"], head["w_lm"], parent,
                                     cfg.n_heads, cfg.rms_eps, cfg.rope_theta)
        for node, copies in logits.items():
            assert rel_err(copies[0], one_pass["logits"][node]) < 1e-11


def _hf_layer(cfg, w):
    from transformers.models.llama import modeling_llama as m
    hf_cfg = m.LlamaConfig(hidden_size=cfg.hidden, intermediate_size=cfg.mlp_dim,
                           num_attention_heads=cfg.n_heads, num_key_value_heads=cfg.n_heads,
                           num_hidden_layers=1, rms_norm_eps=cfg.rms_eps,
                           rope_theta=cfg.rope_theta, vocab_size=cfg.vocab,
                           attention_bias=False, mlp_bias=False,
                           max_position_embeddings=4096)
    hf_cfg._attn_implementation = "eager"
    layer = m.LlamaDecoderLayer(hf_cfg, 0).double()
    names = {"self_attn.q_proj.weight": "wq", "self_attn.k_proj.weight": "wk",
             "self_attn.v_proj.weight": "wv", "self_attn.o_proj.weight": "wo",
             "mlp.gate_proj.weight": "wg", "mlp.up_proj.weight": "wu",
             "mlp.down_proj.weight": "wd", "input_layernorm.weight": "g1",
             "post_attention_layernorm.weight": "g2"}
    with torch.no_grad():
        for n, p in layer.named_parameters():
            p.copy_(torch.from_numpy(w[names[n]]))
    return layer, m.LlamaRotaryEmbedding(hf_cfg)


@pytest.mark.parametrize("shape", ["chain", "tree"])
def test_layer_matches_transformers_llama_decoder_layer(shape):
    """Run the library's decoder layer over [prefix rows ; tree rows] with an explicit
    additive mask and position ids, and the oracle's layer over the tree rows with the
    prefix keys/values that the library layer's own projections define."""
    cfg = TINY
    layers, _, _, x_tree, parent = make_inputs(cfg)
    w = layers[0]
    T, P, H, nh, d = cfg.tree_nodes, 6, cfg.hidden, cfg.n_heads, cfg.head_dim
    if shape == "chain":
        parent = np.arange(-1, T - 1)
    rng = np.random.default_rng(5)
    x_prefix = rng.standard_normal((P, H))

    # mask and positions by walking the parent links (not via the oracle)
    depth = [0] * T
    allowed = np.zeros((P + T, P + T), dtype=bool)
    for i in range(P):
        allowed[i, :i + 1] = True
    for i in range(T):
        allowed[P + i, :P] = True
        n, steps = i, 0
        while n != -1:
            allowed[P + i, P + n] = True
            n = int(parent[n])
            steps += 1
        depth[i] = steps - 1
    pos = torch.tensor([list(range(P)) + [P + dd for dd in depth]])
    mask = torch.where(torch.from_numpy(allowed), 0.0, -1e30).to(torch.float64)[None, None]

    layer, rotary = _hf_layer(cfg, w)
    xs = torch.from_numpy(np.concatenate([x_prefix, x_tree]))[None]
    cos, sin = rotary(xs, pos)
    with torch.no_grad():
        out = layer(xs, attention_mask=mask, position_ids=pos, position_embeddings=(cos, sin))
    out = (out[0] if isinstance(out, tuple) else out)[0].numpy()

    # prefix keys / values as the cache would hold them: projections of the normed
    # prefix rows, keys rotated at positions 0..P-1 (library's own modules)
    with torch.no_grad():
        xn = layer.input_layernorm(xs[:, :P])
        k = layer.self_attn.k_proj(xn).view(1, P, nh, d).transpose(1, 2)
        v = layer.self_attn.v_proj(xn).view(1, P, nh, d).transpose(1, 2)
        from transformers.models.llama.modeling_llama import apply_rotary_pos_emb
        _, k = apply_rotary_pos_emb(k, k, cos[:, :P], sin[:, :P])
    ours = vo.verify_layer(x_tree, w, k[0].numpy(), v[0].numpy(), parent, nh,
                           cfg.rms_eps, cfg.rope_theta)
    # the library evaluates cos/sin in float32, hence 1e-5 and not 1e-12
    assert rel_err(ours["x"], out[P:]) < 1e-5


def test_rms_norm_and_silu_against_torch():
    rng = np.random.default_rng(0)
    x, g = rng.standard_normal((7, 40)), rng.standard_normal(40)
    ref = F.rms_norm(torch.from_numpy(x), (40,), torch.from_numpy(g), eps=1e-5).numpy()
    assert np.allclose(vo.rms_norm(x, g, 1e-5), ref, rtol=1e-13, atol=1e-13)
    z = rng.standard_normal(100) * 4
    assert np.allclose(vo.silu(z), F.silu(torch.from_numpy(z)).numpy(), rtol=1e-13, atol=1e-15)


def test_root_only_tree_is_one_decode_step_over_the_cache():
    """T = 1: attention is softmax(q K^T / sqrt(d)) V over prefix + self (torch's SDPA)."""
    cfg = TINY
    layers, kv, _, x, _ = make_inputs(cfg)
    w, (kp, vp) = layers[0], kv[0]
    out = vo.verify_layer(x[:1], w, kp, vp, [-1], cfg.n_heads, cfg.rms_eps, cfg.rope_theta)
    q = torch.from_numpy(vo.rope((vo.rms_norm(x[:1], w["g1"], cfg.rms_eps) @ w["wq"].T)
                                 .reshape(1, cfg.n_heads, cfg.head_dim), [kp.shape[1]],
                                 cfg.rope_theta)).transpose(0, 1)            # [nh, 1, d]
    K = torch.from_numpy(np.concatenate([kp, out["k_tree"].transpose(1, 0, 2)], axis=1))
    V = torch.from_numpy(np.concatenate([vp, out["v_tree"].transpose(1, 0, 2)], axis=1))
    ref = F.scaled_dot_product_attention(q[None], K[None], V[None])[0]        # [nh, 1, d]
    assert np.allclose(out["attn"].reshape(cfg.n_heads, cfg.head_dim), ref[:, 0].numpy(),
                       rtol=1e-12, atol=1e-13)


def test_rope_closed_forms():
    # d = 2: a plain rotation by `pos` radians (theta^0 = 1)
    v = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])
    out = vo.rope(v, np.array([3, 3]), 1e4)
    assert np.allclose(out[0, 0], [math.cos(3), math.sin(3)])
    assert np.allclose(out[1, 0], [-math.sin(3), math.cos(3)])
    # d = 4: pair (0,2) turns by pos, pair (1,3) by pos / theta^(1/2)
    v = np.array([[[1.0, 1.0, 0.0, 0.0]]])
    out = vo.rope(v, np.array([2]), 1e4)[0, 0]
    assert np.allclose(out, [math.cos(2), math.cos(0.02), math.sin(2), math.sin(0.02)])
    # position 0 is the identity; norms are kept; scores depend on the offset only
    rng = np.random.default_rng(1)
    q, k = rng.standard_normal((1, 1, 16)), rng.standard_normal((1, 1, 16))
    assert np.allclose(vo.rope(q, [0], 1e4), q)
    assert np.isclose(np.linalg.norm(vo.rope(q, [37], 1e4)), np.linalg.norm(q))
    s1 = np.sum(vo.rope(q, [10], 1e4) * vo.rope(k, [4], 1e4))
    s2 = np.sum(vo.rope(q, [106], 1e4) * vo.rope(k, [100], 1e4))
    assert np.isclose(s1, s2, rtol=1e-10)


def test_tree_structure():
    depth, anc = vo.tree_structure([-1, 0, 0, 1, 3, 2])
    assert depth.tolist() == [0, 1, 1, 2, 3, 2]
    assert anc[4].tolist() == [True, True, False, True, True, False]
    assert anc[5].tolist() == [True, False, True, False, False, True]
    for bad in ([0, 0], [-1, 1], [-1, -1], [-1, 0, 3, 1]):
        with pytest.raises(ValueError):
            vo.tree_structure(bad)


def test_action_head_planted_maximum_and_ties():
    rng = np.random.default_rng(2)
    H, A = 24, 16
    x, g = rng.standard_normal((5, H)), 1 + 0.1 * rng.standard_normal(H)
    w = rng.standard_normal((A, H)) * 0.01
    z = vo.rms_norm(x, g, 1e-5)
    # row 11 is made parallel to node 3's normed state: by Cauchy-Schwarz it wins there
    w[11] = 5.0 * z[3] / np.linalg.norm(z[3]) * np.max(np.linalg.norm(w, axis=1)) * 2
    logits, tok = vo.action_head(x, g, w, 100, 1e-5)
    assert tok[3] == 111
    assert np.allclose(logits, z @ w.T)
    # exact tie between rows 4 and 9: the lower id is taken
    w[9] = w[4] = w[11]
    _, tok = vo.action_head(x, g, w, 100, 1e-5)
    assert tok[3] == 104
