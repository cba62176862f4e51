"""ctypes binding of libspecvla_verify: same names as include/specvla_verify.h.

Argument marshalling only - every step of the verification pass runs in the HIP kernels of
the library.  PyTorch supplies device memory (tensors) and the stream.  There is no CPU
fallback: if the library has not been built, importing a function from it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence, Tuple

import numpy as np
import torch

from .build import LIB_PATH

SV_F32, SV_BF16, SV_BF16_W8, SV_BF16_W4 = 0, 1, 2, 3
(SV_OK, SV_ERR_NULL, SV_ERR_SHAPE, SV_ERR_TREE, SV_ERR_TOKEN, SV_ERR_WORKSPACE, SV_ERR_DTYPE,
 SV_ERR_LAUNCH) = (0, -1, -2, -3, -4, -5, -6, -7)
SV_MAX_TREE_NODES = 128
SV_MAX_DEPTH = 31
SV_WS_ATTN_OUT, SV_WS_Q, SV_WS_STATUS = 0, 1, 2

EXPORTS = ("sv_version", "sv_strerror", "sv_tree_build_masks", "sv_packed_layer_bytes",
           "sv_pack_layer", "sv_pack_layer_w8", "sv_pack_layer_w4", "sv_workspace_bytes", "sv_workspace_init", "sv_workspace_region",
           "sv_verify_layer",
           "sv_verify_layer_timed", "sv_verify_stack",
           "sv_action_head_argmax", "sv_action_head_argmax_noalloc", "sv_packed_head_bytes", "sv_pack_head",
           "sv_action_head_argmax_packed", "sv_stream_read", "sv_relaxed_accept",
           "sv_commit_path", "sv_advance_prefix", "sv_tree_build_device")
SV_N_TIMING_EVENTS = 9


class SvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {sv_strerror(status)} (status {status})")


class ModelCfg(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("hidden", C.c_int32), ("n_heads", C.c_int32),
                ("head_dim", C.c_int32), ("mlp_dim", C.c_int32), ("vocab", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float)]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")]


class LayerScales(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("sq", "sk", "sv", "so", "sg", "su", "sd")]


class KvView(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("prefix_len", C.c_void_p),
                ("prefix_len_max", C.c_int32), ("capacity", C.c_int32)]


class Tree(C.Structure):
    _fields_ = [("parent", C.c_void_p), ("depth", C.c_void_p), ("anc_mask", C.c_void_p),
                ("n_nodes", C.c_int32), ("n_words", C.c_int32)]


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it was never built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2507_22424_amd.build`"
                               " (or __graft_entry__.build()) first")
        l = C.CDLL(LIB_PATH)
        l.sv_version.restype = C.c_char_p
        l.sv_strerror.restype = C.c_char_p
        l.sv_strerror.argtypes = [C.c_int]
        l.sv_tree_build_masks.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        l.sv_packed_layer_bytes.argtypes = [C.POINTER(ModelCfg), C.POINTER(C.c_size_t)]
        l.sv_pack_layer.argtypes = [C.POINTER(ModelCfg), C.POINTER(LayerWeights), C.c_void_p,
                                    C.c_size_t, C.c_void_p]
        l.sv_pack_layer_w8.argtypes = [C.POINTER(ModelCfg), C.POINTER(LayerWeights),
                                       C.POINTER(LayerScales), C.c_void_p, C.c_size_t, C.c_void_p]
        l.sv_pack_layer_w4.argtypes = l.sv_pack_layer_w8.argtypes
        l.sv_workspace_bytes.argtypes = [C.POINTER(ModelCfg), C.c_int, C.c_int, C.c_int,
                                         C.POINTER(C.c_size_t)]
        l.sv_workspace_init.argtypes = [C.POINTER(ModelCfg), C.c_int, C.c_int, C.c_int, C.c_void_p,
                                        C.c_size_t, C.c_void_p]
        l.sv_workspace_region.argtypes = [C.POINTER(ModelCfg), C.c_int, C.c_int, C.c_int, C.c_int,
                                          C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        l.sv_verify_layer.argtypes = [C.POINTER(ModelCfg), C.c_void_p, C.c_void_p,
                                      C.POINTER(KvView), C.POINTER(Tree), C.c_int, C.c_void_p,
                                      C.c_size_t, C.c_void_p]
        l.sv_verify_layer_timed.argtypes = l.sv_verify_layer.argtypes + [C.c_void_p]
        l.sv_verify_stack.argtypes = [C.POINTER(ModelCfg), C.c_int, C.POINTER(C.c_void_p), C.c_void_p,
                                      C.POINTER(KvView), C.POINTER(Tree), C.c_int, C.c_void_p,
                                      C.c_size_t, C.c_void_p]
        l.sv_action_head_argmax.argtypes = [C.POINTER(ModelCfg), C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_size_t, C.c_void_p]
        l.sv_action_head_argmax_noalloc.argtypes = [C.POINTER(ModelCfg), C.c_void_p, C.c_void_p,
                                                    C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                                    C.c_void_p, C.c_void_p]
        l.sv_packed_head_bytes.argtypes = [C.POINTER(ModelCfg), C.c_int, C.c_int, C.POINTER(C.c_size_t)]
        l.sv_pack_head.argtypes = [C.POINTER(ModelCfg), C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                   C.c_void_p, C.c_size_t, C.c_void_p]
        l.sv_action_head_argmax_packed.argtypes = [C.POINTER(ModelCfg), C.c_void_p, C.c_void_p, C.c_int,
                                                   C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                                   C.c_size_t, C.c_void_p]
        l.sv_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        l.sv_relaxed_accept.argtypes = [C.POINTER(Tree), C.c_void_p, C.c_void_p, C.c_int, C.c_int,
                                        C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        l.sv_commit_path.argtypes = [C.POINTER(ModelCfg), C.POINTER(KvView), C.c_int, C.c_void_p,
                                     C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        l.sv_advance_prefix.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        l.sv_tree_build_device.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p,
                                           C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib = l
    return _lib


def _check(status: int, where: str) -> None:
    if status != 0:
        raise SvError(status, where)


def _dev(t: Optional[torch.Tensor], dtype=None, name="tensor") -> int:
    """Device pointer of a contiguous CUDA tensor (0 for None)."""
    if t is None:
        return 0
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def model_cfg(dtype: str, hidden: int, n_heads: int, head_dim: int, mlp_dim: int, vocab: int,
              rms_eps: float = 1e-5, rope_theta: float = 1e4) -> ModelCfg:
    code = {"f32": SV_F32, "bf16": SV_BF16, "bf16_w8": SV_BF16_W8, "bf16_w4": SV_BF16_W4}.get(dtype, dtype)
    return ModelCfg(int(code), hidden, n_heads, head_dim, mlp_dim, vocab, rms_eps, rope_theta)


def storage_dtype(cfg: ModelCfg) -> torch.dtype:
    return torch.float32 if cfg.dtype == SV_F32 else torch.bfloat16


# ---- the calls of include/specvla_verify.h -------------------------------------------

def sv_version() -> str:
    return lib().sv_version().decode()


def sv_strerror(status: int) -> str:
    return lib().sv_strerror(int(status)).decode()


def sv_tree_build_masks(parent: np.ndarray, B: int, T: int, d_cap: int
                        ) -> Tuple[np.ndarray, np.ndarray]:
    """Host: depth int32[B*T] and ancestor masks uint64[B*T*ceil(T/64)] of B parent arrays."""
    parent = np.ascontiguousarray(parent, dtype=np.int32).reshape(-1)
    if parent.size != B * T:
        raise ValueError("parent must hold B*T entries")
    W = (T + 63) // 64
    depth = np.zeros(B * T, dtype=np.int32)
    anc = np.zeros(B * T * max(W, 1), dtype=np.uint64)
    _check(lib().sv_tree_build_masks(parent.ctypes.data, B, T, d_cap, depth.ctypes.data,
                                     anc.ctypes.data), "sv_tree_build_masks")
    return depth, anc


def sv_packed_layer_bytes(cfg: ModelCfg) -> int:
    out = C.c_size_t(0)
    _check(lib().sv_packed_layer_bytes(C.byref(cfg), C.byref(out)), "sv_packed_layer_bytes")
    return out.value


def sv_pack_layer(cfg: ModelCfg, raw: Dict[str, torch.Tensor], packed: torch.Tensor,
                  stream=None) -> None:
    dt = storage_dtype(cfg)
    w = LayerWeights(*[_dev(raw[n], dt, n) for n, _ in LayerWeights._fields_])
    _check(lib().sv_pack_layer(C.byref(cfg), C.byref(w), _dev(packed, torch.uint8, "packed"),
                               packed.numel(), _stream(stream)), "sv_pack_layer")


def sv_pack_layer_w8(cfg: ModelCfg, raw: Dict[str, torch.Tensor], packed: torch.Tensor,
                     stream=None) -> None:
    """raw: gains g1, g2 (bf16), codes wq .. wd (uint8 E4M3) and row scales wq_scale .. wd_scale
    (float32)."""
    w = LayerWeights(*[_dev(raw[n], torch.bfloat16 if n.startswith("g") else torch.uint8, n)
                       for n, _ in LayerWeights._fields_])
    sc = LayerScales(*[_dev(raw["w" + n[1] + "_scale"], torch.float32, n) for n, _ in LayerScales._fields_])
    _check(lib().sv_pack_layer_w8(C.byref(cfg), C.byref(w), C.byref(sc),
                                  _dev(packed, torch.uint8, "packed"), packed.numel(),
                                  _stream(stream)), "sv_pack_layer_w8")


def sv_pack_layer_w4(cfg: ModelCfg, raw: Dict[str, torch.Tensor], packed: torch.Tensor,
                     stream=None) -> None:
    """raw: gains g1, g2 (bf16), int4 codes wq .. wd (uint8 [out, in / 2], two codes per byte, even
    k in the low four bits) and row scales wq_scale .. wd_scale (float32)."""
    w = LayerWeights(*[_dev(raw[n], torch.bfloat16 if n.startswith("g") else torch.uint8, n)
                       for n, _ in LayerWeights._fields_])
    sc = LayerScales(*[_dev(raw["w" + n[1] + "_scale"], torch.float32, n) for n, _ in LayerScales._fields_])
    _check(lib().sv_pack_layer_w4(C.byref(cfg), C.byref(w), C.byref(sc),
                                  _dev(packed, torch.uint8, "packed"), packed.numel(),
                                  _stream(stream)), "sv_pack_layer_w4")


def sv_workspace_bytes(cfg: ModelCfg, B: int, T: int, n_scored: int) -> int:
    out = C.c_size_t(0)
    _check(lib().sv_workspace_bytes(C.byref(cfg), B, T, n_scored, C.byref(out)),
           "sv_workspace_bytes")
    return out.value


def sv_workspace_init(cfg: ModelCfg, B: int, T: int, n_scored: int, workspace: torch.Tensor,
                      stream=None) -> None:
    _check(lib().sv_workspace_init(C.byref(cfg), B, T, n_scored,
                                   _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
                                   _stream(stream)), "sv_workspace_init")


def sv_workspace_region(cfg: ModelCfg, B: int, T: int, n_scored: int, which: int
                        ) -> Tuple[int, int]:
    off, nb = C.c_size_t(0), C.c_size_t(0)
    _check(lib().sv_workspace_region(C.byref(cfg), B, T, n_scored, which, C.byref(off),
                                     C.byref(nb)), "sv_workspace_region")
    return off.value, nb.value


def sv_verify_layer(cfg: ModelCfg, packed: torch.Tensor, x: torch.Tensor, kv: KvView,
                    tree: Tree, B: int, workspace: torch.Tensor, stream=None) -> None:
    if x.numel() != B * tree.n_nodes * cfg.hidden:
        raise ValueError("x must be [B*T, hidden]")
    _check(lib().sv_verify_layer(C.byref(cfg), _dev(packed, torch.uint8, "packed"),
                                 _dev(x, torch.float32, "x"), C.byref(kv), C.byref(tree), B,
                                 _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
                                 _stream(stream)), "sv_verify_layer")


def sv_verify_layer_timed(cfg: ModelCfg, packed: torch.Tensor, x: torch.Tensor, kv: KvView,
                          tree: Tree, B: int, workspace: torch.Tensor, events, stream=None) -> None:
    """`events`: ctypes array (c_void_p * SV_N_TIMING_EVENTS) of hipEvent_t handles."""
    _check(lib().sv_verify_layer_timed(C.byref(cfg), _dev(packed, torch.uint8, "packed"),
                                       _dev(x, torch.float32, "x"), C.byref(kv), C.byref(tree), B,
                                       _dev(workspace, torch.uint8, "workspace"),
                                       workspace.numel(), _stream(stream),
                                       C.cast(events, C.c_void_p)), "sv_verify_layer_timed")


def _stack_arrays(packed: Sequence[torch.Tensor], kv: Sequence[KvView]):
    n = len(packed)
    if n < 1 or len(kv) != n:
        raise ValueError("verify_stack: one packed blob and one KV view per layer")
    ptrs = (C.c_void_p * n)(*[_dev(p, torch.uint8, "packed") for p in packed])
    views = (KvView * n)(*kv)
    return n, ptrs, views


def sv_verify_stack(cfg: ModelCfg, packed: Sequence[torch.Tensor], x: torch.Tensor,
                    kv: Sequence[KvView], tree: Tree, B: int, workspace: torch.Tensor,
                    stream=None) -> None:
    n, ptrs, views = _stack_arrays(packed, kv)
    _check(lib().sv_verify_stack(C.byref(cfg), n, ptrs, _dev(x, torch.float32, "x"), views,
                                 C.byref(tree), B, _dev(workspace, torch.uint8, "workspace"),
                                 workspace.numel(), _stream(stream)), "sv_verify_stack")


def sv_action_head_argmax(cfg: ModelCfg, g_final: torch.Tensor, w_lm: torch.Tensor,
                          x: torch.Tensor, n_rows: int, vocab_lo: int, vocab_hi: int,
                          out_token: torch.Tensor, out_logits: Optional[torch.Tensor],
                          workspace: torch.Tensor, stream=None) -> None:
    dt = storage_dtype(cfg)
    if w_lm.numel() != cfg.vocab * cfg.hidden or x.numel() < n_rows * cfg.hidden:
        raise ValueError("w_lm must be [vocab, hidden] and x [n_rows, hidden]")
    if out_token.numel() < n_rows or (out_logits is not None and
                                      out_logits.numel() < n_rows * (vocab_hi - vocab_lo)):
        raise ValueError("output tensors too small")
    _check(lib().sv_action_head_argmax(
        C.byref(cfg), _dev(g_final, dt, "g_final"), _dev(w_lm, dt, "w_lm"),
        _dev(x, torch.float32, "x"), n_rows, vocab_lo, vocab_hi,
        _dev(out_token, torch.int32, "out_token"), _dev(out_logits, torch.float32, "out_logits"),
        _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream(stream)),
        "sv_action_head_argmax")


def sv_action_head_argmax_noalloc(cfg: ModelCfg, g_final: torch.Tensor, w_lm: torch.Tensor,
                                  x: torch.Tensor, n_rows: int, vocab_lo: int, vocab_hi: int,
                                  out_token: torch.Tensor, out_logits: Optional[torch.Tensor],
                                  stream=None) -> None:
    dt = storage_dtype(cfg)
    if w_lm.numel() != cfg.vocab * cfg.hidden or x.numel() < n_rows * cfg.hidden:
        raise ValueError("w_lm must be [vocab, hidden] and x [n_rows, hidden]")
    if out_token.numel() < n_rows or (out_logits is not None and
                                      out_logits.numel() < n_rows * (vocab_hi - vocab_lo)):
        raise ValueError("output tensors too small")
    _check(lib().sv_action_head_argmax_noalloc(
        C.byref(cfg), _dev(g_final, dt, "g_final"), _dev(w_lm, dt, "w_lm"),
        _dev(x, torch.float32, "x"), n_rows, vocab_lo, vocab_hi,
        _dev(out_token, torch.int32, "out_token"), _dev(out_logits, torch.float32, "out_logits"),
        _stream(stream)), "sv_action_head_argmax_noalloc")


def sv_packed_head_bytes(cfg: ModelCfg, vocab_lo: int, vocab_hi: int) -> int:
    out = C.c_size_t(0)
    _check(lib().sv_packed_head_bytes(C.byref(cfg), vocab_lo, vocab_hi, C.byref(out)),
           "sv_packed_head_bytes")
    return out.value


def sv_pack_head(cfg: ModelCfg, g_final: torch.Tensor, w_lm: torch.Tensor, vocab_lo: int,
                 vocab_hi: int, packed: torch.Tensor, stream=None) -> None:
    if w_lm.numel() != cfg.vocab * cfg.hidden or g_final.numel() != cfg.hidden:
        raise ValueError("w_lm must be [vocab, hidden] and g_final [hidden]")
    _check(lib().sv_pack_head(
        C.byref(cfg), _dev(g_final, torch.bfloat16, "g_final"), _dev(w_lm, torch.bfloat16, "w_lm"),
        vocab_lo, vocab_hi, _dev(packed, torch.uint8, "packed"), packed.numel(), _stream(stream)),
        "sv_pack_head")


def sv_action_head_argmax_packed(cfg: ModelCfg, packed_head: torch.Tensor, x: torch.Tensor,
                                 n_rows: int, vocab_lo: int, vocab_hi: int,
                                 out_token: torch.Tensor, out_logits: Optional[torch.Tensor],
                                 workspace: torch.Tensor, stream=None) -> None:
    if x.numel() < n_rows * cfg.hidden:
        raise ValueError("x must be [n_rows, hidden]")
    if out_token.numel() < n_rows or (out_logits is not None and
                                      out_logits.numel() < n_rows * (vocab_hi - vocab_lo)):
        raise ValueError("output tensors too small")
    _check(lib().sv_action_head_argmax_packed(
        C.byref(cfg), _dev(packed_head, torch.uint8, "packed_head"), _dev(x, torch.float32, "x"),
        n_rows, vocab_lo, vocab_hi, _dev(out_token, torch.int32, "out_token"),
        _dev(out_logits, torch.float32, "out_logits"), _dev(workspace, torch.uint8, "workspace"),
        workspace.numel(), _stream(stream)), "sv_action_head_argmax_packed")


def sv_stream_read(buf: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    """Measurement aid: one streaming read of `buf` (any dtype, contiguous, on the device)."""
    if not buf.is_cuda or not buf.is_contiguous():
        raise ValueError("buf must be a contiguous device tensor")
    _check(lib().sv_stream_read(buf.data_ptr(), buf.numel() * buf.element_size(),
                                _dev(sink, torch.uint8, "sink"), _stream(stream)), "sv_stream_read")


def sv_relaxed_accept(tree: Tree, draft_token: torch.Tensor, target_token: torch.Tensor,
                      action_lo: int, n_bins: int, r: int, B: int, d_cap: int,
                      accept_mask: torch.Tensor, accepted_len: torch.Tensor,
                      best_node: torch.Tensor, path: torch.Tensor, out_tokens: torch.Tensor,
                      stream=None) -> None:
    T = tree.n_nodes
    if draft_token.numel() != B * T or target_token.numel() != B * T or \
            accept_mask.numel() != B * T or accepted_len.numel() != B or \
            best_node.numel() != B or path.numel() != B * (d_cap + 1) or \
            out_tokens.numel() != B * (d_cap + 1):
        raise ValueError("relaxed_accept: tensor sizes do not match B, T, d_cap")
    _check(lib().sv_relaxed_accept(
        C.byref(tree), _dev(draft_token, torch.int32, "draft_token"),
        _dev(target_token, torch.int32, "target_token"), action_lo, n_bins, r, B, d_cap,
        _dev(accept_mask, torch.uint8, "accept_mask"), _dev(accepted_len, torch.int32, "accepted_len"),
        _dev(best_node, torch.int32, "best_node"), _dev(path, torch.int32, "path"),
        _dev(out_tokens, torch.int32, "out_tokens"), _stream(stream)), "sv_relaxed_accept")


def sv_commit_path(cfg: ModelCfg, kv: KvView, T: int, path: torch.Tensor,
                   accepted_len: torch.Tensor, B: int, d_cap: int, stream=None) -> None:
    if path.numel() != B * (d_cap + 1) or accepted_len.numel() != B:
        raise ValueError("commit_path: tensor sizes do not match B, d_cap")
    _check(lib().sv_commit_path(C.byref(cfg), C.byref(kv), T, _dev(path, torch.int32, "path"),
                                _dev(accepted_len, torch.int32, "accepted_len"), B, d_cap,
                                _stream(stream)), "sv_commit_path")


def sv_advance_prefix(prefix_len: torch.Tensor, accepted_len: torch.Tensor, B: int, d_cap: int,
                      stream=None) -> None:
    _check(lib().sv_advance_prefix(_dev(prefix_len, torch.int32, "prefix_len"),
                                   _dev(accepted_len, torch.int32, "accepted_len"), B, d_cap,
                                   _stream(stream)), "sv_advance_prefix")


def sv_tree_build_device(cand_parent: torch.Tensor, cand_logp: torch.Tensor, cand_token: torch.Tensor,
                         root_token: torch.Tensor, B: int, T: int, d_cap: int, parent: torch.Tensor,
                         depth: torch.Tensor, anc_mask: torch.Tensor, draft_token: torch.Tensor,
                         status: torch.Tensor, stream=None) -> None:
    n_cand = cand_parent.numel() // B
    W = (T + 63) // 64
    if (cand_parent.numel() != B * n_cand or cand_logp.numel() != B * n_cand or
            cand_token.numel() != B * n_cand or root_token.numel() != B or parent.numel() != B * T or
            depth.numel() != B * T or draft_token.numel() != B * T or anc_mask.numel() != B * T * W or
            status.numel() != B):
        raise ValueError("tree_build_device: tensor sizes do not match B, T, n_cand")
    _check(lib().sv_tree_build_device(
        _dev(cand_parent, torch.int32, "cand_parent"), _dev(cand_logp, torch.float32, "cand_logp"),
        _dev(cand_token, torch.int32, "cand_token"), n_cand, _dev(root_token, torch.int32, "root_token"),
        B, T, d_cap, _dev(parent, torch.int32, "parent"), _dev(depth, torch.int32, "depth"),
        _dev(anc_mask, torch.int64, "anc_mask"), _dev(draft_token, torch.int32, "draft_token"),
        _dev(status, torch.int32, "status"), _stream(stream)), "sv_tree_build_device")


# ---- holders that keep the device tensors behind the C structs alive -------------------

class DeviceTree:
    """B trees on the device: builds depth / masks with sv_tree_build_masks and uploads."""

    def __init__(self, parent: np.ndarray, B: int, T: int, d_cap: int, device="cuda"):
        parent = np.ascontiguousarray(parent, dtype=np.int32).reshape(-1)
        depth, anc = sv_tree_build_masks(parent, B, T, d_cap)
        self.B, self.T, self.d_cap = B, T, d_cap
        self.host_parent, self.host_depth, self.host_anc = parent, depth, anc
        self.parent = torch.from_numpy(parent).to(device)
        self.depth = torch.from_numpy(depth).to(device)
        self.anc = torch.from_numpy(anc.view(np.int64)).to(device)
        self.struct = Tree(self.parent.data_ptr(), self.depth.data_ptr(), self.anc.data_ptr(),
                           T, (T + 63) // 64)


class KvCache:
    """KV cache of one layer, [B, n_heads, capacity, head_dim], prefix rows filled by the caller."""

    def __init__(self, cfg: ModelCfg, B: int, capacity: int, prefix_len: Sequence[int],
                 device="cuda", share_prefix_with: Optional["KvCache"] = None):
        dt = storage_dtype(cfg)
        self.k = torch.zeros(B, cfg.n_heads, capacity, cfg.head_dim, dtype=dt, device=device)
        self.v = torch.zeros_like(self.k)
        pl = np.ascontiguousarray(prefix_len, dtype=np.int32)
        # the layers of one model have the same prefix lengths: one device array can serve all
        self.prefix_len = (share_prefix_with.prefix_len if share_prefix_with is not None
                           else torch.from_numpy(pl).to(device))
        self.struct = KvView(self.k.data_ptr(), self.v.data_ptr(), self.prefix_len.data_ptr(),
                             int(pl.max()), capacity)
