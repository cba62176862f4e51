"""Sequencing of one verification step through the C-ABI calls (no arithmetic here).

`VerifyPass` owns the device buffers of one model + one batch of episodes and issues, per
step,  n_layers x sv_verify_layer -> sv_action_head_argmax -> sv_relaxed_accept  on the
current stream.  Used by the tests, the smoke check and the benchmark.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as sv
from .workload import VerifyConfig


class VerifyPass:
    def __init__(self, wc: VerifyConfig, prefix_len: Sequence[int], parent: np.ndarray,
                 full_vocab: bool = False, device: str = "cuda", extra_capacity: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("VerifyPass needs a GPU; there is no CPU path")
        self.wc = wc
        self.device = device
        self.cfg = sv.model_cfg(wc.dtype, wc.hidden, wc.n_heads, wc.head_dim, wc.mlp_dim,
                                wc.vocab, wc.rms_eps, wc.rope_theta)
        self.B, self.T = wc.n_episodes, wc.tree_nodes
        self.M = self.B * self.T
        self.d_cap = wc.max_depth
        self.vocab_lo = 0 if full_vocab else wc.action_lo
        self.vocab_hi = wc.vocab
        self.n_scored = self.vocab_hi - self.vocab_lo
        self.tree = sv.DeviceTree(parent, self.B, self.T, self.d_cap, device)
        pl = np.asarray(prefix_len, dtype=np.int32)
        self.capacity = int(-(-(int(pl.max()) + self.T + extra_capacity) // 64) * 64)
        self.kv: List[sv.KvCache] = []
        for _ in range(wc.n_layers):       # one prefix-length array for all layers
            self.kv.append(sv.KvCache(self.cfg, self.B, self.capacity, pl, device,
                                      share_prefix_with=self.kv[0] if self.kv else None))
        self.packed: List[Optional[torch.Tensor]] = [None] * wc.n_layers
        self.packed_bytes = sv.sv_packed_layer_bytes(self.cfg)
        self.ws_bytes = sv.sv_workspace_bytes(self.cfg, self.B, self.T, self.n_scored)
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=device)
        sv.sv_workspace_init(self.cfg, self.B, self.T, self.n_scored, self.workspace)
        dt = sv.storage_dtype(self.cfg)
        self.g_final = torch.ones(wc.hidden, dtype=dt, device=device)
        self.w_lm = torch.zeros(wc.vocab, wc.hidden, dtype=dt, device=device)
        # bf16 models score the head on the streaming kernel, from a packed copy of its rows
        self.packed_head: Optional[torch.Tensor] = None
        self.head_packable = self.cfg.dtype != sv.SV_F32 and self.n_scored % 32 == 0
        self.x0 = torch.zeros(self.M, wc.hidden, dtype=torch.float32, device=device)
        self.x = torch.zeros_like(self.x0)
        self.draft = torch.zeros(self.M, dtype=torch.int32, device=device)
        self.token = torch.zeros(self.M, dtype=torch.int32, device=device)
        self.logits = torch.zeros(self.M, self.n_scored, dtype=torch.float32, device=device)
        self.accept_mask = torch.zeros(self.M, dtype=torch.uint8, device=device)
        self.accepted_len = torch.zeros(self.B, dtype=torch.int32, device=device)
        self.best_node = torch.zeros(self.B, dtype=torch.int32, device=device)
        self.path = torch.zeros(self.B, self.d_cap + 1, dtype=torch.int32, device=device)
        self.out_tokens = torch.zeros(self.B, self.d_cap + 1, dtype=torch.int32, device=device)

    # ---- loading -------------------------------------------------------------------
    def load_layer(self, layer: int, raw: Dict[str, torch.Tensor]) -> None:
        """Upload the nine tensors of a layer, pack them, drop the raw copies."""
        dev = {k: v.to(self.device).contiguous() for k, v in raw.items()}
        packed = torch.empty(self.packed_bytes, dtype=torch.uint8, device=self.device)
        if self.cfg.dtype == sv.SV_BF16_W8:
            sv.sv_pack_layer_w8(self.cfg, dev, packed)
        elif self.cfg.dtype == sv.SV_BF16_W4:
            sv.sv_pack_layer_w4(self.cfg, dev, packed)
        else:
            sv.sv_pack_layer(self.cfg, dev, packed)
        torch.cuda.current_stream().synchronize()
        self.packed[layer] = packed

    def load_head(self, g_final: torch.Tensor, w_rows: torch.Tensor) -> None:
        """w_rows: either the full [V, H] head or only the action rows [n_bins, H]."""
        self.g_final.copy_(g_final)
        if w_rows.shape[0] == self.wc.vocab:
            self.w_lm.copy_(w_rows)
        else:
            self.w_lm[self.wc.action_lo:].copy_(w_rows)
        if self.head_packable:
            nb = sv.sv_packed_head_bytes(self.cfg, self.vocab_lo, self.vocab_hi)
            self.packed_head = torch.empty(nb, dtype=torch.uint8, device=self.device)
            sv.sv_pack_head(self.cfg, self.g_final, self.w_lm, self.vocab_lo, self.vocab_hi,
                            self.packed_head)
            torch.cuda.current_stream().synchronize()

    def load_prefix(self, layer: int, episode: int, k: torch.Tensor, v: torch.Tensor) -> None:
        P = k.shape[1]
        self.kv[layer].k[episode, :, :P].copy_(k)
        self.kv[layer].v[episode, :, :P].copy_(v)

    def set_hidden(self, x: torch.Tensor) -> None:
        """x: [B*T, H] in the storage dtype or float32; widened to the float32 stream."""
        self.x0.copy_(x.reshape(self.M, -1).to(torch.float32))

    def set_draft(self, draft: np.ndarray) -> None:
        self.draft.copy_(torch.from_numpy(np.ascontiguousarray(draft, dtype=np.int32).reshape(-1)))

    # ---- one step ------------------------------------------------------------------
    def forward(self, n_layers: Optional[int] = None, want_logits: bool = True,
                route: str = "stack", head: str = "auto") -> None:
        """All layers, then the head.  route: "stack" (one sv_verify_stack call) or "layers" (one
        sv_verify_layer call per layer).  head:
        "packed" (sv_action_head_argmax_packed), "plain" (sv_action_head_argmax on the raw
        rows) or "auto" (packed where a packed head has been loaded)."""
        self.x.copy_(self.x0)
        n = self.wc.n_layers if n_layers is None else n_layers
        views = [kv.struct for kv in self.kv[:n]]
        if route == "layers":
            for l in range(n):
                sv.sv_verify_layer(self.cfg, self.packed[l], self.x, views[l], self.tree.struct,
                                   self.B, self.workspace)
        else:
            sv.sv_verify_stack(self.cfg, self.packed[:n], self.x, views, self.tree.struct, self.B,
                               self.workspace)
        if head == "auto":
            head = "packed" if self.packed_head is not None else "plain"
        if head == "packed":
            if self.packed_head is None:
                raise RuntimeError("no packed head loaded (bf16 model, scored rows a multiple of 32)")
            sv.sv_action_head_argmax_packed(self.cfg, self.packed_head, self.x, self.M,
                                            self.vocab_lo, self.vocab_hi, self.token,
                                            self.logits if want_logits else None, self.workspace)
        else:
            sv.sv_action_head_argmax(self.cfg, self.g_final, self.w_lm, self.x, self.M,
                                     self.vocab_lo, self.vocab_hi, self.token,
                                     self.logits if want_logits else None, self.workspace)

    def accept(self, r: int, target: Optional[torch.Tensor] = None) -> None:
        sv.sv_relaxed_accept(self.tree.struct, self.draft, self.token if target is None else target,
                             self.wc.action_lo, self.wc.n_bins, r, self.B, self.d_cap,
                             self.accept_mask, self.accepted_len, self.best_node, self.path,
                             self.out_tokens)

    def step(self, r: int, want_logits: bool = False, head: str = "auto") -> None:
        self.forward(want_logits=want_logits, head=head)
        self.accept(r)

    def capture_step(self, r: int, want_logits: bool = False, head: str = "auto"):
        """One step (all layers, head, acceptance) recorded into a HIP graph; `replay()` of the
        returned graph reissues it on the current stream.  Every launch of the step reads its
        inputs from this object's buffers (set_hidden, set_draft write into them), so a replay
        sees new inputs; sizes, trees' buffers, prefix bounds and weights are those at capture
        time (capture again after commit() or set_tree()).  Between empty kernels a replayed
        graph turns around in 1.2 us against 2.1 us for launches from the host; the step itself,
        whose kernels run 10-50 us each, takes the same time either way (the host keeps ahead)."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):        # once outside the capture: nothing is set up lazily inside it
            self.step(r, want_logits, head)
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.step(r, want_logits, head)
        return graph

    def set_tree(self, parent: np.ndarray) -> None:
        """New draft trees (same B, T) for the next step."""
        self.tree = sv.DeviceTree(parent, self.B, self.T, self.d_cap, self.device)

    def commit(self) -> None:
        """Make the accepted paths part of the prefix in every layer (outer loop of Alg. 1).
        Refuses when the last pass raised the status word (its results are then undefined) or
        when the cache has no room left for another tree behind the longest possible prefix."""
        st = self.placement_status()
        if st != 0:
            raise RuntimeError(f"verification pass raised status {st}: results undefined, nothing committed")
        # (the status read above has synchronised: the accepted lengths are on hand)
        advance = int(self.accepted_len.max().item()) + 1
        if self.kv[0].struct.prefix_len_max + advance > self.capacity - self.T:
            raise RuntimeError("KV cache full: prefix + accepted path + next tree exceed the capacity "
                               "(construct VerifyPass with a larger extra_capacity)")
        for l in range(self.wc.n_layers):
            sv.sv_commit_path(self.cfg, self.kv[l].struct, self.T, self.path, self.accepted_len,
                              self.B, self.d_cap)
        # all layers share the prefix lengths of layer 0's holder
        sv.sv_advance_prefix(self.kv[0].prefix_len, self.accepted_len, self.B, self.d_cap)
        for l in range(self.wc.n_layers):
            self.kv[l].struct.prefix_len_max = self.kv[l].struct.prefix_len_max + advance

    def placement_status(self) -> int:
        """0 unless a GEMM saw the slices of one tile on different XCDs (see SV_WS_STATUS)."""
        off, nb = sv.sv_workspace_region(self.cfg, self.B, self.T, self.n_scored, sv.SV_WS_STATUS)
        return int(self.workspace[off:off + 4].view(torch.int32).item()) if nb else 0

    def workspace_view(self, which: int) -> torch.Tensor:
        off, nb = sv.sv_workspace_region(self.cfg, self.B, self.T, self.n_scored, which)
        raw = self.workspace[off:off + nb]
        D = self.wc.n_heads * self.wc.head_dim
        return raw.view(torch.float32).reshape(self.M, D)
