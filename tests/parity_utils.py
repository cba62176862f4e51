"""Runs the HIP path and the CPU oracle side by side on the same seeded inputs.

Both sides are fed layer by layer from paper_2507_22424_amd.workload (so a 13 GB model never
has to sit in host memory twice); the oracle gets the stored values widened to float64.
Error measure (per node row): max_k |gpu - ref| / max_k |ref|.
"""
import os
import sys
import time

import numpy as np
import torch

from oracle import fp8_weights as f8
from oracle import int4_weights as i4
from oracle import verify_oracle as vo
from paper_2507_22424_amd import binding as sv
from paper_2507_22424_amd import workload as wl
from paper_2507_22424_amd.runner import VerifyPass


_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
_LOG_DIR = os.path.join(_ROOT, os.environ.get("SV_TEST_LOG_DIR", "gpurun_out"))


def say(msg):
    """Progress / result line: printed (visible with `pytest -s`) and appended to a log file in
    the run's output folder, so that a long GPU test shows signs of life and leaves its measured
    errors behind even when pytest captures the output."""
    print(msg, flush=True)
    try:
        os.makedirs(_LOG_DIR, exist_ok=True)
        with open(os.path.join(_LOG_DIR, "parity.log"), "a") as f:
            f.write(msg + "\n")
    except OSError:
        pass


def f64(t):
    return t.to(torch.float64).numpy()


def row_rel_err(gpu, ref):
    """Per row: max |gpu - ref| / max |ref|.  A NaN or infinity must sit in the same element on
    both sides (asserted); such elements are then left out of the row's maximum."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    bad_gpu, bad_ref = ~np.isfinite(gpu), ~np.isfinite(ref)
    assert np.array_equal(bad_gpu, bad_ref), \
        f"non-finite values differ: {int(bad_gpu.sum())} on the GPU, {int(bad_ref.sum())} in the oracle"
    diff = np.where(bad_ref, 0.0, np.abs(np.where(bad_gpu, 0.0, gpu) - np.where(bad_ref, 0.0, ref)))
    den = np.max(np.where(bad_ref, 0.0, np.abs(ref)), axis=-1)
    return np.max(diff, axis=-1) / den


def worst_row(err):
    """Largest per-row error; a NaN (0 / 0: an all-zero or all-non-finite oracle row) counts as a failure."""
    err = np.asarray(err)
    assert not np.isnan(err).any(), "a row's error is undefined (oracle row is zero or not finite)"
    return float(err.max())


def same_up_to_rounding(a, b, tol=1e-3):
    """NaNs in the same places, and every row within tol of the other's (max |diff| / max |b|)."""
    if not np.array_equal(np.isnan(a), np.isnan(b)):
        return False
    a0, b0 = np.nan_to_num(a), np.nan_to_num(b)
    scale = np.maximum(np.max(np.abs(b0), axis=-1, keepdims=True), 1e-30)
    return bool(np.all(np.abs(a0 - b0) <= tol * scale))


class SideBySide:
    """Outputs of one configuration from both sides."""

    def __init__(self, cfg, n_layers=None, full_vocab=False, per_layer=True, tag="",
                 hidden_transform=None, finite_rows=None, stack_tol=2e-3):
        """hidden_transform(b, rows float32 [T, H]) -> rows: applied to the seeded input rows of
        episode b before either side sees them.  finite_rows: only the first `finite_rows` node
        rows enter the error figures (a test that plants a NaN in a later episode checks those
        rows itself); by default every row does, and a NaN or infinity anywhere must then sit in
        the same element on both sides."""
        self.finite_rows = finite_rows
        L = cfg.n_layers if n_layers is None else n_layers
        self.cfg = cfg = cfg.scaled(n_layers=L)
        B, T = cfg.n_episodes, cfg.tree_nodes
        self.prefix_len = wl.prefix_lengths(cfg)
        self.parents = [wl.episode_tree(cfg, b) for b in range(B)]
        self.gpu = VerifyPass(cfg, self.prefix_len, np.concatenate(self.parents),
                              full_vocab=full_vocab)
        hidden = [wl.hidden_rows(cfg, b) for b in range(B)]
        if hidden_transform is not None:
            hidden = [hidden_transform(b, h.to(torch.float32)) for b, h in enumerate(hidden)]
        self.gpu.set_hidden(torch.cat(hidden))
        self.gpu.x.copy_(self.gpu.x0)
        x_ref = [f64(h) for h in hidden]
        self.attn_err, self.x_err = [], []
        t0 = time.time()
        for l in range(L):
            if cfg.dtype == "bf16_w8":       # 8-bit matrices: the oracle computes on the dequantised ones
                w = wl.layer_weights_w8(cfg, l)
                self.gpu.load_layer(l, w)
                w64 = {k: (f64(v) if k.startswith("g") else
                           f8.dequantise(v.numpy(), w[k + "_scale"].numpy()))
                       for k, v in w.items() if not k.endswith("_scale")}
            elif cfg.dtype == "bf16_w4":     # 4-bit integer matrices: likewise
                w = wl.layer_weights_w4(cfg, l)
                self.gpu.load_layer(l, w)
                w64 = {k: (f64(v) if k.startswith("g") else
                           i4.dequantise(v.numpy(), w[k + "_scale"].numpy()))
                       for k, v in w.items() if not k.endswith("_scale")}
            else:
                w = wl.layer_weights(cfg, l)
                self.gpu.load_layer(l, w)
                w64 = {k: f64(v) for k, v in w.items()}
            del w
            ref_attn = []
            for b in range(B):
                P = int(self.prefix_len[b])
                kp, vp = wl.prefix_kv(cfg, b, l, P)
                self.gpu.load_prefix(l, b, kp, vp)
                out = vo.verify_layer(x_ref[b], w64, f64(kp), f64(vp), self.parents[b],
                                      cfg.n_heads, cfg.rms_eps, cfg.rope_theta)
                x_ref[b] = out["x"]
                ref_attn.append(out["attn"])
            if per_layer:
                sv.sv_verify_layer(self.gpu.cfg, self.gpu.packed[l], self.gpu.x,
                                   self.gpu.kv[l].struct, self.gpu.tree.struct, B,
                                   self.gpu.workspace)
                torch.cuda.synchronize()
                attn = self.gpu.workspace_view(sv.SV_WS_ATTN_OUT).float().cpu().numpy()
                self.attn_err.append(worst_row(row_rel_err(attn[:finite_rows], np.concatenate(ref_attn)[:finite_rows])))
                self.x_err.append(worst_row(row_rel_err(self.gpu.x.cpu().numpy()[:finite_rows],
                                                       np.concatenate(x_ref)[:finite_rows])))
            say(f"[{tag or cfg.name}] layer {l + 1}/{L} done, {time.time() - t0:.0f}s"
                + (f", attn err {self.attn_err[-1]:.2e}, x err {self.x_err[-1]:.2e}"
                   if per_layer else ""))
        x_layer_calls = self.gpu.x.clone() if per_layer else None
        head = wl.head_weights(cfg, full_vocab=full_vocab)
        self.gpu.load_head(head["g_final"], head["w_lm"])
        self.ref_x = np.concatenate(x_ref)
        lo = 0 if full_vocab else cfg.action_lo
        self.ref_logits, self.ref_token = vo.action_head(self.ref_x, f64(head["g_final"]),
                                                         f64(head["w_lm"]), lo, cfg.rms_eps)
        # the whole pass again, in one go, the way the benchmark issues it
        self.gpu.forward(want_logits=True)
        torch.cuda.synchronize()
        self.gpu_logits = self.gpu.logits.cpu().numpy()
        self.gpu_token = self.gpu.token.cpu().numpy()
        self.gpu_x = self.gpu.x.cpu().numpy()
        # sv_verify_layer calls and sv_verify_stack compute the same thing; where both were run
        # they must agree to rounding (the stack call may order its work differently)
        if x_layer_calls is not None:
            assert same_up_to_rounding(self.gpu_x, x_layer_calls.cpu().numpy(), tol=stack_tol), \
                "stack and per-layer routes differ"
        self.logit_err = row_rel_err(self.gpu_logits[:finite_rows], self.ref_logits[:finite_rows])
        worst_row(self.logit_err)
        st = self.gpu.placement_status()
        assert st == 0, (f"status word {st}: bit 0 = K slices of a tile ran on different XCDs, bit 1 = a "
                         "group wait ran out, bit 2 = a wait for the product before ran out")

    def tolerated_ties(self, tol, n_rows=None):
        """Nodes (of the first n_rows; default all) whose GPU token differs from the oracle's:
        (n tolerated, n not tolerated, largest tolerated gap as a fraction of the row's largest
        |logit|).  A difference is tolerated only when it can be explained by the logit error
        that was actually measured on that node: if every GPU logit of the row is within e of the
        oracle's, the first maximum can move only between candidates whose oracle logits differ
        by at most 2 e.  e itself is held to tol * max |logit| by the logit check, so this is
        never looser than "closer than 2 * tol * max |logit|" and usually far tighter."""
        lo = self.gpu.vocab_lo
        ok = bad = 0
        worst_gap = 0.0
        for i in np.flatnonzero((self.gpu_token != self.ref_token)[:n_rows]):
            row = self.ref_logits[i]
            top = np.max(np.abs(row))
            e = np.max(np.abs(self.gpu_logits[i] - row))
            gap = row[self.ref_token[i] - lo] - row[self.gpu_token[i] - lo]
            if gap <= 2 * e and e <= tol * top:
                ok += 1
                worst_gap = max(worst_gap, gap / top)
            else:
                bad += 1
        return ok, bad, worst_gap

    def check_gpu_argmax_of_own_logits(self):
        """The integer decision: the GPU token is the first maximum of the GPU's own logits."""
        lo = self.gpu.vocab_lo
        assert np.array_equal(self.gpu_token, lo + np.argmax(self.gpu_logits, axis=-1))

    def accept_both(self, r, draft, target):
        """sv_relaxed_accept on given target tokens vs the oracle; returns both results."""
        cfg, B, T = self.cfg, self.cfg.n_episodes, self.cfg.tree_nodes
        self.gpu.set_draft(draft)
        tgt = torch.from_numpy(np.ascontiguousarray(target, dtype=np.int32)).cuda()
        self.gpu.accept(r, tgt)
        torch.cuda.synchronize()
        g = {"mask": self.gpu.accept_mask.cpu().numpy().reshape(B, T),
             "length": self.gpu.accepted_len.cpu().numpy(),
             "best": self.gpu.best_node.cpu().numpy(),
             "path": self.gpu.path.cpu().numpy(), "tokens": self.gpu.out_tokens.cpu().numpy()}
        refs = [vo.relaxed_accept(self.parents[b], draft[b * T:(b + 1) * T],
                                  target[b * T:(b + 1) * T], cfg.action_lo, cfg.n_bins, r)
                for b in range(B)]
        return g, refs


def assert_accept_equal(g, refs, d_cap):
    for b, ref in enumerate(refs):
        assert g["mask"][b].astype(bool).tolist() == ref["mask"].tolist()
        assert int(g["length"][b]) == ref["length"]
        assert int(g["best"][b]) == ref["best"]
        pad = [-1] * (d_cap + 1)
        assert g["path"][b].tolist() == (ref["path"] + pad)[:d_cap + 1]
        assert g["tokens"][b].tolist() == (ref["tokens"] + pad)[:d_cap + 1]
