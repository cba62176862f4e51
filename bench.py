"""Benchmark of one Spec-VLA tree-verification step on one MI355X.

step = sv_verify_stack (32 layers) -> sv_action_head_argmax_packed -> sv_relaxed_accept for the full
7B-shaped configuration (60-node tree, 280-token prefix, bf16 weights), all inputs resident
in HBM.  Prints ONE JSON line: verified tree tokens/s, step latency, the HBM roofline of the
dominant kernel (the weight-streaming GEMM, timed live with HIP events) and the CPU oracle
timed on a bounded sample of the same workload.
"""
import argparse
import ctypes as C
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# HBM-side bytes per launch of the dominant kernel (average over the four GEMM launches of a
# layer), from the two rocprofv3 --pmc runs summarised in profiles/c3_step_hbm_traffic.txt:
# fetched (FETCH_SIZE x 2, calibrated with a 1 GiB copy) + written (WRITE_SIZE x 1):
# gate/up 211.7 + 25.3, q/k/v 122.0 + 14.6, down 117.0 + 5.2, output 47.1 + 5.2 (MB).
GEMM_TRAFFIC_BYTES_PER_LAUNCH = (211.68 + 25.30 + 121.97 + 14.64 + 117.04 + 5.20 + 47.08 + 5.20) / 4 * 1e6


def log(msg):
    print(msg, file=sys.stderr, flush=True)


class HipEvents:
    """hipEvent_t handles through the HIP runtime's C API (for sv_verify_layer_timed)."""

    def __init__(self, n):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.arr = (C.c_void_p * n)()
        for i in range(n):
            ev = C.c_void_p()
            assert self.hip.hipEventCreate(C.byref(ev)) == 0
            self.arr[i] = ev.value

    def block(self, first, count):
        return C.cast(C.byref(self.arr, first * C.sizeof(C.c_void_p)), C.c_void_p)

    def elapsed_ms(self, a, b):
        out = C.c_float()
        rc = self.hip.hipEventElapsedTime(C.byref(out), self.arr[a], self.arr[b])
        assert rc == 0, rc
        return out.value


def cpu_baseline(cfg, wl, n_sample_layers=2):
    """The oracle as it stands on a bounded sample: n_sample_layers of the 32 layers of the
    same workload + head + acceptance, scaled to a whole step."""
    import numpy as np
    import torch
    from threadpoolctl import threadpool_info
    from oracle import verify_oracle as vo
    f64 = lambda t: t.to(torch.float64).numpy()
    P = int(wl.prefix_lengths(cfg)[0])
    parent = wl.episode_tree(cfg, 0)
    x = f64(wl.hidden_rows(cfg, 0))
    head = wl.head_weights(cfg)
    gf, wlm = f64(head["g_final"]), f64(head["w_lm"])
    t_layers = 0.0
    for l in range(n_sample_layers):
        w = {k: f64(v) for k, v in wl.layer_weights(cfg, l).items()}
        kp, vp = (f64(t) for t in wl.prefix_kv(cfg, 0, l, P))
        t0 = time.perf_counter()
        x = vo.verify_layer(x, w, kp, vp, parent, cfg.n_heads, cfg.rms_eps, cfg.rope_theta)["x"]
        t_layers += time.perf_counter() - t0
    t0 = time.perf_counter()
    _, tok = vo.action_head(x, gf, wlm, cfg.action_lo, cfg.rms_eps)
    draft = wl.noisy_draft_tokens(cfg, 0, parent, tok)
    vo.relaxed_accept(parent, draft, tok, cfg.action_lo, cfg.n_bins, 4)
    t_tail = time.perf_counter() - t0
    step_s = t_layers / n_sample_layers * cfg.n_layers + t_tail
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": cfg.tree_nodes / step_s, "unit": "verified tree tokens/s", "cores": threads,
            "kind": "oracle",
            "sample": f"{n_sample_layers} of {cfg.n_layers} layers + head + accept of the same "
                      f"workload, float64 numpy; layer time scaled x{cfg.n_layers / n_sample_layers:g}",
            "step_s_extrapolated": step_s}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--r", type=int, default=4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", type=int, default=None, help="debug: fewer layers (invalid as a result)")
    ap.add_argument("--config", choices=("C3", "C4", "C5"), default="C3",
                    help="C3 is the benchmark workload; C4 (16 episodes) and C5 (prefix 2048, 128 "
                         "nodes) are parity configurations that can be timed and profiled the "
                         "same way (no CPU baseline, no stored traffic figure)")
    ap.add_argument("--weights", choices=("bf16", "w8"), default="bf16",
                    help="w8: the same workload with 8-bit (E4M3 + row scale) matrices, a variant "
                         "of its own: half the weight bytes, not the headline configuration")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (calibrates rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters in the same profile)")
    ap.add_argument("--launch", choices=("stream", "graph"), default="stream",
                    help="issue the timed steps launch by launch from the host (default) or as "
                         "replays of one HIP graph (measured: the same step time within 0.2 %%)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures ONE GPU only (the tree-verification pass of one "
                 "MI355X); --gpus must be 1")

    import numpy as np
    import torch
    from paper_2507_22424_amd import binding as sv
    from paper_2507_22424_amd import workload as wl
    from paper_2507_22424_amd.runner import VerifyPass

    base = {"C3": wl.C3, "C4": wl.C4, "C5": wl.C5}[args.config]
    cfg = base if args.layers is None else base.scaled(n_layers=args.layers)
    w8 = args.weights == "w8"
    if w8:
        cfg = cfg.scaled(dtype="bf16_w8")
    if w8 or args.config != "C3":
        args.no_cpu_baseline = True      # the baseline leg times the bf16 benchmark workload
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    B, T, L = cfg.n_episodes, cfg.tree_nodes, cfg.n_layers
    prefix_len = wl.prefix_lengths(cfg)
    parents = [wl.episode_tree(cfg, b) for b in range(B)]
    parent = parents[0]
    vp = VerifyPass(cfg, prefix_len, np.concatenate(parents))

    t0 = time.time()
    with ThreadPoolExecutor(max_workers=8) as ex:
        futs = [ex.submit(wl.layer_weights_w8 if w8 else wl.layer_weights, cfg, l) for l in range(L)]
        for l, f in enumerate(futs):
            vp.load_layer(l, f.result())
            futs[l] = None
            for b in range(B):
                k, v = wl.prefix_kv(cfg, b, l, int(prefix_len[b]))
                vp.load_prefix(l, b, k, v)
            if l % 8 == 7:
                log(f"bench: {l + 1}/{L} layers resident ({time.time() - t0:.0f}s)")
    head = wl.head_weights(cfg)
    vp.load_head(head["g_final"], head["w_lm"])
    vp.set_hidden(torch.cat([wl.hidden_rows(cfg, b) for b in range(B)]))

    # draft ids within +-8 bins of the verifier's own choice (two-phase: one untimed forward)
    vp.forward(want_logits=False)
    torch.cuda.synchronize()
    tok = vp.token.cpu().numpy()
    vp.set_draft(np.concatenate([wl.noisy_draft_tokens(cfg, b, parents[b], tok[b * T:(b + 1) * T])
                                 for b in range(B)]))

    # --launch graph: the step recorded once into a HIP graph and replayed (the same launches in
    # the same order)
    graph = vp.capture_step(args.r) if args.launch == "graph" else None
    one_step = graph.replay if graph is not None else (lambda: vp.step(args.r))
    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    # spread of single steps (torch events on the same stream; one more pass of `steps` steps)
    se = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    for e0, e1 in se:
        e0.record()
        one_step()
        e1.record()
    torch.cuda.synchronize()
    step_ms = sorted(e0.elapsed_time(e1) for e0, e1 in se)
    pct = lambda q: step_ms[min(len(step_ms) - 1, int(q * len(step_ms)))]
    tokens_per_s = B * T / (dt / args.steps)
    accepted = vp.accepted_len.cpu().tolist()
    accepted_by_r = {}
    for r in cfg.r_values:
        vp.accept(r)
        torch.cuda.synchronize()
        accepted_by_r[str(r)] = vp.accepted_len.cpu().tolist()
    assert vp.placement_status() == 0, "GEMM placement check failed (see SV_WS_STATUS)"

    # per-kernel durations with HIP events around single launches, same stream, same inputs
    n_ev = sv.SV_N_TIMING_EVENTS
    evs = HipEvents(n_ev * L)
    prof_steps = max(1, min(args.steps, 10))
    pairs = {"qkv": (0, 1), "attn": (2, 3), "o": (3, 4), "gate_up": (5, 6), "down": (7, 8)}
    acc_ms = {k: 0.0 for k in pairs}
    for _ in range(prof_steps):
        vp.x.copy_(vp.x0)
        for l in range(L):
            sv.sv_verify_layer_timed(vp.cfg, vp.packed[l], vp.x, vp.kv[l].struct, vp.tree.struct,
                                     B, vp.workspace, evs.block(l * n_ev, n_ev))
        torch.cuda.synchronize()
        for l in range(L):
            for k, (a, b) in pairs.items():
                acc_ms[k] += evs.elapsed_ms(l * n_ev + a, l * n_ev + b)
    per_step_ms = {k: v / prof_steps for k, v in acc_ms.items()}
    H, D, F = cfg.hidden, cfg.n_heads * cfg.head_dim, cfg.mlp_dim
    wb = 1 if w8 else 2                  # bytes per weight (the row scales of w8 are 0.1 % more)
    gemm_bytes = {"qkv": 3 * D * H * wb, "o": H * D * wb, "gate_up": 2 * F * H * wb, "down": H * F * wb}
    gemm_ms = sum(per_step_ms[k] for k in gemm_bytes)
    gemm_gbs = sum(gemm_bytes.values()) * L / (gemm_ms * 1e-3) / 1e9
    kv_bytes = sum(2 * cfg.n_heads * (int(p) + T) * cfg.head_dim * 2 for p in prefix_len)   # all episodes, one layer
    weights_total = sum(gemm_bytes.values()) * L
    step_bytes = weights_total + kv_bytes * L + cfg.n_bins * H * 2 + 2 * cfg.n_heads * B * T * cfg.head_dim * 2 * L

    out = {
        "metric": "verified tree tokens/sec + step latency (7B-shaped, tree 60); % HBM peak",
        "value": tokens_per_s, "unit": "verified tree tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 (8-bit E4M3 weights)" if w8 else "bf16",
        "data": "synthetic",
        "config": {"workload": f"{args.config}: {L}-layer 7B-shaped verify pass + 256-bin action head + "
                               f"relaxed accept (r={args.r}), tree {T} nodes depth 7, prefix "
                               f"{int(prefix_len.min())}" + (f"..{int(prefix_len.max())}" if B > 1 else "") +
                               f", {B} episode" + ("s" if B > 1 else "") + (", 8-bit weights" if w8 else ""),
                   "hidden": H, "layers": L, "tree_nodes": T, "prefix": int(prefix_len[0]),
                   "episodes": B,
                   "launch": "HIP graph replay" if graph is not None else "host launches"},
        "step_hbm_frac": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "step_algorithmic_bytes": step_bytes,
        "accepted_len": accepted, "accepted_len_by_r": accepted_by_r,
        "kernel_ms_per_step": per_step_ms,
        "roofline": {"bound": "hbm", "kernel": "gemm_stream_bf16 (4 launches per layer: q/k/v, o, gate/up, down)",
                     "achieved": gemm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": gemm_gbs / HBM_PEAK_GBS,
                     "traffic": None if (w8 or args.config != "C3") else GEMM_TRAFFIC_BYTES_PER_LAUNCH,
                     "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, profiles/c3_step_hbm_traffic.txt",
                     "bytes_per_launch_avg": weights_total / (4 * L),
                     "avg_launch_us": gemm_ms * 1e3 / (4 * L)},
        # the K/V stream of the tree attention (prefix + tree rows of every head, once per layer)
        "kv_stream": {"bound": "hbm", "kernel": "tree_attention_mfma", "bytes_per_launch": kv_bytes,
                      "avg_launch_us": per_step_ms["attn"] * 1e3 / L,
                      "achieved": kv_bytes * L / (per_step_ms["attn"] * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                      "unit": "GB/s", "frac": kv_bytes * L / (per_step_ms["attn"] * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }
    # what a plain streaming read reaches on this GPU (sv_stream_read over 2 GiB, best of 5)
    probe = torch.empty(1 << 31, dtype=torch.uint8, device="cuda").fill_(1)
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    best = float("inf")
    for _ in range(6):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        sv.sv_stream_read(probe, sink)
        e1.record()
        torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1))
    ceiling = probe.numel() / (best * 1e-3) / 1e9
    del probe
    out["step_ms_p10_p50_p90"] = [pct(0.1), pct(0.5), pct(0.9)]
    out["roofline"]["stream_read_measured"] = ceiling
    out["roofline"]["frac_of_stream_read"] = gemm_gbs / ceiling
    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, wl)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
