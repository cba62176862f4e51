"""Benchmark of one Spec-VLA tree-verification step on one MI355X.

step = sv_verify_stack (32 layers) -> sv_action_head_argmax_packed -> sv_relaxed_accept for the full
7B-shaped configuration (60-node tree, 280-token prefix, bf16 weights), all inputs resident
in HBM.  Prints ONE JSON line: verified tree tokens/s, step latency, the roofline of the
dominant kernel (timed live with HIP events), the CPU oracle timed on the same workload, and
the acceptance rule alone CPU against GPU.
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
MFMA_PEAK_TFLOPS = 2500.0           # dense bf16
# HBM-side bytes per launch of the dominant kernel, from the two rocprofv3 --pmc runs (FETCH_SIZE,
# then WRITE_SIZE, each calibrated with a transfer of known size in the same run) whose summaries
# are under profiles/: fetched + written bytes, averaged over the four products of a layer (for
# the many-row kernels with the split / row-norm / reduction launches that belong to a product).
TRAFFIC_BYTES_PER_LAUNCH = {
    ("C3", "bf16"): 137.02e6,
    ("C3", "w8"): 86.46e6,
    ("C4", "bf16"): 479.19e6,
    ("C5", "bf16"): 185.86e6,
}
TRAFFIC_SOURCE = {
    ("C3", "bf16"): "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, profiles/c3_step_hbm_traffic.txt",
    ("C3", "w8"): "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, profiles/c3_w8_step_hbm_traffic.txt",
    ("C4", "bf16"): "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, profiles/c4_step_hbm_traffic.txt",
    ("C5", "bf16"): "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, profiles/c5_step_hbm_traffic.txt",
}


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


def host_cores():
    """(logical cores the process may run on, threads the BLAS pool behind numpy uses)."""
    from threadpoolctl import threadpool_info
    try:
        nproc = len(os.sched_getaffinity(0))
    except AttributeError:
        nproc = os.cpu_count() or 1
    blas = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return nproc, blas


def cpu_baseline(cfg, wl):
    """The oracle as it stands on the whole step of the same workload, episode 0: every layer,
    head, acceptance (float64 numpy; its matrix products go through numpy's BLAS).  Weights are
    drawn layer by layer outside the timed parts."""
    import torch
    from oracle import verify_oracle as vo
    f64 = lambda t: t.to(torch.float64).numpy()
    P = int(wl.prefix_lengths(cfg)[0])
    parent = wl.episode_tree(cfg, 0)
    x = f64(wl.hidden_rows(cfg, 0))
    head = wl.head_weights(cfg)
    gf, wlm = f64(head["g_final"]), f64(head["w_lm"])
    t_layers = 0.0
    for l in range(cfg.n_layers):
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
    step_s = t_layers + t_tail
    nproc, blas = host_cores()
    return {"value": cfg.tree_nodes / step_s, "unit": "verified tree tokens/s", "cores": blas,
            "kind": "oracle",
            "sample": f"one whole step of episode 0 ({cfg.n_layers} layers + head + accept), float64 "
                      "numpy, matrix products through numpy's BLAS",
            "nproc": nproc, "blas_threads": blas, "step_s": step_s}


def accept_alone(sv, wl, steps=200):
    """sv_relaxed_accept against the oracle's relaxed_accept on 16 trees of 60 nodes (seeded
    target tokens, drafts within +-8 bins, r = 4): microseconds per call for all 16 episodes."""
    import numpy as np
    import torch
    from oracle import verify_oracle as vo
    B, T, dmax, lo, nb, r = 16, 60, 7, 31744, 256, 4
    rng = np.random.default_rng(16060)
    parents = [wl.draft_tree(T, dmax, 4, dmax, rng) for _ in range(B)]
    target = lo + rng.integers(0, nb, size=B * T)
    draft = np.empty(B * T, dtype=np.int64)
    for b in range(B):
        for c in range(T):
            p = max(int(parents[b][c]), 0)
            draft[b * T + c] = np.clip(target[b * T + p] + rng.integers(-8, 9), lo, lo + nb - 1)
    t0 = time.perf_counter()
    reps = 20
    for _ in range(reps):
        ref = [vo.relaxed_accept(parents[b], draft[b * T:(b + 1) * T], target[b * T:(b + 1) * T], lo, nb, r)
               for b in range(B)]
    cpu_us = (time.perf_counter() - t0) / reps * 1e6
    tree = sv.DeviceTree(np.concatenate(parents), B, T, dmax)
    d_t = torch.from_numpy(draft.astype(np.int32)).cuda()
    t_t = torch.from_numpy(target.astype(np.int32)).cuda()
    out = dict(mask=torch.zeros(B * T, dtype=torch.uint8, device="cuda"),
               length=torch.zeros(B, dtype=torch.int32, device="cuda"),
               best=torch.zeros(B, dtype=torch.int32, device="cuda"),
               path=torch.zeros(B, dmax + 1, dtype=torch.int32, device="cuda"),
               tokens=torch.zeros(B, dmax + 1, dtype=torch.int32, device="cuda"))
    call = lambda: sv.sv_relaxed_accept(tree.struct, d_t, t_t, lo, nb, r, B, dmax, out["mask"], out["length"],
                                        out["best"], out["path"], out["tokens"])
    for _ in range(10):
        call()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        call()
    e1.record()
    torch.cuda.synchronize()
    gpu_us = e0.elapsed_time(e1) / steps * 1e3
    same = out["length"].cpu().tolist() == [x["length"] for x in ref]
    return {"episodes": B, "tree_nodes": T, "r": r, "cpu_oracle_us": cpu_us, "gpu_us": gpu_us,
            "lengths_equal": same, "note": "GPU figure is one launch of one workgroup per episode, i.e. launch latency"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--r", type=int, default=4)
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the legs that run the CPU oracle (whole-step baseline, acceptance alone)")
    ap.add_argument("--layers", type=int, default=None, help="debug: fewer layers (invalid as a result)")
    ap.add_argument("--config", choices=("C3", "C4", "C5"), default="C3",
                    help="C3 is the benchmark workload; C4 (16 episodes) and C5 (prefix 2048, 128 "
                         "nodes) are parity configurations that can be timed and profiled the "
                         "same way (no CPU baseline)")
    ap.add_argument("--weights", choices=("bf16", "w8", "w4"), default="bf16",
                    help="w8 / w4: the same workload with 8-bit (E4M3) or 4-bit integer matrices "
                         "(+ a scale per output row), variants of their own: half / a quarter of "
                         "the weight bytes, not the headline configuration")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy (calibrates rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters in the same profile)")
    ap.add_argument("--launch", choices=("stream", "graph"), default="stream",
                    help="issue the timed steps launch by launch from the host (default) or as "
                         "replays of one HIP graph")
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
    w8 = args.weights != "bf16"          # low-precision weight storage (8-bit E4M3 or 4-bit integer codes)
    w4 = args.weights == "w4"
    if w8:
        cfg = cfg.scaled(dtype="bf16_w4" if w4 else "bf16_w8")
    headline = args.config == "C3" and not w8 and args.layers is None
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    B, T, L = cfg.n_episodes, cfg.tree_nodes, cfg.n_layers
    M = B * T
    prefix_len = wl.prefix_lengths(cfg)
    parents = [wl.episode_tree(cfg, b) for b in range(B)]
    vp = VerifyPass(cfg, prefix_len, np.concatenate(parents))

    t0 = time.time()
    with ThreadPoolExecutor(max_workers=8) as ex:
        futs = [ex.submit(wl.layer_weights_w4 if w4 else (wl.layer_weights_w8 if w8 else wl.layer_weights), cfg, l)
                for l in range(L)]
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
    tokens_per_s = M / (dt / args.steps)
    accepted = vp.accepted_len.cpu().tolist()
    accepted_by_r = {}
    for r in cfg.r_values:
        vp.accept(r)
        torch.cuda.synchronize()
        accepted_by_r[str(r)] = vp.accepted_len.cpu().tolist()
    assert vp.placement_status() == 0, "status word raised (see SV_WS_STATUS)"

    # the layers alone, untimed by events, for the split of the step into layers and tail
    views = [kv.struct for kv in vp.kv]
    def layers_only():
        sv.sv_verify_stack(vp.cfg, vp.packed, vp.x, views, vp.tree.struct, B, vp.workspace)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        layers_only()
    e0.record()
    n_lay = max(1, min(args.steps, 20))
    for _ in range(n_lay):
        layers_only()
    e1.record()
    torch.cuda.synchronize()
    layers_ms = e0.elapsed_time(e1) / n_lay

    # per-kernel durations with HIP events around single launches, same stream, same inputs.
    # An event pair costs the stream about 2 us per interval, so the raw figures add up to more
    # than the layers take unobserved; `kernel_ms_per_step` is therefore the raw figures scaled
    # by (layers unobserved) / (their sum) - it adds up to `layers_ms_per_step` - and the raw
    # ones are kept beside it.
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
    raw_ms = {k: v / prof_steps for k, v in acc_ms.items()}
    scale = layers_ms / sum(raw_ms.values())
    per_step_ms = {k: v * scale for k, v in raw_ms.items()}
    H, D, F = cfg.hidden, cfg.n_heads * cfg.head_dim, cfg.mlp_dim
    wb = 0.5 if w4 else (1 if w8 else 2)   # bytes per weight (the row scales of w8 / w4 are 0.1 % more)
    gemm_bytes = {"qkv": 3 * D * H * wb, "o": H * D * wb, "gate_up": 2 * F * H * wb, "down": H * F * wb}
    gemm_flops = {k: 2.0 * M * v / wb for k, v in gemm_bytes.items()}          # algorithmic, per layer
    gemm_ms_raw = sum(raw_ms[k] for k in gemm_bytes)
    gemm_gbs = sum(gemm_bytes.values()) * L / (gemm_ms_raw * 1e-3) / 1e9
    # matrix-core work as issued: every product is done on the hi and on the lo half of the
    # float32 activations (2 x the algorithmic flops), on row tiles padded to 64 (128 for the
    # many-row kernels)
    rows_path = M > 64 and not w8        # what sv_verify_layer routes to the many-row kernels
    m_issue = -(-M // 128) * 128 if rows_path else -(-M // 64) * 64
    issued_flops = 2.0 * sum(gemm_flops.values()) * L * m_issue / M
    mfma_tflops = issued_flops / (gemm_ms_raw * 1e-3) / 1e12
    kv_bytes = sum(2 * cfg.n_heads * (int(p) + T) * cfg.head_dim * 2 for p in prefix_len)   # all episodes, one layer
    weights_total = sum(gemm_bytes.values()) * L
    step_bytes = weights_total + kv_bytes * L + cfg.n_bins * H * 2 + 2 * cfg.n_heads * M * cfg.head_dim * 2 * L
    step_flops = sum(gemm_flops.values()) * L

    mfma_bound = M > 128                 # many rows: the products are bound by the matrix cores
    key = (args.config, args.weights)
    if mfma_bound:
        roofline = {"bound": "mfma", "kernel": "gemm_rows_kernel (4 products per layer, with their split_rows / "
                                               "rows_rstd / rows_reduce_resid launches)",
                    "achieved": mfma_tflops, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": mfma_tflops / MFMA_PEAK_TFLOPS,
                    "traffic": TRAFFIC_BYTES_PER_LAUNCH.get(key),
                    "traffic_source": TRAFFIC_SOURCE.get(key),
                    "flops_counted": "matrix-core flops as issued: hi and lo halves of the activations, rows padded to 128",
                    "algorithmic_frac": step_flops / (gemm_ms_raw * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
                    "flops_per_launch_avg": issued_flops / (4 * L),
                    "avg_launch_us": gemm_ms_raw * 1e3 / (4 * L)}
    else:
        roofline = {"bound": "hbm",
                    "kernel": ("gemm_rows_kernel (4 products per layer, K split across workgroups, with their "
                               "split_rows / rows_rstd / rows_reduce_* launches)" if rows_path else
                               "gemm_stream_bf16 (4 launches per layer: q/k/v, o, gate/up, down)"),
                    "achieved": gemm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": gemm_gbs / HBM_PEAK_GBS,
                    "traffic": TRAFFIC_BYTES_PER_LAUNCH.get(key),
                    "traffic_source": TRAFFIC_SOURCE.get(key),
                    "bytes_per_launch_avg": weights_total / (4 * L),
                    "avg_launch_us": gemm_ms_raw * 1e3 / (4 * L),
                    "timing": "HIP events around single launches (raw; about 2 us per interval above the "
                              "profiler's kernel durations)"}

    out = {
        "metric": "verified tree tokens/sec + step latency (7B-shaped, tree 60); % HBM peak",
        "value": tokens_per_s, "unit": "verified tree tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 (4-bit integer weights)" if w4 else ("bf16 (8-bit E4M3 weights)" if w8 else "bf16"),
        "data": "synthetic",
        "config": {"workload": f"{args.config}: {L}-layer 7B-shaped verify pass + 256-bin action head + "
                               f"relaxed accept (r={args.r}), tree {T} nodes depth 7, prefix "
                               f"{int(prefix_len.min())}" + (f"..{int(prefix_len.max())}" if B > 1 else "") +
                               f", {B} episode" + ("s" if B > 1 else "") + (", 4-bit weights" if w4 else (", 8-bit weights" if w8 else "")),
                   "hidden": H, "layers": L, "tree_nodes": T, "prefix": int(prefix_len[0]),
                   "episodes": B,
                   "launch": "HIP graph replay" if graph is not None else "host launches"},
        "step_hbm_frac": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "step_algorithmic_bytes": step_bytes,
        "step_mfma_frac": 2.0 * step_flops * m_issue / M / (ms_per_step * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
        "mfma_frac": mfma_tflops / MFMA_PEAK_TFLOPS,
        "accepted_len": accepted, "accepted_len_by_r": accepted_by_r,
        "layers_ms_per_step": layers_ms,
        "tail_ms_per_step": ms_per_step - layers_ms,
        "kernel_ms_per_step": per_step_ms,
        "kernel_ms_per_step_event_timed": raw_ms,
        "roofline": roofline,
        # the K/V stream of the tree attention (prefix + tree rows of every head, once per layer)
        "kv_stream": {"bound": "hbm", "kernel": "tree_attention_mfma", "bytes_per_launch": kv_bytes,
                      "avg_launch_us": raw_ms["attn"] * 1e3 / L,
                      "achieved": kv_bytes * L / (raw_ms["attn"] * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                      "unit": "GB/s", "frac": kv_bytes * L / (raw_ms["attn"] * 1e-3) / 1e9 / HBM_PEAK_GBS},
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
    if not mfma_bound:
        out["roofline"]["frac_of_stream_read"] = gemm_gbs / ceiling
    if headline:
        # how often the greedy choice over the WHOLE vocabulary leaves the 256 action tokens
        # (the acceptance rule then rejects): the full head on the packed streaming kernel, once
        full = wl.head_weights(cfg, full_vocab=True)
        nb = sv.sv_packed_head_bytes(vp.cfg, 0, cfg.vocab)
        ph = torch.empty(nb, dtype=torch.uint8, device="cuda")
        gf, wf = full["g_final"].cuda(), full["w_lm"].cuda()
        sv.sv_pack_head(vp.cfg, gf, wf, 0, cfg.vocab, ph)
        ws = torch.empty(sv.sv_workspace_bytes(vp.cfg, B, T, cfg.vocab), dtype=torch.uint8, device="cuda")
        sv.sv_workspace_init(vp.cfg, B, T, cfg.vocab, ws)
        tok_full = torch.zeros(M, dtype=torch.int32, device="cuda")
        sv.sv_action_head_argmax_packed(vp.cfg, ph, vp.x, M, 0, cfg.vocab, tok_full, None, ws)
        torch.cuda.synchronize()
        outside = int((tok_full.cpu().numpy() < cfg.action_lo).sum())
        out["full_vocabulary_argmax"] = {"nodes": M, "outside_action_slice": outside,
                                         "note": "random-init head: with 32000 rows of equal scale the "
                                                 "maximum lies among the 256 action rows with probability 0.8 %"}
        del ph, ws, wf
    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        out["accept_alone"] = accept_alone(sv, wl)
        if args.config == "C3" and not w8:
            out["cpu_baseline"] = cpu_baseline(cfg, wl)
            out["cpu_baseline"]["gpu_speedup"] = tokens_per_s / out["cpu_baseline"]["value"]
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
