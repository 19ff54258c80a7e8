#!/usr/bin/env python3
"""Benchmark of the hybrid decode-attention layer-step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--layers L] [--streams 1|2] [--no-cpu]

Protocol: --reps repetitions (default 5) of (--warmup untimed steps, then exactly --steps timed steps); the
line reports the median repetition, with the minimum and maximum beside it.

A step is one pass of the whole hot path over one batch: dense window attention,
salient selection, sparse attention and log-sum-exp merge on the 8B-shape 32K-context
workload (C2: bf16, B=8, Hq=32, Hkv=8, d=128, window 4096, pool 28672, k=2048) with
seeded synthetic K/V already resident in HBM.  Steps cycle over L independently drawn
layers so that consecutive steps do not re-read K/V still held in L2 / Infinity Cache.
Prints ONE JSON line.

`value` is the full step (selection every step) as ONE call of hgca_hybrid_decode_step: score pass over
the pool, per-head top-k, one launch for the window's split kernels and the gather of the kept entries' V
rows, one fold of all split partials.  `separate_calls_deferred` is the same work as five kernels through
hgca_dense_window_attn (result deferred), hgca_select_salient, hgca_sparse_attn (result deferred)
and hgca_lse_merge_splits; `four_calls` is the step with each part folding its own splits and
hgca_lse_merge joining them.  In all of them the selection hands the scores of
the kept entries to the sparse part, which therefore re-reads only V of those entries;
`algorithmic_bytes_per_step` keeps counting their K rows (the definition of the metric),
`moved_bytes_per_step` does not.  The `steady` step reuses a selection, as the paper's decode
branch does, and gathers K and V (ONE call of hgca_hybrid_decode_step_selected).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
METRIC = "hybrid decode-attn layer-steps/s + achieved HBM GB/s vs peak (8B shape, 32K)"

TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "c2_step_hbm_traffic.md")


def measured_traffic(kernel: str):
    """HBM bytes per launch of `kernel` from the tracked rocprofv3 --pmc summary (FETCH_SIZE / WRITE_SIZE scaled by
    the same counters on a copy of known size): its `total MB` column, and the commit the summary was measured at.
    (None, None) if the summary does not list the kernel."""
    try:
        text = open(TRAFFIC_PROFILE).read()
    except OSError:
        return None, None
    import re
    at = re.search(r"measured at commit `?([0-9a-f]{7,40})`?", text, re.I)
    for line in text.splitlines():
        cells = [c.strip() for c in line.split("|")]
        if len(cells) > 6 and cells[1].strip("`").startswith(kernel):
            return int(round(float(cells[6]) * 1e6)), (at.group(1) if at else None)
    return None, None


WORKLOADS = {
    "C2": "C2: Llama-3-8B-like layer, bf16, B=8, Hq=32, Hkv=8, d=128, ctx 32768 (window 4096 + pool 28672), "
          "per-head top-k 2048",
    "C3": "C3: OPT-13B-like MHA layer, bf16, B=32, Hq=Hkv=40, d=128, ctx 16384 (window 2048 + pool 14336), "
          "per-head top-k 1024",
    "C4": "C4: Llama-3-70B-like layer, bf16, B=4, Hq=64, Hkv=8, d=128, ctx 131072 (window 8192 + pool 122880), "
          "per-head top-k 4096",
    "C5": "C5: ragged large batch, bf16, B=64, Hq=32, Hkv=8, d=128, lengths U[2048,16384], window 2048, "
          "top-k 10 % of the pool, both tiers in 16-token pages",
}


def log(msg: str) -> None:
    print(msg, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--reps", type=int, default=5,
                    help="repetitions of (warm-up, timed steps); the line reports their median, min and max")
    ap.add_argument("--spin-up", type=float, default=0.5,
                    help="seconds of untimed steps before the first repetition: the figures are those of a device that "
                         "is already serving (clocks and power state settled), as in a decode loop; 0 disables it")
    ap.add_argument("--layers", type=int, default=4, help="independent KV draws cycled through")
    ap.add_argument("--config", default="C2", choices=("C2", "C3", "C4", "C5"),
                    help="workload; C2 is the one the metric is quoted on (the others are for comparison)")
    ap.add_argument("--streams", type=int, default=1, choices=(1, 2),
                    help="2: the dense window part runs on a second stream beside select+sparse")
    ap.add_argument("--four-calls", action="store_true",
                    help="headline = the step with per-part outputs and hgca_lse_merge (no deferred results)")
    ap.add_argument("--no-pass-scores", action="store_true",
                    help="sparse part recomputes its scores from K even right after a selection")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-decode-loop", action="store_true",
                    help="skip the extra timing of the paper-literal decode loop (KV manager + moving averages)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU work of the baseline sample")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run plain device copies of known size (reference for the HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2507_03153_amd import hgca, runner, workloads as wl

    hgca.lib()                                                  # no fallback: fails loudly if not built
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = "cuda:0"
    if args.copy_calibration:
        return copy_calibration(torch, dev)

    cfg = wl.CONFIGS[args.config]
    w_lens, p_lens, k = wl.seq_lengths(cfg)
    nbytes = wl.step_bytes(cfg, w_lens, p_lens, k)
    k_sum = int(np.minimum(np.full(cfg.B, k) if np.isscalar(k) else k, p_lens).sum())   # kept entries per head
    k_gather = nbytes["sparse"] - 4 * cfg.Hq * k_sum            # K+V rows of the kept entries
    pass_scores = not args.no_pass_scores
    moved_full = nbytes["full"] - (k_gather // 2 if pass_scores else 0)

    t0 = time.time()
    host_layers = [wl.make_layer(cfg, layer) for layer in range(args.layers)]
    layers = [runner.DeviceLayer.upload(L, dev) for L in host_layers]
    log(f"[bench] {args.layers} layers of {cfg.name} generated and uploaded in {time.time() - t0:.1f}s "
        f"({sum(L.kv_bytes() for L in host_layers) / 2**30:.2f} GiB of KV)")
    main_stream = torch.cuda.current_stream()
    k_max = layers[0].k_max
    steps_by_tail = {fused: runner.HybridStep(layers[0].shape, cfg.W, cfg.P, k_max, dev,
                                              two_streams=(args.streams == 2), pass_scores=pass_scores,
                                              fused_tail=fused) for fused in (True, False)}
    prepared_by_tail = {fused: [st.prepare(L) for L in layers] for fused, st in steps_by_tail.items()}
    step = steps_by_tail[False]                                 # buffers used by the per-call timings below

    def timed(fused, select: bool) -> dict:
        """args.reps repetitions of (args.warmup untimed steps, then exactly args.steps timed steps between two events
        on the launch stream, bracketed by device synchronisations); a step's time is the larger of the device and the
        wall-clock figure (host-side launch cost counts too).  Median, min and max over the repetitions."""
        prepared = prepared_by_tail[fused]                      # arguments marshalled once per layer

        def run_steps(n: int, first: int = 0) -> None:
            for i in range(n):
                prepared[(first + i) % len(prepared)](select)

        per_rep, dev_rep, wall_rep = [], [], []
        for _ in range(max(1, args.reps)):
            run_steps(args.warmup)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t_wall = time.perf_counter()
            e0.record(main_stream)
            run_steps(args.steps, args.warmup)
            e1.record(main_stream)
            torch.cuda.synchronize()
            wall = (time.perf_counter() - t_wall) * 1e3 / args.steps
            dev_ms = e0.elapsed_time(e1) / args.steps
            per_rep.append(max(dev_ms, wall))
            dev_rep.append(dev_ms)
            wall_rep.append(wall)
        return {"ms": float(np.median(per_rep)), "min": min(per_rep), "max": max(per_rep), "reps": per_rep,
                "dev_ms": float(np.median(dev_rep)), "wall_ms": float(np.median(wall_rep))}

    def spin_up(prepared) -> int:
        """Untimed steps for args.spin_up seconds (nothing of it is measured)."""
        n, t_end = 0, time.perf_counter() + args.spin_up
        while args.spin_up > 0 and time.perf_counter() < t_end:
            for i in range(16):
                prepared[(n + i) % len(prepared)](True)
            n += 16
            torch.cuda.synchronize()
        return n

    head = not args.four_calls                                  # tail of the headline step
    one_call = head and pass_scores and args.streams == 1       # the whole step through hgca_hybrid_decode_step
    separate = None
    if one_call:
        steps_by_tail["one"] = runner.HybridStep(layers[0].shape, cfg.W, cfg.P, k_max, dev, fused_tail=True,
                                                 one_call=True)
        prepared_by_tail["one"] = [steps_by_tail["one"].prepare(L) for L in layers]
        spin_steps = spin_up(prepared_by_tail["one"])
        full = timed("one", True)
        steady = timed("one", False)                            # selection reused: hgca_hybrid_decode_step_selected
        separate = timed(head, True)                            # the same work through the separate entry points
        separate_steady = timed(head, False)
    else:
        spin_steps = spin_up(prepared_by_tail[head])
        full = timed(head, True)
        steady = timed(head, False)                             # selection reused
    other = timed(not head, True)
    other_steady = timed(not head, False)
    ms_per_step, steady_ms = full["ms"], steady["ms"]

    # ---- per-call device time: HIP events on the stream the kernels are launched on ---------------------
    def time_call(fn, n=args.steps) -> float:
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        for i in range(args.warmup):
            fn(layers[i % len(layers)])
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(evs):
            L = layers[i % len(layers)]
            a.record(main_stream)
            fn(L)
            b.record(main_stream)
        torch.cuda.synchronize()
        return float(np.mean([a.elapsed_time(b) for a, b in evs]))

    scores_buf = torch.empty(cfg.B, cfg.Hq, cfg.P, dtype=torch.float32, device=dev)
    sh = layers[0].shape
    a_gpu = torch.zeros(cfg.B, cfg.Hq, cfg.W, dtype=torch.float32, device=dev)
    a_maw = torch.zeros_like(a_gpu)
    thr_idx = torch.empty(cfg.B, cfg.Hq, cfg.W, dtype=torch.int32, device=dev)
    thr_cnt = torch.empty(cfg.B, cfg.Hq, dtype=torch.int32, device=dev)
    g_idx = torch.full((cfg.B, cfg.Hkv, max(k_max, 1)), -1, dtype=torch.int32, device=dev)
    g_cnt = torch.zeros(cfg.B, cfg.Hkv, dtype=torch.int32, device=dev)
    # KV_ctx of Alg. 1: the kept entries copied to per-head contiguous storage, then read as a stream
    kc = max(k_max, 1)
    k_ctx = torch.zeros(cfg.B, cfg.Hq, kc, cfg.d, dtype=layers[0].q.dtype, device=dev)
    v_ctx = torch.zeros_like(k_ctx)
    ctx_cnt = torch.zeros(cfg.B, cfg.Hq, dtype=torch.int32, device=dev)
    per_head = hgca.Shape(sh.dtype, cfg.B * cfg.Hq, 1, 1, cfg.d, sh.sm_scale)
    ctx_tier = hgca.Tier(k_ctx.view(-1, 1, kc, cfg.d), v_ctx.view(-1, 1, kc, cfg.d), k_max, ctx_cnt.view(-1))
    ws_ctx = hgca.alloc_workspace(per_head, k_max, 0, 0, dev)
    calls = {
        "dense_window_attn": lambda L: hgca.dense_window_attn(sh, L.q, L.window, step.o_w, step.lse_w, step.ws_dense),
        "pool_scores": lambda L: hgca.pool_scores(sh, L.q, L.pool, scores_buf),
        "select_salient": lambda L: hgca.select_salient(sh, L.q, L.pool, L.k, k_max, step.idx, step.cnt,
                                                        step.ws_sparse, sel_scores_out=step.sel_scores),
        "sparse_attn": lambda L: hgca.sparse_attn(sh, L.q, L.pool, step.idx, step.cnt, k_max, step.o_s, step.lse_s,
                                                  step.ws_sparse),
        "sparse_attn_given_scores": lambda L: hgca.sparse_attn(sh, L.q, L.pool, step.idx, step.cnt, k_max, step.o_s,
                                                               step.lse_s, step.ws_sparse,
                                                               sel_scores=step.sel_scores),
        "lse_merge": lambda L: hgca.lse_merge(sh, step.o_s, step.lse_s, step.o_w, step.lse_w, step.o, step.lse),
        # the paper's own sparsifier (Alg. 1): window weights, their moving average, the beta/size rule
        "dense_window_attn_weights": lambda L: hgca.dense_window_attn_weights(sh, L.q, L.window, step.o_w, step.lse_w,
                                                                              a_gpu, step.ws_dense),
        "maw_update": lambda L: hgca.maw_update(sh, a_maw, a_gpu, L.window.seq_lens, cfg.W, 1, 0.3),
        "threshold_select": lambda L: hgca.threshold_select(sh, a_maw, L.window.seq_lens, cfg.W, cfg.W, 1.0, cfg.W,
                                                            thr_idx, thr_cnt),
        # group-shared lists under GQA (Sec. 3.3, merged heads): one list per KV head
        "select_salient_grouped": lambda L: hgca.select_salient_grouped(sh, L.q, L.pool, L.k, k_max, g_idx, g_cnt,
                                                                        step.ws_sparse),
        "sparse_attn_grouped": lambda L: hgca.sparse_attn_grouped(sh, L.q, L.pool, g_idx, g_cnt, k_max, step.o_s,
                                                                  step.lse_s, step.ws_sparse),
        "ctx_compact": lambda L: hgca.ctx_compact(sh, L.pool, step.idx, step.cnt, k_max, k_ctx, v_ctx, k_max,
                                                  cnt_out=ctx_cnt),
        "attn_over_kv_ctx": lambda L: hgca.dense_window_attn(per_head, L.q.view(-1, 1, cfg.d), ctx_tier,
                                                             step.o_s.view(-1, 1, cfg.d), step.lse_s.view(-1, 1),
                                                             ws_ctx),
    }
    call_ms = {name: time_call(fn) for name, fn in calls.items()}
    call_bytes = {"dense_window_attn": nbytes["dense"], "pool_scores": int(p_lens.sum()) * cfg.Hkv * cfg.d * cfg.elem_bytes,
                  "select_salient": nbytes["select"], "sparse_attn": nbytes["sparse"],
                  "sparse_attn_given_scores": nbytes["sparse"] - k_gather // 2,
                  # weights: one fp32 per (head, window token) written as a score, then read and rewritten
                  "dense_window_attn_weights": nbytes["dense"] + 3 * 4 * cfg.Hq * int(w_lens.sum()),
                  "maw_update": 3 * 4 * cfg.Hq * int(w_lens.sum()),
                  "threshold_select": 4 * cfg.Hq * int(w_lens.sum()),
                  # K of the pool once per KV head + one fp32 score per (KV head, token) written and read
                  "select_salient_grouped": int(p_lens.sum()) * cfg.Hkv * (cfg.d * cfg.elem_bytes + 8),
                  # K and V rows of the kept entries once per KV head
                  "sparse_attn_grouped": 2 * cfg.Hkv * k_sum * cfg.d * cfg.elem_bytes,
                  # kept rows read and written once; then streamed once
                  "ctx_compact": 2 * k_gather, "attn_over_kv_ctx": k_gather}
    call_gbps = {n: call_bytes[n] / (call_ms[n] * 1e-3) / 1e9 for n in call_bytes}
    log("[bench] per call (ms, moved GB/s): " + ", ".join(
        f"{n}={call_ms[n]:.4f}" + (f"/{call_gbps[n]:.0f}" if n in call_gbps else "") for n in call_ms))

    # dominant kernel: the pool-score pass (K of the whole older context, once per KV head).  Its launch duration is
    # taken over a run of back-to-back launches between ONE pair of events on the launch stream (an event pair around
    # every single launch, as for the per-call figures above, adds the events' own turn-around to each launch)
    def launches_back_to_back(fn, n) -> float:
        for i in range(args.warmup):
            fn(layers[i % len(layers)])
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(main_stream)
        for i in range(n):
            fn(layers[i % len(layers)])
        b.record(main_stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n
    score_launch_ms = float(np.median([launches_back_to_back(calls["pool_scores"], max(args.steps, 20)) for _ in range(args.reps)]))
    score_bytes = call_bytes["pool_scores"]
    achieved = score_bytes / (score_launch_ms * 1e-3) / 1e9
    traffic, traffic_commit = measured_traffic("pool_scores_mfma_kernel") if args.config == "C2" else (None, None)
    roof = {"bound": "hbm", "kernel": "pool_scores_mfma_kernel<128,4> (hgca_pool_scores; first kernel of "
                                      "hgca_select_salient): a figure of this ONE kernel, not of the step",
            "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
            "traffic": traffic, "traffic_source": "profiles/c2_step_hbm_traffic.md" if traffic else None,
            "traffic_measured_at_commit": traffic_commit, "bytes_per_launch": score_bytes,
            "avg_launch_ms": score_launch_ms, "avg_launch_ms_event_pair_per_launch": call_ms["pool_scores"],
            # the step as a whole against the same peak, on algorithmic bytes (the metric) and on the bytes it moves
            "step_frac_algorithmic": nbytes["full"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "step_frac_moved": moved_full / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "steady_step_frac_algorithmic": nbytes["steady"] / (steady_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}

    def rate(nb, ms):
        return nb / (ms * 1e-3) / 1e9

    props = torch.cuda.get_device_properties(0)
    device = {"name": torch.cuda.get_device_name(0), "arch": getattr(props, "gcnArchName", None),
              "compute_units": props.multi_processor_count, "hbm_gib": round(props.total_memory / 2**30, 1),
              "clock_mhz": getattr(props, "clock_rate", 0) / 1e3 or None,
              "memory_clock_mhz": getattr(props, "memory_clock_rate", 0) / 1e3 or None,
              "rocm": torch.version.hip, "torch": torch.__version__}

    def spread(t: dict) -> dict:
        return {"ms_per_step": t["ms"], "min_ms": t["min"], "max_ms": t["max"], "repetitions": len(t["reps"]),
                "device_ms_per_step": t["dev_ms"], "wall_ms_per_step": t["wall_ms"]}

    out = {
        "metric": METRIC, "value": 1e3 / ms_per_step, "unit": "layer-steps/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOADS[args.config] + "; full step = dense + select + sparse + merge",
                   "layers_cycled": args.layers, "streams": args.streams,
                   "select_passes_scores_to_sparse": pass_scores,
                   "calls": "hgca_hybrid_decode_step" if one_call else
                            "hgca_dense_window_attn, hgca_select_salient, hgca_sparse_attn (results deferred), "
                            "hgca_lse_merge_splits" if head else
                            "hgca_select_salient, hgca_sparse_attn, hgca_dense_window_attn, hgca_lse_merge"},
        "protocol": f"{len(full['reps'])} repetitions of ({args.warmup} warm-up steps, {args.steps} timed steps between "
                    "two HIP events, device synchronised on both sides); ms_per_step and value are the median "
                    "repetition, a step's time the larger of device and wall-clock time; before the first "
                    f"repetition the device runs {spin_steps} untimed steps ({args.spin_up:g} s) so that clocks and "
                    "power state are those of a device that is already serving",
        "repetitions": len(full["reps"]), "ms_per_step_min": full["min"], "ms_per_step_max": full["max"],
        "ms_per_step_reps": full["reps"], "device": device,
        "achieved_hbm_gbps": rate(nbytes["full"], ms_per_step),
        "hbm_frac": rate(nbytes["full"], ms_per_step) / HBM_PEAK_GBPS,
        "algorithmic_bytes_per_step": nbytes["full"],
        "moved_bytes_per_step": moved_full,
        "moved_hbm_frac": rate(moved_full, ms_per_step) / HBM_PEAK_GBPS,
        "steady": {**spread(steady), "layer_steps_per_s": 1e3 / steady_ms,
                   "achieved_hbm_gbps": rate(nbytes["steady"], steady_ms),
                   "hbm_frac": rate(nbytes["steady"], steady_ms) / HBM_PEAK_GBPS,
                   "algorithmic_bytes_per_step": nbytes["steady"],
                   "calls": "hgca_hybrid_decode_step_selected" if one_call else "separate entry points"},
        ("four_calls" if head else "deferred_tail"): {
            **spread(other), "layer_steps_per_s": 1e3 / other["ms"],
            "hbm_frac": rate(nbytes["full"], other["ms"]) / HBM_PEAK_GBPS,
            "steady_ms_per_step": other_steady["ms"],
            "steady_hbm_frac": rate(nbytes["steady"], other_steady["ms"]) / HBM_PEAK_GBPS},
        "separate_calls_deferred": None if separate is None else {
            **spread(separate), "hbm_frac": rate(nbytes["full"], separate["ms"]) / HBM_PEAK_GBPS,
            "steady_ms_per_step": separate_steady["ms"],
            "steady_hbm_frac": rate(nbytes["steady"], separate_steady["ms"]) / HBM_PEAK_GBPS},
        "per_call_ms": call_ms, "per_call_gbps": call_gbps,
        "device_ms_per_step": full["dev_ms"], "wall_ms_per_step": full["wall_ms"],
        "roofline": roof,
    }
    if args.config == "C2" and not args.no_decode_loop:
        out["paper_literal_decode"] = decode_loop_timing(torch, hgca, cfg, layers[0], k_max, dev)
        # Alg. 1's blk_size is a free constant: the same loop with the cache in 64-token blocks
        out["paper_literal_decode_blocks_of_64"] = decode_loop_timing(torch, hgca, cfg, layers[0], k_max, dev,
                                                                      block_size=64)
        out["append_stage"] = append_stage_timing(torch, hgca, cfg, layers[0], dev)
        out["paper_literal_append_turn"] = append_turn_timing(torch, hgca, cfg, layers[0], k_max, dev)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(host_layers[0], args.cpu_seconds)
    print(json.dumps(out), flush=True)
    return 0


def decode_loop_timing(torch, hgca, cfg, L, k_max, dev, block_size: int = 16, n_steps: int = 64) -> dict:
    """The paper's own decode step over a managed cache (Alg. 2 then Alg. 1) at the workload's shape: token
    insert, dense window attention with weights, sparse attention over the per-head salient lists, merge,
    moving-average update, eviction of the oldest block when the window is full (every block_size steps).
    The cache starts from the workload's tensors: pool and window copied into 16-token blocks, the salient
    lists seeded with the top-k selection, the window one block short of full."""
    from paper_2507_03153_amd import cache

    B, Hq, Hkv, d, W, P = cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cfg.W, cfg.P
    win_blocks, pool_blocks = W // block_size, P // block_size
    runs = 3                                                   # timed runs below, each with its untimed steps first
    warm = max(64, block_size)                                 # untimed steps per run: the device settles to its clocks
    spare = runs * ((n_steps + warm) // block_size + 1) + 4    # blocks for every step run below
    C = cache.LayerCache(L.q.dtype, B, Hq, Hkv, d, block_size, win_blocks, pool_blocks + win_blocks + spare,
                         k_max + runs * (n_steps + warm + block_size), float(L.shape.sm_scale), dev)

    def to_blocks(dst, src, first):                            # [B,Hkv,n,d] -> blocks first.. of every sequence
        n_blk = src.shape[2] // block_size
        blocks = src[:, :, :n_blk * block_size].reshape(B, Hkv, n_blk, block_size, d).permute(0, 2, 1, 3, 4)
        dst.view(B, C.max_blocks, Hkv, block_size, d)[:, first:first + n_blk] = blocks
    for dst, pool, win in ((C.k_blocks, L.pool.k, L.window.k), (C.v_blocks, L.pool.v, L.window.v)):
        to_blocks(dst, pool, 0)
        to_blocks(dst, win[:, :, :W - block_size], pool_blocks)
    C.first_win_block.fill_(pool_blocks)
    C.pool_lens.fill_(pool_blocks * block_size)
    C.win_lens.fill_(W - block_size)
    ws = hgca.alloc_workspace(L.shape, 0, C.pool_cap, C.k_max, dev)
    hgca.select_salient(L.shape, L.q, C.pool, L.k, C.k_max, C.ctx_idx, C.ctx_cnt, ws)
    C.a_maw.fill_(1.0 / W)
    k_in = L.window.k[:, :, W - 1].contiguous()
    v_in = L.window.v[:, :, W - 1].contiguous()
    stream = torch.cuda.current_stream()

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def eager(one_call: bool) -> float:
        def run(n):
            for _ in range(n):
                C.decode_step(L.q, k_in, v_in, 0.3, 1.0, one_call=one_call)
        run(warm)                                              # untimed steps, with their evictions
        torch.cuda.synchronize()
        t_wall = time.perf_counter()
        e0.record(stream)
        run(n_steps)
        e1.record(stream)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t_wall) * 1e3 / n_steps
        return max(e0.elapsed_time(e1) / n_steps, wall)
    eager_ms = eager(True)                                     # hgca_managed_decode_step: one call per step
    separate_ms = eager(False)                                 # the five entry points it stands for

    # the same step captured once in a HIP graph (every decision of the step is taken on the device, so the
    # captured launch sequence is valid for every step) and replayed: removes the host cost of the launches
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        C.decode_step(L.q, k_in, v_in, 0.3, 1.0, one_call=True)
    for _ in range(warm - 1):                                  # the capture ran no step; the untimed steps of this run
        graph.replay()
    torch.cuda.synchronize()
    t_wall = time.perf_counter()
    e0.record(torch.cuda.current_stream())
    for _ in range(n_steps):
        graph.replay()
    e1.record(torch.cuda.current_stream())
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t_wall) * 1e3 / n_steps
    graph_ms = max(e0.elapsed_time(e1) / n_steps, wall)
    ms = eager_ms
    status = int(C.status.cpu()[0])
    kept = C.ctx_cnt.float().mean().item()
    elem = 2 if L.q.dtype == torch.bfloat16 else 4
    moved = 2 * B * Hkv * (W - block_size // 2) * d * elem + 2 * B * Hq * kept * d * elem + 6 * 4 * B * Hq * W
    return {"ms_per_step": ms, "layer_steps_per_s": 1e3 / ms, "graph_replay_ms_per_step": graph_ms,
            "separate_calls_ms_per_step": separate_ms, "steps": n_steps, "evictions": n_steps // block_size,
            "block_size": block_size, "salient_per_head": kept, "cache_status": status,
            "bytes_per_step": int(moved), "hbm_frac": moved / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "calls_per_step": "hgca_managed_decode_step (2 launches: window splits with scores, the token's insert "
                              "and the gather over the salient lists; then fold, weights + moving average and "
                              "eviction per row)",
            "separate_calls": "kv_append, dense_window_attn_maw, sparse_attn (deferred), lse_merge_splits, kv_evict "
                              "(7 kernels)"}


def append_stage_timing(torch, hgca, cfg, L, dev, n_q: int = 32, reps: int = 40) -> dict:
    """The append branch (N incoming tokens per sequence) on the workload's tensors: causal attention over the
    window (whose last N tokens stand for the incoming ones), attention over the COMPLETE pool, merge, and the
    query-averaged weights of both parts (what the KV manager's re-evaluation thresholds).  Both contractions run on
    the matrix cores, so the figure is set beside the MFMA peak as well as the HBM peak."""
    B, Hq, Hkv, d, W, P = cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cfg.W, cfg.P
    g = torch.Generator(device="cpu").manual_seed(7)
    q = torch.randn(B, n_q, Hq, d, generator=g).to(torch.bfloat16).to(dev)
    f32 = dict(dtype=torch.float32, device=dev)
    ws = hgca.append_workspace(L.shape, n_q, max(W, P), dev)
    ws_t = hgca.append_tiers_workspace(L.shape, n_q, W, P, dev)
    ow, lw = torch.empty(B, n_q, Hq, d, **f32), torch.empty(B, n_q, Hq, **f32)
    op, lp = torch.empty_like(ow), torch.empty_like(lw)
    o, lse = torch.empty_like(ow), torch.empty_like(lw)
    a_gpu, a_cpu = torch.empty(B, Hq, W, **f32), torch.empty(B, Hq, P, **f32)
    merged = hgca.Shape(L.shape.dtype, B * n_q, Hq, Hkv, d, L.shape.sm_scale)
    stream = torch.cuda.current_stream()
    calls = {
        "append_attn_window": lambda: hgca.append_attn(L.shape, q, L.window, True, ow, lw, ws),
        "append_attn_pool": lambda: hgca.append_attn(L.shape, q, L.pool, False, op, lp, ws),
        "lse_merge": lambda: hgca.lse_merge(merged, op, lp, ow, lw, o, lse),
        "append_weights_window": lambda: hgca.append_weights(L.shape, q, L.window, True, lw, a_gpu),
        "append_weights_pool": lambda: hgca.append_weights(L.shape, q, L.pool, False, lp, a_cpu),
        # the same attention with the weights rounded once to bf16 for the second contraction (HGCA_APPEND_ONE_PART_P)
        "append_attn_window_one_part_p": lambda: hgca.append_attn(L.shape, q, L.window, True, ow, lw, ws, one_part_p=True),
        "append_attn_pool_one_part_p": lambda: hgca.append_attn(L.shape, q, L.pool, False, op, lp, ws, one_part_p=True),
        # both tiers in one call: one launch for the splits of window and pool, one fold (merged output + per-tier lse)
        "append_attn_tiers": lambda: hgca.append_attn_tiers(L.shape, q, L.window, L.pool, o, lse, ws_t, lse_window_out=lw,
                                                            lse_pool_out=lp),
        "append_weights_tiers": lambda: hgca.append_weights_tiers(L.shape, q, L.window, L.pool, lw, lp, a_gpu, a_cpu),
        "append_attn_tiers_one_part_p": lambda: hgca.append_attn_tiers(L.shape, q, L.window, L.pool, o, lse, ws_t,
                                                                       lse_window_out=lw, lse_pool_out=lp, one_part_p=True),
    }
    ms = {}
    for name, fn in calls.items():
        # these kernels keep matrix cores, vector units, LDS and HBM busy at once and the device settles to its
        # clocks for that mix only after some tens of calls (a call takes 20 % longer in between): 60 untimed calls
        for _ in range(60):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        ms[name] = e0.elapsed_time(e1) / reps
    elem = 2
    kv_bytes = 2 * B * Hkv * (W + P) * d * elem                 # K and V of both tiers, once per KV head
    flops = 4.0 * B * Hq * n_q * (W + P) * d                    # QK^T and PV, 2 flops per multiply-add (causal skip ignored)
    attn_ms = ms["append_attn_tiers"]                           # window + pool + merge as the one call that serves them
    one_ms = ms["append_attn_tiers_one_part_p"]
    three_calls_ms = ms["append_attn_window"] + ms["append_attn_pool"] + ms["lse_merge"]
    weights_ms = ms["append_weights_tiers"]
    return {"n_q": n_q, "per_call_ms": ms, "attention_ms": attn_ms, "attention_three_calls_ms": three_calls_ms,
            "with_weights_ms": attn_ms + weights_ms,
            "tokens_per_s": B * n_q / (attn_ms * 1e-3),
            "kv_bytes": kv_bytes, "hbm_frac": kv_bytes / (attn_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "tflops": flops / (attn_ms * 1e-3) / 1e12, "mfma_frac_bf16": flops / (attn_ms * 1e-3) / 2.5e15,
            "note": "probabilities enter the second contraction as a high and a low bf16 part, so the matrix cores "
                    "execute 1.5x the counted flops",
            "one_part_p": {"attention_ms": one_ms, "hbm_frac": kv_bytes / (one_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                           "tflops": flops / (one_ms * 1e-3) / 1e12,
                           "mfma_frac_bf16": flops / (one_ms * 1e-3) / 2.5e15}}


def append_turn_timing(torch, hgca, cfg, L, k_max, dev, n_q: int = 32, turns: int = 8, block_size: int = 16) -> dict:
    """Whole append turns over a managed cache at the workload's shape (hgca_managed_append_step: insert of n_q tokens
    per sequence, attention over the window and the complete pool, merge, query-averaged weights of both parts,
    moving averages, re-evaluation of the salient lists, eviction of the blocks the insert pushed out).  The cache
    starts as in the decode loop; the turns run back to back in one timed region."""
    from paper_2507_03153_amd import cache

    B, Hq, Hkv, d, W, P = cfg.B, cfg.Hq, cfg.Hkv, cfg.d, cfg.W, cfg.P
    win_blocks, pool_blocks = W // block_size, P // block_size
    n_blk = -(-n_q // block_size)
    warm_turns = 8
    spare = (turns + warm_turns + 1) * n_blk + 4
    C = cache.LayerCache(L.q.dtype, B, Hq, Hkv, d, block_size, win_blocks, pool_blocks + win_blocks + spare,
                         4 * k_max, float(L.shape.sm_scale), dev, win_cap_blocks=win_blocks + n_blk)
    for dst, pool, win in ((C.k_blocks, L.pool.k, L.window.k), (C.v_blocks, L.pool.v, L.window.v)):
        view = dst.view(B, C.max_blocks, Hkv, block_size, d)
        view[:, :pool_blocks] = pool.reshape(B, Hkv, pool_blocks, block_size, d).permute(0, 2, 1, 3, 4)
        view[:, pool_blocks:pool_blocks + win_blocks - 1] = \
            win[:, :, :W - block_size].reshape(B, Hkv, win_blocks - 1, block_size, d).permute(0, 2, 1, 3, 4)
    C.first_win_block.fill_(pool_blocks)
    C.pool_lens.fill_(pool_blocks * block_size)
    C.win_lens.fill_(W - block_size)
    C.a_maw.fill_(1.0 / W)
    g = torch.Generator(device="cpu").manual_seed(11)
    q = torch.randn(B, n_q, Hq, d, generator=g).to(L.q.dtype).to(dev)
    k_in = torch.randn(B, n_q, Hkv, d, generator=g).to(L.q.dtype).to(dev)
    v_in = torch.randn(B, n_q, Hkv, d, generator=g).to(L.q.dtype).to(dev)
    BETA = 2.0                                                 # keeps a few thousand entries per head on these inputs
    stream = torch.cuda.current_stream()
    for _ in range(warm_turns):                                # untimed (the first allocates the turn's buffers; the device
        C.append_step(q, k_in, v_in, 0.3, BETA)                # settles to its clocks for this mix of work over some ms)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_wall = time.perf_counter()
    e0.record(stream)
    for _ in range(turns):
        C.append_step(q, k_in, v_in, 0.3, BETA)
    e1.record(stream)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t_wall) * 1e3 / turns
    ms = max(e0.elapsed_time(e1) / turns, wall)
    kv_bytes = 2 * B * Hkv * (W + P) * d * 2 + B * Hkv * (W + P) * d * 2      # K and V once for the attention, K again for the weights
    return {"n_q": n_q, "turns": turns, "ms_per_turn": ms,
            "tokens_per_s": B * n_q / (ms * 1e-3), "kv_bytes": kv_bytes,
            "hbm_frac": kv_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, "beta": BETA, "cache_status": int(C.status.cpu()[0]),
            "salient_per_head_after": C.ctx_cnt.float().mean().item(),
            "calls_per_turn": "hgca_managed_append_step (insert, both tiers' attention in one launch, fold, weights of "
                              "window and pool in one launch, then moving average + re-evaluation + eviction per row: 5 kernels)"}


def copy_calibration(torch, dev) -> int:
    """Plain device-to-device copies of 1 GiB: what FETCH_SIZE / WRITE_SIZE read for a known size."""
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    for _ in range(10):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"copy_bytes_read": n, "copy_bytes_written": n, "copies": 10}), flush=True)
    return 0


def cpu_baseline(L, target_s: float) -> dict:
    """The fp64 oracle as it stands, timed on this machine's host cores: whole layer-steps of the workload
    (dense, select, sparse, merge for all sequences and heads), first on ONE core (a few steps), then on all
    cores until about `target_s` seconds have gone.  `value` is the all-core rate."""
    import oracle

    def tier(t):
        return oracle.Tier(t.k, t.v, t.cap, t.seq_lens, t.block_table, t.block_size)

    def one_step():
        t0 = time.perf_counter()
        oracle.hybrid_step(L.q, tier(L.window), tier(L.pool), L.k, L.k_max, L.scale)
        return time.perf_counter() - t0

    def sample(budget_s: float, at_most: int):
        times = [one_step()]
        while sum(times) < budget_s and len(times) < at_most:
            times.append(one_step())
        return times

    all_cores = oracle.num_threads()
    oracle.set_num_threads(1)
    single = sample(min(6.0, target_s / 2), 5)
    oracle.set_num_threads(all_cores)
    times = sample(target_s, 200)
    med, med1 = float(np_median(times)), float(np_median(single))
    return {"value": 1.0 / med, "unit": "layer-steps/s", "cores": all_cores, "kind": "oracle",
            "one_core": {"value": 1.0 / med1, "unit": "layer-steps/s", "cores": 1,
                         "sample": f"{len(single)} whole {L.cfg.name} layer-steps ({sum(single):.1f}s), median"},
            "sample": f"{len(times)} whole {L.cfg.name} layer-steps on layer 0 ({sum(times):.1f}s of fp64 oracle time, "
                      f"OpenMP over (batch, head)), median"}


def np_median(xs):
    xs = sorted(xs)
    n = len(xs)
    return xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])


if __name__ == "__main__":
    sys.exit(main())
