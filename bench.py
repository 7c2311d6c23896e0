#!/usr/bin/env python3
"""Throughput of the R-KV compression step on one MI355X.

A step = one pass of the whole hot path (key pre-pass, similarity pass, finalize + select, gather)
over every layer of one sequence, i.e. one `rkv_compress` call with num_problems = layers, on
seeded synthetic inputs already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2_llama8b_b1024]
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK = 2.5e15      # MI355X dense bf16, flop/s
HBM_PEAK = 8.0e12            # B/s

# HBM bytes per launch of the similarity (Gram) kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# of this same command, scaled by a plain 256 MiB device copy (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0 KiB);
# the runs are summarised in profiles/rkv_compress_cfg2_counters.md.
GRAM_TRAFFIC_BYTES = {"cfg2_llama8b_b1024": int((9.082e4 * 2.0 + 1144) * 1024)}


def hip_runtime(torch):
    """The HIP runtime already loaded by torch (used here only for event timing)."""
    cand = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
    hip = ctypes.CDLL(cand if os.path.exists(cand) else "libamdhip64.so.7")
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
    return hip


def cpu_baseline(w, q, k, v, seconds: float):
    """The CPU oracle, as it stands, on a bounded sample of the same workload's heads."""
    from oracle import rkv_oracle as O
    prm = O.Params(alpha=w.alpha, budget=w.budget, pool_w=w.pool_w, beta=w.beta,
                   sim_threshold=w.sim_threshold, lam=w.lam, eps=w.eps)
    heads = [(p, h) for p in range(w.num_problems) for h in range(w.kv_heads)]
    G = w.group
    done, t0 = 0, time.perf_counter()
    for (p, h) in heads:
        O.compress_head(q[p, h * G:(h + 1) * G], k[p, h], v[p, h], prm)
        done += 1
        if time.perf_counter() - t0 > seconds:
            break
    dt = time.perf_counter() - t0
    per_head = dt / done
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    steps_per_s = 1.0 / (per_head * len(heads))
    return {"value": steps_per_s, "unit": "steps/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{done} of {len(heads)} heads of the same workload in {dt:.1f} s, "
                      f"extrapolated linearly to one step (all heads)"}


def other_modes(torch, rkv, synth, w, shp, qd, kd, vd, ws, ko, vo, idx, reps=50):
    """The same workload launched in other ways, for context next to the headline figure (ms per step):
    one call per layer back to back on one stream (eager, and replayed from a HIP graph), a high
    threshold at which only true near-duplicates count as similar, attention-only eviction
    (lambda = 1, no similarity pass), the exact shortcut of the similarity pass, and in-place compaction."""
    import dataclasses

    def timed(fn):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / reps

    res = {}
    one = dataclasses.replace(shp, num_problems=1)
    layers = range(w.num_problems)

    def per_layer():
        for l in layers:
            rkv.rkv_compress(one, qd[l:l + 1], kd[l:l + 1], vd[l:l + 1], ws=ws, k_out=ko[l:l + 1], v_out=vo[l:l + 1],
                             kept_idx=idx[l:l + 1])
    res["per_layer_calls_ms"] = timed(per_layer)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        per_layer()                                  # every kernel has run once before the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        per_layer()
    res["per_layer_calls_hip_graph_ms"] = timed(graph.replay)
    for name, change in (("sim_threshold_0.95_ms", {"sim_threshold": 0.95}), ("attention_only_lambda_1_ms", {"lam": 1.0})):
        alt = dataclasses.replace(shp, **change)
        res[name] = timed(lambda: rkv.rkv_compress(alt, qd, kd, vd, ws=ws, k_out=ko, v_out=vo, kept_idx=idx))
    # the exact shortcut of the similarity pass (a row that has met its beta partners is left alone;
    # same results, data-dependent time: with these keys nearly every row is done after one column tile)
    alt = dataclasses.replace(shp, flags=shp.flags | rkv.RKV_FLAG_SKIP_SATURATED)
    res["skip_saturated_ms"] = timed(lambda: rkv.rkv_compress(alt, qd, kd, vd, ws=ws, k_out=ko, v_out=vo, kept_idx=idx))
    # compaction inside the cache allocation instead of into a second one (copies of the caches: the
    # call overwrites them; only rows behind the first evicted one move)
    kc, vc = kd.clone(), vd.clone()
    spans = []
    for _ in range(5 + reps):
        kc.copy_(kd)
        vc.copy_(vd)                                 # every call sees the same cache contents
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0.record()
        rkv.rkv_compress_inplace(shp, qd, kc, vc, ws=ws, kept_idx=idx)
        t1.record()
        spans.append((t0, t1))
    torch.cuda.synchronize()
    res["inplace_ms"] = sum(a.elapsed_time(b) for a, b in spans[5:]) / reps
    return {k_: float(v_) for k_, v_ in res.items()}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2_llama8b_b1024")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sim-threshold", type=float, default=None)
    ap.add_argument("--beta", type=int, default=None)
    ap.add_argument("--lam", type=float, default=None, help="lambda of Eq. 7 (1.0 = attention-only eviction, similarity pass skipped)")
    ap.add_argument("--skip-saturated", action="store_true",
                    help="set RKV_FLAG_SKIP_SATURATED (exact, data-dependent shortcut of the similarity pass); "
                         "the roofline entry is then not meaningful and is omitted")
    ap.add_argument("--no-other-modes", action="store_true",
                    help="skip the extra launch modes reported for context (per-layer calls, T = 0.95, attention-only)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy a few times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (heads shard across GPUs with no exchange; "
              "no multi-GPU figure is produced). Re-run with --gpus 1.", file=sys.stderr)
        return 2

    import torch
    from paper_2505_24133_amd import rkv, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    rkv.load_library()
    w = synth.CONFIGS[args.workload]
    if args.sim_threshold is not None:
        w = synth.scaled(w, sim_threshold=args.sim_threshold)
    if args.beta is not None:
        w = synth.scaled(w, beta=args.beta)
    if args.lam is not None:
        w = synth.scaled(w, lam=args.lam)
    q, k, v = synth.make_batch(w)

    def dev(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)

    qd, kd, vd = dev(q), dev(k), dev(v)
    shp = rkv.Shape(num_problems=w.num_problems, kv_heads=w.kv_heads, q_heads=w.q_heads, n_tokens=w.n_tokens,
                    budget=w.budget, alpha=w.alpha, pool_w=w.pool_w, beta=w.beta,
                    sim_threshold=w.sim_threshold, lam=w.lam, eps=w.eps,
                    flags=rkv.RKV_FLAG_SKIP_SATURATED if args.skip_saturated else 0)
    ws = rkv.make_workspace(shp)
    oshape = (w.num_problems, w.kv_heads, w.budget, w.head_dim)
    ko = torch.empty(oshape, dtype=torch.bfloat16, device="cuda")
    vo = torch.empty(oshape, dtype=torch.bfloat16, device="cuda")
    idx = torch.empty(oshape[:3], dtype=torch.int32, device="cuda")

    def step(events=None):
        st = rkv.rkv_compress(shp, qd, kd, vd, ws=ws, k_out=ko, v_out=vo, kept_idx=idx, events=events)[0]
        assert st == rkv.RKV_OK

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps, wall clock between two device synchronisations
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # ---- the same K steps again with HIP events between the stages (on the launch stream)
    hip = hip_runtime(torch)
    K = args.steps
    handles = (ctypes.c_void_p * (5 * K))()
    for i in range(5 * K):
        e = ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(e)) == 0
        handles[i] = e
    t0 = time.perf_counter()
    for s in range(K):
        ev = (ctypes.c_void_p * 5).from_buffer(handles, s * 5 * ctypes.sizeof(ctypes.c_void_p))
        step(ev)
    torch.cuda.synchronize()
    ms_per_step_events = (time.perf_counter() - t0) * 1e3 / K
    stage_ms = np.zeros((K, 4))
    for s in range(K):
        for i in range(4):
            f = ctypes.c_float()
            assert hip.hipEventElapsedTime(ctypes.byref(f), handles[s * 5 + i], handles[s * 5 + i + 1]) == 0
            stage_ms[s, i] = f.value
    for i in range(5 * K):
        hip.hipEventDestroy(handles[i])
    avg = stage_ms.mean(axis=0)

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()

    # ---- algorithmic work of one launch (one step)
    heads = w.num_problems * w.kv_heads
    n, d = w.n_cand, w.head_dim
    gram_flops = 2.0 * n * n * d * heads                         # dense cosine matrix of Eq. 5
    k_bytes = heads * n * d * 2
    prepass_bytes = k_bytes + heads * w.group * w.alpha * d * 2 + heads * n * 4 * (1 + w.alpha)
    select_bytes = heads * (n * 4 * (2 + w.alpha) + w.budget * 4)
    gather_bytes = heads * w.budget * d * 2 * 2 * 2              # K and V, read + write
    stages = {
        "prepass": {"ms": avg[0], "GB/s": prepass_bytes / avg[0] / 1e6, "frac_hbm": prepass_bytes / (avg[0] * 1e-3) / HBM_PEAK},
        "gram": {"ms": avg[1], "TFLOP/s": gram_flops / avg[1] / 1e9, "frac_mfma": gram_flops / (avg[1] * 1e-3) / MFMA_BF16_PEAK},
        "finalize_select": {"ms": avg[2], "GB/s": select_bytes / avg[2] / 1e6, "frac_hbm": select_bytes / (avg[2] * 1e-3) / HBM_PEAK},
        "gather": {"ms": avg[3], "GB/s": gather_bytes / avg[3] / 1e6, "frac_hbm": gather_bytes / (avg[3] * 1e-3) / HBM_PEAK},
    }
    if w.lam == 1.0:                     # attention-only: the similarity pass is not run
        stages["gram"] = {"ms": avg[1]}
    dominant = max(stages, key=lambda s: stages[s]["ms"])
    if dominant == "gram":
        roofline = {"kernel": "gram_kernel", "bound": "mfma", "achieved": gram_flops / (avg[1] * 1e-3) / 1e12,
                    "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s",
                    "frac": gram_flops / (avg[1] * 1e-3) / MFMA_BF16_PEAK,
                    "traffic": GRAM_TRAFFIC_BYTES.get(w.name) if args.sim_threshold is None and args.beta is None else None}
    else:
        b = {"prepass": prepass_bytes, "finalize_select": select_bytes, "gather": gather_bytes}[dominant]
        i = ["prepass", "gram", "finalize_select", "gather"].index(dominant)
        roofline = {"kernel": dominant + "_kernel", "bound": "hbm", "achieved": b / (avg[i] * 1e-3) / 1e9,
                    "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": b / (avg[i] * 1e-3) / HBM_PEAK, "traffic": None}

    out = {
        "metric": "compression steps/sec (all layers, 1 seq)",
        "value": 1e3 / ms_per_step,
        "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "layers": w.num_problems, "kv_heads": w.kv_heads, "q_heads": w.q_heads,
                   "n_tokens": w.n_tokens, "budget": w.budget, "alpha": w.alpha, "head_dim": d,
                   "pool_w": w.pool_w, "beta": w.beta, "sim_threshold": w.sim_threshold, "lambda": w.lam},
        "cached_tokens_scored_per_sec": w.num_problems * n / (ms_per_step * 1e-3),
        "cached_head_tokens_scored_per_sec": heads * n / (ms_per_step * 1e-3),
        "ms_per_step_with_stage_events": ms_per_step_events,
        "stages": {s: {kk: float(vv) for kk, vv in st.items()} for s, st in stages.items()},
        "roofline": roofline,
    }
    if not (args.skip_saturated or args.no_other_modes) and args.sim_threshold is None and args.beta is None and args.lam is None:
        out["other_modes"] = other_modes(torch, rkv, synth, w, shp, qd, kd, vd, ws, ko, vo, idx)
    if args.skip_saturated:
        out["config"]["flags"] = "RKV_FLAG_SKIP_SATURATED"
        out["roofline"] = None          # executed matrix work is data dependent in this mode
        out["stages"]["gram"].pop("TFLOP/s"), out["stages"]["gram"].pop("frac_mfma")
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, q, k, v, args.cpu_seconds)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
