#!/usr/bin/env python3
"""Throughput of the R-KV compression step on one MI355X.

A step = one pass of the whole hot path (key pre-pass, similarity pass, finalize + select, gather)
over every layer of every sequence of the workload, i.e. one `rkv_compress` call with
num_problems = sequences x layers, on seeded synthetic inputs already resident in HBM.  The headline
workload (`value`, `roofline`) is the 8B model at budget 1024, one sequence; the other full-size
configurations are timed after it with fewer steps and reported under `workloads`.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2_llama8b_b1024]
"""
from __future__ import annotations

import argparse
import ctypes
import hashlib
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK = 2.5e15      # MI355X dense bf16, flop/s
HBM_PEAK = 8.0e12            # B/s
HEADLINE = "cfg2_llama8b_b1024"
OTHERS = {"cfg3_llama8b_b4096": 30, "cfg4_qwen14b_b2048_bs16": 8, "cfg5_llama8b_b8192_bs4": 8}   # timed steps each
HOST_WORKERS = max(1, min(16, os.cpu_count() or 1))       # the machine's CPU share for one GPU


def gram_traffic(workload: str):
    """HBM bytes per launch of the similarity kernel, from the committed rocprofv3 counter summary of this
    workload (profiles/rkv_compress_<workload>_counters.md), or None when there is none or it was taken
    with another version of the kernel's source (the summary records the SHA-256 of gram.hip)."""
    path = os.path.join(ROOT, "profiles", f"rkv_compress_{workload}_counters.md")
    src = os.path.join(ROOT, "paper_2505_24133_amd", "csrc", "gram.hip")
    try:
        text = open(path).read()
        digest = hashlib.sha256(open(src, "rb").read()).hexdigest()
    except OSError:
        return None, None
    m_hash = re.search(r"gram\.hip sha256: ([0-9a-f]{64})", text)
    m_bytes = re.search(r"gram_kernel HBM bytes per launch \(FETCH \+ WRITE\): (\d+)", text)
    if not m_hash or not m_bytes or m_hash.group(1) != digest:
        return None, os.path.relpath(path, ROOT)
    return int(m_bytes.group(1)), os.path.relpath(path, ROOT)


def hip_runtime(torch):
    """The HIP runtime already loaded by torch (used here only for event timing)."""
    cand = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
    hip = ctypes.CDLL(cand if os.path.exists(cand) else "libamdhip64.so.7")
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
    return hip


# ------------------------------------------------------------------------------ CPU oracle leg
def _oracle_task(args):
    """Worker process: draw problem p from its recipe and run the oracle, as it stands, on heads hs."""
    w, p, hs = args
    try:
        from threadpoolctl import threadpool_limits
        limit = threadpool_limits(limits=1)          # one core per worker; the pool supplies the parallelism
    except Exception:                                # pragma: no cover
        limit = None
    from oracle import rkv_oracle as O
    from paper_2505_24133_amd import synth
    q, k, v = synth.make_problem(w, p)
    prm = O.Params(alpha=w.alpha, budget=w.budget, pool_w=w.pool_w, beta=w.beta,
                   sim_threshold=w.sim_threshold, lam=w.lam, eps=w.eps)
    G = w.group
    t0 = time.perf_counter()
    for h in hs:
        O.compress_head(q[h * G:(h + 1) * G], k[h], v[h], prm)
    del limit
    return len(hs), time.perf_counter() - t0


def cpu_baseline(w, seconds: float, max_heads: int):
    """The CPU oracle on a bounded, seeded sample of the workload's heads: one oracle call per head, the
    heads dealt to HOST_WORKERS single-threaded worker processes (drawing the inputs is not timed as
    oracle work but is inside the wall clock).  Returns steps/s extrapolated linearly in heads."""
    import multiprocessing as mp
    from concurrent.futures import ProcessPoolExecutor, wait, FIRST_COMPLETED
    total = w.num_problems * w.kv_heads
    rng = np.random.default_rng(12345)
    if total <= max_heads:
        heads = [(p, h) for p in range(w.num_problems) for h in range(w.kv_heads)]
    else:
        # every sequence, its first and last layer first, then random layers; one random head each
        seqs = w.num_problems // w.layers
        layer_order = [0, w.layers - 1] + [int(x) for x in rng.permutation(np.arange(1, w.layers - 1))]
        heads = [(s * w.layers + l, int(rng.integers(w.kv_heads))) for l in layer_order for s in range(seqs)][:max_heads]
    by_problem = {}
    for p, h in heads:
        by_problem.setdefault(p, []).append(h)
    tasks = [(w, p, hs[i:i + 2]) for p, hs in by_problem.items() for i in range(0, len(hs), 2)]
    done, busy = 0, 0.0
    t0 = time.perf_counter()
    with ProcessPoolExecutor(max_workers=HOST_WORKERS, mp_context=mp.get_context("spawn")) as ex:
        pending, it = set(), iter(tasks)
        stop = False
        while True:
            while not stop and len(pending) < 2 * HOST_WORKERS:
                t = next(it, None)
                if t is None:
                    stop = True
                    break
                pending.add(ex.submit(_oracle_task, t))
            if not pending:
                break
            finished, pending = wait(pending, return_when=FIRST_COMPLETED)
            for f in finished:
                n_, dt_ = f.result()
                done += n_
                busy += dt_
            if time.perf_counter() - t0 > seconds:
                stop = True                          # let what is in flight finish, submit nothing more
    wall = time.perf_counter() - t0
    steps_per_s = done / wall / total
    return {"value": steps_per_s, "unit": "steps/s", "cores": HOST_WORKERS, "kind": "oracle",
            "sample": f"{done} of {total} heads of {w.name} (seeded sample covering every sequence and its first and "
                      f"last layer) in {wall:.1f} s wall on {HOST_WORKERS} single-threaded worker processes "
                      f"({busy:.1f} core-seconds inside the oracle), extrapolated linearly in heads to one step"}


# ------------------------------------------------------------------------------ GPU timing
def measure(torch, rkv, w, q, k, v, steps, warmup, sets=1, flags=0):
    """Time `steps` calls of rkv_compress on workload w: wall clock between two device synchronisations,
    then the same number of calls again with HIP events between the stages.  `sets` > 1 rotates that many
    copies of the inputs and outputs so that no call finds its data in the caches (L2, 256 MB MALL)."""
    def dev(bits):
        return torch.from_numpy(np.asarray(bits).view(np.int16)).cuda().view(torch.bfloat16)

    shp = rkv.Shape(num_problems=w.num_problems, kv_heads=w.kv_heads, q_heads=w.q_heads, n_tokens=w.n_tokens,
                    budget=w.budget, alpha=w.alpha, pool_w=w.pool_w, beta=w.beta,
                    sim_threshold=w.sim_threshold, lam=w.lam, eps=w.eps, flags=flags)
    ins = [(dev(q), dev(k), dev(v))]
    for _ in range(sets - 1):
        ins.append(tuple(t.clone() for t in ins[0]))
    oshape = (w.num_problems, w.kv_heads, w.budget, w.head_dim)
    outs = [(torch.empty(oshape, dtype=torch.bfloat16, device="cuda"), torch.empty(oshape, dtype=torch.bfloat16, device="cuda"),
             torch.empty(oshape[:3], dtype=torch.int32, device="cuda")) for _ in range(sets)]
    ws = rkv.make_workspace(shp)

    def step(i, events=None):
        qd, kd, vd = ins[i % sets]
        ko, vo, idx = outs[i % sets]
        st = rkv.rkv_compress(shp, qd, kd, vd, ws=ws, k_out=ko, v_out=vo, kept_idx=idx, events=events)[0]
        assert st == rkv.RKV_OK

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    # ---- timed region: exactly `steps` steps, wall clock between two device synchronisations
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps

    # ---- the same steps again with HIP events between the stages (on the launch stream)
    hip = hip_runtime(torch)
    handles = (ctypes.c_void_p * (5 * steps))()
    for i in range(5 * steps):
        e = ctypes.c_void_p()
        assert hip.hipEventCreate(ctypes.byref(e)) == 0
        handles[i] = e
    t0 = time.perf_counter()
    for s in range(steps):
        step(s, (ctypes.c_void_p * 5).from_buffer(handles, s * 5 * ctypes.sizeof(ctypes.c_void_p)))
    torch.cuda.synchronize()
    ms_events = (time.perf_counter() - t0) * 1e3 / steps
    stage_ms = np.zeros((steps, 4))
    for s in range(steps):
        for i in range(4):
            f = ctypes.c_float()
            assert hip.hipEventElapsedTime(ctypes.byref(f), handles[s * 5 + i], handles[s * 5 + i + 1]) == 0
            stage_ms[s, i] = f.value
    for i in range(5 * steps):
        hip.hipEventDestroy(handles[i])
    avg = stage_ms.mean(axis=0)

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
    stages = {s: {kk: float(vv) for kk, vv in st.items()} for s, st in stages.items()}
    work = {"gram_flops": gram_flops, "prepass_bytes": prepass_bytes, "select_bytes": select_bytes, "gather_bytes": gather_bytes}
    state = {"shp": shp, "ins": ins, "outs": outs, "ws": ws}
    return ms_per_step, ms_events, stages, work, state


def sclk_under_load(torch, launch):
    """Shader and memory clock the driver reports while `launch` (which only enqueues work) keeps the GPU
    busy; None where the node does not expose them."""
    def starred(path):
        try:
            for line in open(path):
                if "*" in line:
                    return int(re.search(r"(\d+)\s*Mhz", line, re.I).group(1))
        except (OSError, AttributeError):
            return None
        return None
    base = "/sys/class/drm/card0/device"
    seen = []
    launch()                                   # a few tens of milliseconds of queued work
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < 0.02:
        s, m = starred(f"{base}/pp_dpm_sclk"), starred(f"{base}/pp_dpm_mclk")
        if s is not None:
            seen.append((s, m))
        time.sleep(0.002)
    torch.cuda.synchronize()
    if not seen:
        return None
    return {"sclk_mhz": max(s for s, _ in seen), "sclk_mhz_samples": [s for s, _ in seen][:12], "mclk_mhz": seen[-1][1],
            "how": "pp_dpm_sclk / pp_dpm_mclk (the driver's smoothed current value) polled while the queued steps ran"}


def copy_ceiling(torch):
    """A plain 256 MiB device-to-device copy (read + written bytes per second): what a copy reaches here."""
    src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for _ in range(10):
        dst.copy_(src)
    t1.record()
    torch.cuda.synchronize()
    return 10 * 2 * (256 << 20) / (t0.elapsed_time(t1) * 1e-3) / 1e9


def mfma_sustained(torch, rkv, keys):
    """What the matrix pipe sustains on the similarity pass's MFMA instruction alone (TFLOP/s): launches of
    about a millisecond that issue nothing else, on fragments of the workload's keys, back to back for a
    quarter of a second; the second half is timed.  The published peak assumes the top clock; this is the
    rate at the clock the chip settles at on such data."""
    ops = keys.reshape(-1)[: rkv.RKV_PROBE_OPERAND_BYTES // 2].contiguous()
    sink = torch.empty(rkv.RKV_PROBE_SINK_BYTES // 4, dtype=torch.float32, device="cuda")
    chains, launches = 6000, 120
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    flops = 0
    for i in range(2 * launches):
        if i == launches:
            t0.record()
        flops = rkv.rkv_probe_mfma(ops, sink, chains)
    t1.record()
    torch.cuda.synchronize()
    return launches * flops / (t0.elapsed_time(t1) * 1e-3) / 1e12


def other_modes(torch, rkv, w, state, reps=50):
    """The same workload launched in other ways, for context next to the headline figure (ms per step):
    one call per layer back to back on one stream (eager, and replayed from a HIP graph), a high
    threshold at which only true near-duplicates count as similar (dense, with the exact shortcut, and with
    the triangular schedule, which is meant for that case), attention-only eviction (lambda = 1, no
    similarity pass), the exact shortcut of the similarity pass, in-place compaction, and two sequences in flight
    on two streams (time per step of either)."""
    import dataclasses
    shp, ws = state["shp"], state["ws"]
    qd, kd, vd = state["ins"][0]
    ko, vo, idx = state["outs"][0]

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
    # the same per-layer calls dealt to four streams (default priority, a workspace each): kernels of
    # different layers then share the machine, which one call per layer leaves mostly idle
    lanes = [torch.cuda.Stream() for _ in range(4)]
    lane_ws = [rkv.make_workspace(one) for _ in lanes]

    def per_layer_streams():
        main = torch.cuda.current_stream()
        for s_ in lanes:
            s_.wait_stream(main)
        for l in layers:
            with torch.cuda.stream(lanes[l % 4]):
                rkv.rkv_compress(one, qd[l:l + 1], kd[l:l + 1], vd[l:l + 1], ws=lane_ws[l % 4], k_out=ko[l:l + 1],
                                 v_out=vo[l:l + 1], kept_idx=idx[l:l + 1])
        for s_ in lanes:
            main.wait_stream(s_)
    res["per_layer_calls_4_streams_ms"] = timed(per_layer_streams)
    # and that fork-join pattern replayed from a HIP graph (no host time per call)
    torch.cuda.synchronize()
    graph4 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph4):
        per_layer_streams()
    res["per_layer_calls_4_streams_hip_graph_ms"] = timed(graph4.replay)
    # two sequences in flight: steps alternate between two streams (own buffers and workspace each), so that one
    # sequence's memory-bound kernels (pre-pass, gather) share the machine with the other's similarity pass
    pair = [(qd, kd, vd, ko, vo, idx, ws, torch.cuda.Stream()),
            (qd.clone(), kd.clone(), vd.clone(), torch.empty_like(ko), torch.empty_like(vo), torch.empty_like(idx),
             rkv.make_workspace(shp), torch.cuda.Stream())]

    def two_in_flight():
        for q2, k2, v2, ko2, vo2, idx2, ws2, st in pair:
            with torch.cuda.stream(st):
                rkv.rkv_compress(shp, q2, k2, v2, ws=ws2, k_out=ko2, v_out=vo2, kept_idx=idx2)
    for st in (pair[0][7], pair[1][7]):
        st.wait_stream(torch.cuda.current_stream())
    res["two_sequences_two_streams_ms_per_step"] = timed(two_in_flight) / 2
    del pair
    # and two sequences batched into one call (twice the problems: the similarity pass's workgroups then fill
    # whole rounds of the machine)
    both = dataclasses.replace(shp, num_problems=2 * shp.num_problems)
    q2, k2, v2 = torch.cat([qd, qd]), torch.cat([kd, kd]), torch.cat([vd, vd])
    ko2, vo2, idx2 = torch.cat([ko, ko]), torch.cat([vo, vo]), torch.cat([idx, idx])
    ws2 = rkv.make_workspace(both)
    res["two_sequences_one_call_ms_per_step"] = timed(lambda: rkv.rkv_compress(both, q2, k2, v2, ws=ws2, k_out=ko2, v_out=vo2, kept_idx=idx2)) / 2
    del q2, k2, v2, ko2, vo2, idx2, ws2
    for name, change in (("sim_threshold_0.95_ms", {"sim_threshold": 0.95}), ("attention_only_lambda_1_ms", {"lam": 1.0}),
                         ("sim_threshold_0.95_skip_saturated_ms", {"sim_threshold": 0.95, "flags": rkv.RKV_FLAG_SKIP_SATURATED}),
                         ("sim_threshold_0.95_triangular_scan_ms", {"sim_threshold": 0.95, "flags": rkv.RKV_FLAG_TRIANGULAR_SCAN})):
        alt = dataclasses.replace(shp, **change)
        alt_ws = rkv.make_workspace(alt)             # some flags need more scratch than the default call
        res[name] = timed(lambda: rkv.rkv_compress(alt, qd, kd, vd, ws=alt_ws, k_out=ko, v_out=vo, kept_idx=idx))
    # the exact shortcut of the similarity pass (a row that has met its beta partners is left alone;
    # same results, data-dependent time: with these keys nearly every row is done after one column tile)
    alt = dataclasses.replace(shp, flags=shp.flags | rkv.RKV_FLAG_SKIP_SATURATED)
    res["skip_saturated_ms"] = timed(lambda: rkv.rkv_compress(alt, qd, kd, vd, ws=ws, k_out=ko, v_out=vo, kept_idx=idx))
    # the entry point with the library's fixed scratch array (no workspace argument)
    if rkv.rkv_workspace_size(shp) <= rkv.RKV_STATIC_SCRATCH_BYTES:
        res["static_scratch_ms"] = timed(lambda: rkv.rkv_compress_static(shp, qd, kd, vd, ko, vo, idx))
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


def summary(w, ms_per_step, stages):
    seqs = max(1, w.num_problems // w.layers)
    return {"ms_per_step": ms_per_step, "sequences": seqs, "steps_per_s_x_sequences": seqs * 1e3 / ms_per_step,
            "cached_tokens_scored_per_sec": w.num_problems * w.n_cand / (ms_per_step * 1e-3), "stages": stages,
            "gram_frac_mfma": stages["gram"].get("frac_mfma"), "gather_GB/s": stages["gather"]["GB/s"]}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--cpu-seconds", type=float, default=8.0, help="wall-clock bound of each CPU-oracle sample")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sim-threshold", type=float, default=None)
    ap.add_argument("--beta", type=int, default=None)
    ap.add_argument("--lam", type=float, default=None, help="lambda of Eq. 7 (1.0 = attention-only eviction, similarity pass skipped)")
    ap.add_argument("--skip-saturated", action="store_true",
                    help="set RKV_FLAG_SKIP_SATURATED (exact, data-dependent shortcut of the similarity pass); "
                         "the roofline entry is then not meaningful and is omitted")
    ap.add_argument("--no-other-modes", action="store_true",
                    help="skip the extra launch modes reported for context (per-layer calls, T = 0.95, attention-only)")
    ap.add_argument("--no-workloads", action="store_true", help="time the named workload only, not the other full-size configurations")
    ap.add_argument("--no-cold", action="store_true", help="skip the cache-cold repetition (rotating input and output sets)")
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
    plain = args.sim_threshold is None and args.beta is None and args.lam is None and not args.skip_saturated
    if args.sim_threshold is not None:
        w = synth.scaled(w, sim_threshold=args.sim_threshold)
    if args.beta is not None:
        w = synth.scaled(w, beta=args.beta)
    if args.lam is not None:
        w = synth.scaled(w, lam=args.lam)
    flags = rkv.RKV_FLAG_SKIP_SATURATED if args.skip_saturated else 0
    q, k, v = synth.make_batch(w, workers=HOST_WORKERS)

    ms_per_step, ms_events, stages, work, state = measure(torch, rkv, w, q, k, v, args.steps, args.warmup, flags=flags)

    # ---- roofline entry of the dominant kernel, from the HIP-event stage times of this run
    order = ["prepass", "gram", "finalize_select", "gather"]
    dominant = max(stages, key=lambda s: stages[s]["ms"])
    if dominant == "gram":
        traffic, source = gram_traffic(w.name) if plain else (None, None)
        roofline = {"kernel": "gram_kernel", "bound": "mfma", "achieved": stages["gram"]["TFLOP/s"],
                    "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s", "frac": stages["gram"]["frac_mfma"],
                    "traffic": traffic, "traffic_source": source}
    else:
        b = {"prepass": work["prepass_bytes"], "finalize_select": work["select_bytes"], "gather": work["gather_bytes"]}[dominant]
        ms = stages[dominant]["ms"]
        roofline = {"kernel": dominant + "_kernel", "bound": "hbm", "achieved": b / (ms * 1e-3) / 1e9,
                    "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": b / (ms * 1e-3) / HBM_PEAK, "traffic": None}

    n, d = w.n_cand, w.head_dim
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
        "cached_head_tokens_scored_per_sec": w.num_problems * w.kv_heads * n / (ms_per_step * 1e-3),
        "ms_per_step_with_stage_events": ms_events,
        "stages": stages,
        "roofline": roofline,
    }
    if args.skip_saturated:
        out["config"]["flags"] = "RKV_FLAG_SKIP_SATURATED"
        out["roofline"] = None          # executed matrix work is data dependent in this mode
        out["stages"]["gram"].pop("TFLOP/s"), out["stages"]["gram"].pop("frac_mfma")

    # ---- measured clocks and what a plain device copy reaches, next to the published peaks
    shp, ws = state["shp"], state["ws"]

    def burst():
        for i in range(300):
            qd, kd, vd = state["ins"][0]
            ko, vo, idx = state["outs"][0]
            rkv.rkv_compress(shp, qd, kd, vd, ws=ws, k_out=ko, v_out=vo, kept_idx=idx)
    out["device"] = {"name": torch.cuda.get_device_name(0), "clocks_under_load": sclk_under_load(torch, burst),
                     "device_copy_GB/s": copy_ceiling(torch),
                     "mfma_sustained_TFLOP/s": mfma_sustained(torch, rkv, state["ins"][0][1]), "published_peaks": {"bf16_mfma_TFLOP/s": 2500.0, "hbm_GB/s": 8000.0}}

    if out["roofline"]["bound"] == "mfma":
        # the similarity kernel's rate against what the matrix pipe sustains (the roofline entry keeps the published peak)
        out["device"]["gram_over_mfma_sustained"] = round(out["roofline"]["achieved"] / out["device"]["mfma_sustained_TFLOP/s"], 4)
    if plain and not args.no_other_modes:
        out["other_modes"] = other_modes(torch, rkv, w, state)
    del state

    # ---- cache-cold repetition: rotate enough copies of the inputs and outputs that a call's data has left
    # the 256 MB last-level cache before it is used again
    if plain and not args.no_cold:
        per_set = int((k.size + v.size) * 2 * (1 + w.budget / w.n_tokens))     # bytes of K, V read and written per step
        sets = max(2, min(6, int(np.ceil(4 * (256 << 20) / per_set))))
        c_ms, _, c_stages, _, _ = measure(torch, rkv, w, q, k, v, max(args.steps // 2, sets), min(args.warmup, 2 * sets), sets=sets)
        out["cold"] = {"sets_rotated": sets, "bytes_between_reuse": int(sets * per_set), "ms_per_step": c_ms,
                       "value": 1e3 / c_ms, "stages": c_stages,
                       "gather_GB/s_warm_vs_cold": [stages["gather"]["GB/s"], c_stages["gather"]["GB/s"]]}
    torch.cuda.empty_cache()

    # ---- the other full-size configurations, fewer steps each (every problem drawn from its own seed)
    cpu = {}
    if plain and not args.no_workloads and args.workload == HEADLINE:
        out["workloads"] = {w.name: summary(w, ms_per_step, stages)}
        for name, k_steps in OTHERS.items():
            wo = synth.CONFIGS[name]
            qo, ko_, vo_ = synth.make_batch(wo, workers=HOST_WORKERS)
            o_ms, _, o_stages, _, o_state = measure(torch, rkv, wo, qo, ko_, vo_, k_steps, 2)
            out["workloads"][name] = summary(wo, o_ms, o_stages)
            out["workloads"][name]["steps"] = k_steps
            t_bytes, t_src = gram_traffic(name)
            out["workloads"][name]["gram_traffic"] = t_bytes
            if o_stages["gram"].get("TFLOP/s"):
                out["workloads"][name]["gram_over_mfma_sustained"] = round(o_stages["gram"]["TFLOP/s"] / out["device"]["mfma_sustained_TFLOP/s"], 4)
            del o_state, qo, ko_, vo_
            torch.cuda.empty_cache()
            if not args.no_cpu_baseline:
                cpu[name] = cpu_baseline(wo, args.cpu_seconds, 256)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, 2 * args.cpu_seconds, 256)
        if cpu:
            out["cpu_baseline"]["other_workloads"] = cpu
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
