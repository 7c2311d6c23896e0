"""Seeded synthetic inputs for the R-KV compression step.

This module only *draws inputs*: bf16 key/value caches and observation queries with
the shapes of the paper's distilled reasoning models (Sec. 4 "Models and Datasets",
hyper-parameters from Sec. 4 "Hyperparameters") and with injected redundancy that
stands in for the repetitive reasoning traces the paper measures (Sec. 2, Fig. 2).
It contains none of the method's arithmetic (no attention, no similarity, no
selection) and is the only module shared by the CPU oracle's tests and the HIP path.

All tensors are returned as numpy ``uint16`` arrays holding bf16 bit patterns:
    q : [q_heads, alpha, d]      observation queries (last alpha decode steps)
    k : [kv_heads, N, d]         key cache, N = budget + buffer, rows in token order
    v : [kv_heads, N, d]         value cache
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Iterable, Tuple

import numpy as np


# --------------------------------------------------------------------------- bf16
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------- workloads
@dataclass(frozen=True)
class Workload:
    """One benchmark / parity configuration (shapes + hyper-parameters + input recipe)."""
    name: str
    num_problems: int          # P = sequences x layers, each an independent compression
    kv_heads: int
    q_heads: int
    n_tokens: int              # N = budget + buffer rows held when the step triggers
    budget: int                # rows kept in total (selected + the alpha observation rows)
    head_dim: int = 128
    alpha: int = 8
    pool_w: int = 4            # W of the 2W-wide stabilising max-pool
    beta: int = 1              # most-recent similar tokens forgiven per token
    sim_threshold: float = 0.5
    lam: float = 0.1
    eps: float = 1e-8
    seed: int = 0
    recipe: str = "rowcopy"    # rowcopy | spans | clusters
    redundancy: float = 0.3    # fraction of rows that are (near) copies; <0: draw U(0.2,0.6) per sequence
    copy_noise: float = 0.1    # rowcopy: absolute sigma; spans: sigma relative to the source row RMS
    outlier_channels: int = 0
    layers: int = 1            # layers per sequence (num_problems = sequences * layers)
    n_clusters: int = 64
    cluster_sigma: float = 0.31622776601683794   # sqrt(0.1)

    @property
    def group(self) -> int:
        return self.q_heads // self.kv_heads

    @property
    def n_cand(self) -> int:
        return self.n_tokens - self.alpha

    @property
    def k_sel(self) -> int:
        return self.budget - self.alpha


CONFIGS: Dict[str, Workload] = {
    # tiny CPU-fast case
    "cfg1_tiny": Workload("cfg1_tiny", 1, 2, 8, 384, 256, seed=0, recipe="rowcopy",
                          redundancy=0.3, copy_noise=0.1),
    # R1-Distill-Llama-8B shape, one sequence, all 32 layers
    "cfg2_llama8b_b1024": Workload("cfg2_llama8b_b1024", 32, 8, 32, 1152, 1024, seed=1000,
                                   recipe="spans", redundancy=0.4, copy_noise=0.01,
                                   outlier_channels=4, layers=32),
    "cfg3_llama8b_b4096": Workload("cfg3_llama8b_b4096", 32, 8, 32, 4224, 4096, seed=2000,
                                   recipe="spans", redundancy=0.5, copy_noise=0.05,
                                   outlier_channels=4, layers=32),
    # R1-Distill-Qwen-14B shape, 16 sequences x 48 layers
    "cfg4_qwen14b_b2048_bs16": Workload("cfg4_qwen14b_b2048_bs16", 48 * 16, 8, 40, 2176, 2048,
                                        seed=3000, recipe="spans", redundancy=-1.0,
                                        copy_noise=0.01, outlier_channels=4, layers=48),
    # long-trace stress, 4 sequences x 32 layers
    "cfg5_llama8b_b8192_bs4": Workload("cfg5_llama8b_b8192_bs4", 32 * 4, 8, 32, 8320, 8192,
                                       seed=4000, recipe="clusters", layers=32),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (e.g. fewer problems for a CPU test)."""
    return replace(w, **kw)


# ----------------------------------------------------------------------- generators
def _rng(w: Workload, p: int, stream: int) -> np.random.Generator:
    return np.random.default_rng([w.seed, p, stream])


def _unit(x: np.ndarray) -> np.ndarray:
    nrm = np.sqrt((x.astype(np.float64) ** 2).sum(-1, keepdims=True))
    return (x / np.maximum(nrm, 1e-30)).astype(np.float32)


def _keys_rowcopy(w: Workload, p: int) -> np.ndarray:
    H, N, d = w.kv_heads, w.n_tokens, w.head_dim
    g = _rng(w, p, 1)
    k = g.standard_normal((H, N, d), dtype=np.float32)
    n_copy = int(round(w.redundancy * N))
    for h in range(H):
        rows = np.sort(g.choice(np.arange(1, N), size=n_copy, replace=False))
        for i in rows:                      # ascending, so a source may itself be a copy
            j = int(g.integers(0, i))
            k[h, i] = k[h, j] + w.copy_noise * g.standard_normal(d, dtype=np.float32)
    return k


def _span_plan(w: Workload, p: int, frac: float):
    """Token-level copy spans (shared by the heads of one problem): list of (dst, src, len)."""
    N = w.n_tokens
    g = _rng(w, p, 2)
    covered = np.zeros(N, dtype=bool)
    plan = []
    guard = 0
    while covered.mean() < frac and guard < 100000:
        guard += 1
        L = int(g.integers(16, 65))
        if N - L < L:
            L = max(1, N // 4)
        dst = int(g.integers(L, N - L + 1))
        src = int(g.integers(0, dst - L + 1))
        plan.append((dst, src, L))
        covered[dst:dst + L] = True
    return plan


def _keys_spans(w: Workload, p: int) -> np.ndarray:
    H, N, d = w.kv_heads, w.n_tokens, w.head_dim
    g = _rng(w, p, 1)
    k = g.standard_normal((H, N, d), dtype=np.float32)
    if w.outlier_channels:
        for h in range(H):
            ch = g.choice(d, size=w.outlier_channels, replace=False)
            k[h][:, ch] *= 10.0
    frac = w.redundancy
    if frac < 0:                            # per-sequence redundancy level
        seq = p // w.layers
        frac = float(np.random.default_rng([w.seed, seq, 7]).uniform(0.2, 0.6))
    for dst, src, L in _span_plan(w, p, frac):
        blk = k[:, src:src + L, :]
        rms = np.sqrt((blk.astype(np.float64) ** 2).mean(-1, keepdims=True)).astype(np.float32)
        k[:, dst:dst + L, :] = blk + w.copy_noise * rms * g.standard_normal((H, L, d), dtype=np.float32)
    return k


def _keys_clusters(w: Workload, p: int) -> np.ndarray:
    H, N, d = w.kv_heads, w.n_tokens, w.head_dim
    g = _rng(w, p, 1)
    cent = g.standard_normal((H, w.n_clusters, d), dtype=np.float32)
    which = g.integers(0, w.n_clusters, size=(H, N))
    k = np.take_along_axis(cent, which[:, :, None], axis=1)
    k = k + np.float32(w.cluster_sigma) * g.standard_normal((H, N, d), dtype=np.float32)
    return k.astype(np.float32)


def _queries(w: Workload, p: int, k: np.ndarray) -> np.ndarray:
    """Noise plus a pull towards the first four keys ("sink" tokens) and one random candidate
    per query head ("needle"), which gives a few dominant attention columns over a diffuse rest."""
    Hq, a, d, G = w.q_heads, w.alpha, w.head_dim, w.group
    g = _rng(w, p, 3)
    q = g.standard_normal((Hq, a, d), dtype=np.float32)
    root_d = np.float32(np.sqrt(d))
    for hq in range(Hq):
        h = hq // G
        sink = _unit(k[h, :4]).mean(0)
        t = int(g.integers(4, w.n_cand))
        needle = _unit(k[h, t:t + 1])[0]
        q[hq] += root_d * (1.0 * sink + 0.5 * needle)
    return q


def make_problem(w: Workload, p: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Inputs of problem ``p`` (one sequence-layer): (q, k, v) as bf16 bit patterns."""
    if w.recipe == "rowcopy":
        k = _keys_rowcopy(w, p)
    elif w.recipe == "spans":
        k = _keys_spans(w, p)
    elif w.recipe == "clusters":
        k = _keys_clusters(w, p)
    else:
        raise ValueError(f"unknown recipe {w.recipe!r}")
    v = _rng(w, p, 4).standard_normal((w.kv_heads, w.n_tokens, w.head_dim), dtype=np.float32)
    kb = f32_to_bf16_bits(k)
    q = _queries(w, p, bf16_bits_to_f32(kb))
    return f32_to_bf16_bits(q), kb, f32_to_bf16_bits(v)


def _batch_shapes(w: Workload, count: int):
    d = w.head_dim
    return ((count, w.q_heads, w.alpha, d), (count, w.kv_heads, w.n_tokens, d), (count, w.kv_heads, w.n_tokens, d))


def _fill_task(args):
    """Worker of ``make_batch(..., workers > 1)``: draw some problems into the shared files."""
    w, paths, count, todo = args
    maps = [np.memmap(path, dtype=np.uint16, mode="r+", shape=shape) for path, shape in zip(paths, _batch_shapes(w, count))]
    for slot, p in todo:
        for m, x in zip(maps, make_problem(w, p)):
            m[slot] = x
    for m in maps:
        m.flush()
    return len(todo)


def make_batch(w: Workload, problems: Iterable[int] | None = None, workers: int = 1):
    """Stack problems: q [P,Hq,alpha,d], k [P,H,N,d], v [P,H,N,d] (uint16 bf16 bits).

    With ``workers`` > 1 the problems are drawn by that many CPU-only worker processes (spawned, so they
    inherit nothing from a parent that uses the GPU) into memory-mapped scratch files that are unlinked
    before the arrays are returned; the values are those of the serial path, problem by problem."""
    ps = list(range(w.num_problems)) if problems is None else list(problems)
    if workers <= 1 or len(ps) < 2:
        qs, ks, vs = zip(*(make_problem(w, p) for p in ps))
        return np.stack(qs), np.stack(ks), np.stack(vs)
    import multiprocessing as mp
    import os
    import tempfile
    from concurrent.futures import ProcessPoolExecutor
    workers = min(workers, len(ps))
    base = "/dev/shm" if os.path.isdir("/dev/shm") and os.access("/dev/shm", os.W_OK) else None
    paths = []
    try:
        for shape in _batch_shapes(w, len(ps)):
            fd, path = tempfile.mkstemp(prefix="rkv_synth_", suffix=".u16", dir=base)
            os.ftruncate(fd, int(np.prod(shape)) * 2)
            os.close(fd)
            paths.append(path)
        todo = list(enumerate(ps))
        tasks = [(w, paths, len(ps), todo[i::4 * workers]) for i in range(4 * workers) if todo[i::4 * workers]]
        with ProcessPoolExecutor(max_workers=workers, mp_context=mp.get_context("spawn")) as ex:
            done = sum(ex.map(_fill_task, tasks))
        assert done == len(ps)
        out = tuple(np.memmap(path, dtype=np.uint16, mode="r+", shape=shape)
                    for path, shape in zip(paths, _batch_shapes(w, len(ps))))
    finally:
        for path in paths:                      # the mappings above stay valid; the files hold no name any more
            try:
                os.unlink(path)
            except OSError:
                pass
    return out
