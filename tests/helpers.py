"""Host-side helpers for the parity tests: tolerance rules, detection of rows whose threshold
decision is within rounding of T, exact top-k of a score vector, and a pool of CPU-only worker
processes that run the oracle on many heads at once.  CPU only, numpy only."""
from __future__ import annotations

import atexit
import os

import numpy as np

from oracle import rkv_oracle as O
from paper_2505_24133_amd import synth

# Scores: |gpu - oracle| <= ABS_TOL + REL_TOL * |oracle| (fp32 accumulation vs the float64 oracle).
REL_TOL = 1e-3
ABS_TOL = 1e-5
# A similarity closer than this to T may fall on either side in fp32.
SIM_BAND = 1e-5


def oracle_params(w, **variant) -> O.Params:
    return O.Params(alpha=w.alpha, budget=w.budget, pool_w=w.pool_w, beta=w.beta,
                    sim_threshold=w.sim_threshold, lam=w.lam, eps=w.eps, **variant)


def close(gpu: np.ndarray, ref: np.ndarray, rel=REL_TOL, abs_=ABS_TOL) -> np.ndarray:
    return np.abs(gpu.astype(np.float64) - ref) <= abs_ + rel * np.abs(ref)


def max_rel_err(gpu: np.ndarray, ref: np.ndarray) -> float:
    den = np.maximum(np.abs(ref), 1e-30)
    return float(np.max(np.abs(gpu.astype(np.float64) - ref) / den)) if ref.size else 0.0


def fragile_rows(k_cand: np.ndarray, T: float, beta: int, eps: float, band: float = SIM_BAND) -> np.ndarray:
    """Rows whose set of forgiven partners could change if a similarity within `band` of T flips:
    some uncertain j is not preceded (from the recent end) by beta definite hits."""
    n = k_cand.shape[0]
    if beta <= 0:
        return np.zeros(n, dtype=bool)
    S = O.cosine_similarity(k_cand, eps)
    definite = S > T + band
    uncertain = np.abs(S - T) <= band
    np.fill_diagonal(uncertain, False)
    if not uncertain.any():
        return np.zeros(n, dtype=bool)
    # number of definite hits strictly to the right of each column, per row
    right = np.cumsum(definite[:, ::-1], axis=1)[:, ::-1] - definite
    return (uncertain & (right < beta)).any(axis=1)


def fragile_tokens_transposed(k_cand: np.ndarray, T: float, beta: int, eps: float, band: float = SIM_BAND) -> np.ndarray:
    """With the transposed rule a row's forgiven entries change its partners' scores: the tokens that
    a threshold-fragile row could name (similarity above T - band) are the ones left unchecked."""
    rows = fragile_rows(k_cand, T, beta, eps, band)
    if not rows.any():
        return rows
    S = O.cosine_similarity(k_cand, eps)
    return (S[rows] > T - band).any(axis=0)


def exact_topk(z: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest entries, equal values resolved towards the larger index, ascending."""
    n = z.shape[0]
    order = np.lexsort((-np.arange(n), -z.astype(np.float64)))
    return np.sort(order[:k])


def check_kept_against_oracle(kept_sel: np.ndarray, z_ref: np.ndarray, k: int, skip: np.ndarray,
                              rel=REL_TOL, abs_=ABS_TOL):
    """Every candidate clearly above the oracle's k-th score must be kept and every one clearly
    below must not; those within the tolerance of the boundary (or in `skip`) may go either way.
    Returns (#must_keep violated, #must_drop violated, #free)."""
    tau = np.sort(z_ref)[::-1][k - 1]
    tol = abs_ + rel * abs(tau)
    kept_mask = np.zeros(z_ref.shape[0], dtype=bool)
    kept_mask[kept_sel] = True
    must_keep = (z_ref > tau + tol) & ~skip
    must_drop = (z_ref < tau - tol) & ~skip
    free = ~(must_keep | must_drop)
    return int((must_keep & ~kept_mask).sum()), int((must_drop & kept_mask).sum()), int(free.sum())


# Error of the GPU's joint score relative to the size of its two terms, lambda |I| + (1 - lambda) |R|
# (fp32 accumulation against the float64 oracle); the parity tests assert it for every candidate.
TERM_REL_ERR = 5e-5


def decidable_selection(z_ref: np.ndarray, err: np.ndarray, k: int):
    """Which candidates the top-k MUST hold and which it MUST NOT, for any score vector z' with
    |z' - z_ref| <= err element-wise (whatever the tie-break): candidate i is certainly kept when fewer
    than k others can reach its lowest possible score, and certainly dropped when at least k others stay
    above its highest possible score.  Returns (must_keep, must_drop) boolean masks; the rest is free."""
    lo, hi = z_ref - err, z_ref + err
    hi_sorted, lo_sorted = np.sort(hi), np.sort(lo)
    n = z_ref.shape[0]
    # others j with hi_j >= lo_i  (i itself always counts: hi_i >= lo_i)
    can_reach = n - np.searchsorted(hi_sorted, lo, side="left") - 1
    # others j with lo_j > hi_i   (i itself never counts)
    stay_above = n - np.searchsorted(lo_sorted, hi, side="right")
    return can_reach < k, stay_above >= k


# ------------------------------------------------------------------ the oracle on many heads at once
_POOL = None


def oracle_workers() -> int:
    """Worker processes for the oracle: the machine's CPU share (16 per GPU), less on smaller hosts."""
    return max(1, min(16, os.cpu_count() or 1))


def _pool():
    """CPU-only worker processes (spawned, so they never inherit the parent's GPU state), started once."""
    global _POOL
    if _POOL is None:
        import multiprocessing as mp
        from concurrent.futures import ProcessPoolExecutor
        _POOL = ProcessPoolExecutor(max_workers=oracle_workers(), mp_context=mp.get_context("spawn"),
                                    initializer=_worker_init)
        atexit.register(_POOL.shutdown, wait=False, cancel_futures=True)
    return _POOL


def _worker_init():
    """The oracle allocates and frees n x n float64 matrices for every head.  Keeping freed memory in the
    worker's heap (no mmap for large blocks, no trimming) spares the first-touch page faults of fresh
    mappings, which otherwise take several times longer than the oracle's arithmetic."""
    import ctypes
    try:
        libc = ctypes.CDLL("libc.so.6")
        libc.mallopt(-4, 0)                  # M_MMAP_MAX = 0
        libc.mallopt(-1, 2 ** 31 - 1)        # M_TRIM_THRESHOLD
    except OSError:                          # pragma: no cover
        pass


def _single_thread():
    try:
        from threadpoolctl import threadpool_limits
        return threadpool_limits(limits=1)
    except Exception:                                   # pragma: no cover
        import contextlib
        return contextlib.nullcontext()


def _oracle_heads_task(args):
    """Worker: draw problem p of workload w from its seeded recipe and run the oracle on the heads hs."""
    w, p, hs, variant = args
    with _single_thread():
        q, k, v = synth.make_problem(w, p)
        prm = oracle_params(w, **variant)
        G = w.group
        return [(p, h, O.compress_head(q[h * G:(h + 1) * G], k[h], v[h], prm)) for h in hs]


def oracle_heads(w, heads, **variant):
    """Yield ((p, h), oracle dict) for the listed heads of a seeded workload, computed by the worker
    pool (each worker regenerates its problems from the recipe; nothing comes from the GPU)."""
    by_problem = {}
    for (p, h) in heads:
        by_problem.setdefault(p, []).append(h)
    tasks = []
    for p, hs in sorted(by_problem.items()):
        for i in range(0, len(hs), 2):                  # at most two heads per task keeps the workers evenly loaded
            tasks.append((w, p, hs[i:i + 2], variant))
    from concurrent.futures import as_completed
    futs = [_pool().submit(_oracle_heads_task, t) for t in tasks]
    for f in as_completed(futs):
        for (p, h, ref) in f.result():
            yield (p, h), ref


def _oracle_rows_task(args):
    k_bits, rows, T, beta, eps = args
    with _single_thread():
        return O.mean_similarity_rows(O.decode_bf16(k_bits), rows, T, beta, eps)


def mean_similarity_all_rows(k_bits: np.ndarray, T: float, beta: int, eps: float) -> np.ndarray:
    """Eq. 5-6 for every candidate of a head too large for the n x n matrix: the oracle's row-by-row
    form, the rows dealt to the worker pool."""
    n = k_bits.shape[0]
    parts = np.array_split(np.arange(n), 4 * oracle_workers())
    futs = [_pool().submit(_oracle_rows_task, (k_bits, rows, T, beta, eps)) for rows in parts if len(rows)]
    return np.concatenate([f.result() for f in futs])
