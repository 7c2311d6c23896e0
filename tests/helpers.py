"""Host-side helpers for the parity tests: tolerance rules, detection of rows whose threshold
decision is within rounding of T, exact top-k of a score vector.  CPU only, numpy only."""
from __future__ import annotations

import numpy as np

from oracle import rkv_oracle as O

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
