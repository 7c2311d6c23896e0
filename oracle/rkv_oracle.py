"""CPU oracle for the R-KV decode-time KV-cache compression step.

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, float64 numpy implementation of what
the paper's method computes for one KV head, written from the paper's equations so
that a reader can check it against them by eye.  It shares no code with the HIP
path and must never be imported by the product package: only the tests, the smoke
check and the benchmark's CPU-baseline leg call it.  A matrix product, an argsort
and exp are the only library primitives used as steps; nothing is blocked, fused or
reordered.

Notation follows the paper: N rows are held (budget + buffer), the last ``alpha``
are the observation tokens (always kept), the first ``n = N - alpha`` are the
candidates, and ``k = budget - alpha`` of them are selected (Sec. 3.1).

Readings taken where the paper is silent or inconsistent (each is a default here):
  * selection is per KV head (Sec. 3.4 speaks of a per-head budget and score Z^h_i);
  * the softmax of the observation attention spans the n candidates only;
  * grouped-query heads: max over the G raw scaled logit matrices, then softmax (Eq. 2-3);
  * the 2W-wide max-pool is applied to every query row, then the rows are averaged
    (Eq. 4); the window [i-W, i+W-1] is clipped to [0, n); W = 0 switches it off;
  * "zero the similarities of the beta most recent similar tokens": for token i, among
    the j with S[i][j] > T (strict), the beta largest j have S[i][j] set to 0 before
    token i's own average is taken (Sec. 3.3 and the pseudo-code agree on this);
    (``recency_transposed`` zeroes the partner's entry S[j][i] instead, see ``forgive_recent``);
  * the average divides by n (zeroed entries included);
  * ties in the top-k are broken towards the larger (more recent) index;
  * kept rows are emitted in ascending original order, followed by the observation rows.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Params:
    alpha: int = 8           # observation window
    budget: int = 0          # rows kept in total (selected + observation)
    pool_w: int = 4          # W
    beta: int = 1
    sim_threshold: float = 0.5   # T
    lam: float = 0.1         # lambda
    eps: float = 1e-8
    pool_after_mean: bool = False    # pseudo-code order: mean over the alpha rows, then the pooling
    shared_selection: bool = False   # pseudo-code: scores averaged over the KV heads, one index set
    gqa: str = "max_logits"          # "max_logits" (Eq. 2-3) | "softmax_max" | "softmax_mean" (App. A.2)
    recency_transposed: bool = False  # the forgiven similarity leaves the recent partner's average instead


# ----------------------------------------------------------------------------- decode
def decode_bf16(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns -> float64 (exact): sign, 8-bit exponent, 7-bit fraction."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.int64)
    sign = np.where((b >> 15) & 1, -1.0, 1.0)
    expo = (b >> 7) & 0xFF
    frac = (b & 0x7F).astype(np.float64)
    normal = sign * (1.0 + frac / 128.0) * np.exp2((expo - 127).astype(np.float64))
    subnormal = sign * (frac / 128.0) * 2.0 ** -126
    out = np.where(expo == 0, subnormal, normal)
    special = np.where(frac == 0, sign * np.inf, np.nan)
    return np.where(expo == 255, special, out)


# ------------------------------------------------------------------------- importance
def softmax_rows(x: np.ndarray) -> np.ndarray:
    e = np.exp(x - x.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def attention_weights(q: np.ndarray, k_cand: np.ndarray, gqa: str = "max_logits") -> np.ndarray:
    """Eq. 1 (G = 1) and Eq. 2-3 (G > 1).

    q [G, alpha, d] are the observation queries of the G query heads that share this
    KV head, k_cand [n, d] the candidate keys.  Returns A [alpha, n]; rows sum to 1 except with
    "softmax_max".

    ``gqa`` picks how the G heads are merged.  "max_logits" is Eq. 2-3 as printed: element-wise max
    of the raw scaled logits, then one softmax.  App. A.2 instead speaks of pooling attention scores
    (after the softmax), with the max adopted and the mean named as what earlier work used:
    "softmax_max" = max over g of softmax(L^g) (not renormalised), "softmax_mean" = mean over g.
    """
    G, alpha, d = q.shape
    logits = np.stack([q[g] @ k_cand.T / np.sqrt(d) for g in range(G)])   # Eq. 2
    if gqa == "max_logits":
        pooled = logits.max(axis=0)                                       # max over the group
        return softmax_rows(pooled)                                       # Eq. 3
    per_head = np.stack([softmax_rows(logits[g]) for g in range(G)])      # Eq. 1 per query head
    if gqa == "softmax_max":
        return per_head.max(axis=0)
    if gqa == "softmax_mean":
        return per_head.mean(axis=0)
    raise ValueError(gqa)


def stabilise(A: np.ndarray, W: int) -> np.ndarray:
    """Eq. 4, first part: A~[j, i] = max(A[j, i-W .. i+W-1]), window clipped to the row."""
    if W <= 0:
        return A.copy()
    alpha, n = A.shape
    out = np.empty_like(A)
    for i in range(n):
        lo, hi = max(0, i - W), min(n - 1, i + W - 1)
        out[:, i] = A[:, lo:hi + 1].max(axis=1)
    return out


def importance(q: np.ndarray, k_cand: np.ndarray, W: int, gqa: str = "max_logits") -> np.ndarray:
    """Eq. 4: I[i] = mean over the alpha query rows of the stabilised attention."""
    return stabilise(attention_weights(q, k_cand, gqa), W).mean(axis=0)


def importance_mean_then_pool(q: np.ndarray, k_cand: np.ndarray, W: int, gqa: str = "max_logits") -> np.ndarray:
    """The order of the paper's pseudo-code (Alg. 1): I'[k] = mean over the alpha query rows of A[:, k],
    then the same 2W-wide sliding max applied to I'."""
    mean = attention_weights(q, k_cand, gqa).mean(axis=0, keepdims=True)
    return stabilise(mean, W)[0]


# ------------------------------------------------------------------------- redundancy
def cosine_similarity(k_cand: np.ndarray, eps: float) -> np.ndarray:
    """Eq. 5: rows divided by (L2 norm + eps), Gram matrix, diagonal set to 0."""
    norm = np.sqrt((k_cand * k_cand).sum(axis=1, keepdims=True))
    kbar = k_cand / (norm + eps)
    S = kbar @ kbar.T
    np.fill_diagonal(S, 0.0)
    return S


def recent_similar(S: np.ndarray, T: float, beta: int) -> np.ndarray:
    """Sec. 3.3: boolean M with M[i, j] true when j is one of the (up to) beta largest indices among
    the tokens similar to i, i.e. among {j : S[i, j] > T}."""
    n = S.shape[0]
    hit = S > T
    M = np.zeros_like(hit)
    rev_cols = np.arange(n)[::-1]
    for _ in range(max(0, int(beta))):
        has = hit.any(axis=1)
        if not has.any():
            break
        last = rev_cols[np.argmax(hit[:, ::-1], axis=1)]      # largest j with a hit, per row
        rows = np.nonzero(has)[0]
        M[rows, last[rows]] = True
        hit[rows, last[rows]] = False
    return M


def forgive_recent(S: np.ndarray, T: float, beta: int, transposed: bool = False) -> np.ndarray:
    """Sec. 3.3 "retention of recent tokens": for each token i and each of its beta most recent
    similar tokens j, S[i, j] is set to zero (both the text and the pseudo-code say so: token i's own
    average loses the entry).  ``transposed`` is the other direction, which is what the stated purpose
    (keep the most recent of a group of similar tokens) suggests: the entry S[j, i] of the recent
    partner j is zeroed instead, so the most recent copy stops looking redundant and older copies
    keep their full similarity."""
    M = recent_similar(S, T, beta)
    out = S.copy()
    out[M.T if transposed else M] = 0.0
    return out


def mean_similarity(k_cand: np.ndarray, T: float, beta: int, eps: float, transposed: bool = False) -> np.ndarray:
    """Eq. 6, first part: S-bar[i] = (1/n) sum_j S[i, j] after the zeroing above."""
    S = forgive_recent(cosine_similarity(k_cand, eps), T, beta, transposed)
    return S.sum(axis=1) / S.shape[0]


def mean_similarity_rows(k_cand: np.ndarray, rows, T: float, beta: int, eps: float) -> np.ndarray:
    """Eq. 5-6 for a few tokens only (sizes where the full n x n matrix is too large to hold):
    the same definition as ``mean_similarity``, one row of S at a time."""
    n = k_cand.shape[0]
    norm = np.sqrt((k_cand * k_cand).sum(axis=1, keepdims=True))
    kbar = k_cand / (norm + eps)
    out = []
    for i in rows:
        s = kbar @ kbar[i]                       # S[i, :]
        s[i] = 0.0
        similar = np.nonzero(s > T)[0]           # ascending, so the most recent are at the end
        if beta > 0:
            s[similar[-beta:]] = 0.0
        out.append(s.sum() / n)
    return np.array(out)


def redundancy(k_cand: np.ndarray, T: float, beta: int, eps: float) -> np.ndarray:
    """Eq. 6: R = softmax over the n candidates of S-bar."""
    return softmax_rows(mean_similarity(k_cand, T, beta, eps)[None, :])[0]


# -------------------------------------------------------------------- score and select
def selection_score(I: np.ndarray, R: np.ndarray, lam: float) -> np.ndarray:
    """Eq. 7: Z = lambda * I - (1 - lambda) * R."""
    return lam * I - (1.0 - lam) * R


def select_topk(Z: np.ndarray, k: int) -> np.ndarray:
    """The k candidates with the largest Z (equal scores: larger index first), ascending."""
    n = Z.shape[0]
    order = sorted(range(n), key=lambda i: (-Z[i], -i))
    return np.array(sorted(order[:k]), dtype=np.int64)


# ----------------------------------------------------------------------- one KV head
def compress_head(q_bits: np.ndarray, k_bits: np.ndarray, v_bits: np.ndarray, prm: Params):
    """One KV head: q_bits [G, alpha, d], k_bits / v_bits [N, d] (bf16 bit patterns).

    Returns a dict with importance, mean_sim, redundancy, score (each [n], float64),
    kept (the budget kept row indices: k selected ascending, then n..N-1) and the
    compacted k_out / v_out bit patterns [budget, d].
    """
    N = k_bits.shape[0]
    n = N - prm.alpha
    k_sel = prm.budget - prm.alpha
    q = decode_bf16(q_bits)
    k_cand = decode_bf16(k_bits[:n])
    I = (importance_mean_then_pool if prm.pool_after_mean else importance)(q, k_cand, prm.pool_w, prm.gqa)
    sbar = mean_similarity(k_cand, float(np.float32(prm.sim_threshold)), prm.beta, prm.eps, prm.recency_transposed)
    R = softmax_rows(sbar[None, :])[0]
    Z = selection_score(I, R, float(np.float32(prm.lam)))
    keep = select_topk(Z, k_sel)
    kept = np.concatenate([keep, np.arange(n, N, dtype=np.int64)])
    return dict(importance=I, mean_sim=sbar, redundancy=R, score=Z, kept=kept,
                k_out=k_bits[kept].copy(), v_out=v_bits[kept].copy())


def compress_problem(q_bits: np.ndarray, k_bits: np.ndarray, v_bits: np.ndarray, prm: Params):
    """One (sequence, layer) problem: q_bits [Hq, alpha, d], k_bits / v_bits [H, N, d].  Returns the list
    of per-head dicts of ``compress_head``.  With ``prm.shared_selection`` the selection follows the
    paper's pseudo-code: the per-head scores are averaged over the H heads and the k candidates with the
    largest average are kept in every head (each dict then also holds ``shared_score``)."""
    H, N = k_bits.shape[:2]
    G = q_bits.shape[0] // H
    heads = [compress_head(q_bits[h * G:(h + 1) * G], k_bits[h], v_bits[h], prm) for h in range(H)]
    if prm.shared_selection:
        n = N - prm.alpha
        zbar = np.mean(np.stack([hd["score"] for hd in heads]), axis=0)
        keep = select_topk(zbar, prm.budget - prm.alpha)
        kept = np.concatenate([keep, np.arange(n, N, dtype=np.int64)])
        for h, hd in enumerate(heads):
            hd["shared_score"] = zbar
            hd["kept"] = kept
            hd["k_out"] = k_bits[h][kept].copy()
            hd["v_out"] = v_bits[h][kept].copy()
    return heads


def compress(q_bits: np.ndarray, k_bits: np.ndarray, v_bits: np.ndarray, prm: Params, heads=None):
    """Batched form: q_bits [P, Hq, alpha, d], k_bits / v_bits [P, H, N, d].

    Query head hq serves KV head hq // G (contiguous groups).  ``heads`` optionally
    restricts the work to an iterable of (p, h) pairs; the result maps (p, h) to the
    dict of ``compress_head``.
    """
    P, H = k_bits.shape[:2]
    G = q_bits.shape[1] // H
    todo = [(p, h) for p in range(P) for h in range(H)] if heads is None else list(heads)
    return {(p, h): compress_head(q_bits[p, h * G:(h + 1) * G], k_bits[p, h], v_bits[p, h], prm)
            for (p, h) in todo}
