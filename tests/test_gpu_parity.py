"""Parity of the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Scores: |gpu - oracle| <= 1e-5 + 1e-3 |oracle| (rows whose threshold decision is within rounding
of T are exempt).  Kept indices: exactly the top-k of the GPU's own scores under (score desc,
index desc); against the oracle every candidate outside the tolerance band around the k-th score
must agree.  Compacted K/V: bit-exact given the indices."""
import numpy as np
import pytest
import torch

from oracle import rkv_oracle as O
from paper_2505_24133_amd import rkv, synth

import helpers as Hp

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    rkv.load_library()


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def host_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def shape_of(w: synth.Workload, P: int) -> rkv.Shape:
    return rkv.Shape(num_problems=P, kv_heads=w.kv_heads, q_heads=w.q_heads, n_tokens=w.n_tokens,
                     budget=w.budget, alpha=w.alpha, head_dim=w.head_dim, pool_w=w.pool_w, beta=w.beta,
                     sim_threshold=w.sim_threshold, lam=w.lam, eps=w.eps)


class Tally:
    """What a parity run left undecided, summed over the heads it checked."""
    def __init__(self):
        self.heads = self.fragile = self.free_sharp = self.free_band = self.k = 0
        self.term_err = 0.0

    def line(self):
        return (f"{self.heads} heads; score error relative to its terms <= {self.term_err:.1e}; kept lists: "
                f"{self.free_sharp} of {self.k} selections undecidable within that error "
                f"({self.free_band} inside the 1e-5 + 1e-3 |tau| band); {self.fragile} threshold-fragile rows exempt")


def check_head(w, ref, z_gpu, kept_gpu, kout, vout, kb, vb, tag, imp=None, red=None, msim=None,
               z_select=None, frag_select=None, transposed=False, tally=None):
    """Compare one head's GPU results with the oracle's dict `ref`.  With the shared selection the
    kept list is the top-k of `z_select` (the head mean of the GPU's scores, formed as the kernel
    forms it) and is compared with the oracle's `shared_score`; `frag_select` marks the candidates
    that are threshold-fragile in any head.

    Rows whose threshold decision is within rounding of T are exempt from the score comparisons; they are
    looked for (another n x n pass of the oracle's cosine matrix) only when a comparison fails."""
    n, k = w.n_cand, w.k_sel
    frag_cache = []

    def fragile():
        if not frag_cache:
            kc = O.decode_bf16(kb[:n])
            frag_cache.append((Hp.fragile_tokens_transposed if transposed else Hp.fragile_rows)(
                kc, float(np.float32(w.sim_threshold)), w.beta, w.eps))
        return frag_cache[0]

    def rows_close(gpu, want, what, **tol):
        bad = ~Hp.close(gpu, want, **tol)
        if bad.any():
            bad &= ~fragile()
        assert not bad.any(), f"{tag}: {what}, {bad.sum()} rows, max abs {np.abs(gpu - want)[bad].max()}"

    if imp is not None:
        assert Hp.close(imp, ref["importance"]).all(), f"{tag}: importance"
    if msim is not None:
        rows_close(msim, ref["mean_sim"], "mean_sim", rel=1e-3, abs_=2e-6)
    if red is not None:
        rows_close(red, ref["redundancy"], "redundancy")
    lam = float(np.float32(w.lam))
    scale = lam * np.abs(ref["importance"]) + (1 - lam) * np.abs(ref["redundancy"])
    if z_gpu is not None:
        rows_close(z_gpu, ref["score"], "score")
        # much sharper than the contract: error relative to the size of the two terms of Eq. 7
        rel = np.abs(z_gpu.astype(np.float64) - ref["score"]) / (scale + 1e-12)
        if (rel >= Hp.TERM_REL_ERR).any():
            rel[fragile()] = 0.0
        assert rel.max() < Hp.TERM_REL_ERR, f"{tag}: score err relative to its terms {rel.max()}"
        if tally is not None:
            tally.term_err = max(tally.term_err, float(rel.max()))
    if kept_gpu is not None:
        sel = kept_gpu[:k].astype(np.int64)
        assert np.all(np.diff(sel) > 0) and sel[0] >= 0 and sel[-1] < n, f"{tag}: kept order/range"
        np.testing.assert_array_equal(kept_gpu[k:], np.arange(n, w.n_tokens), err_msg=f"{tag}: observation rows")
        own = z_select if z_select is not None else z_gpu
        if own is not None:
            np.testing.assert_array_equal(sel, Hp.exact_topk(own, k), err_msg=f"{tag}: not the top-k of its own score")
        z_ref = ref["shared_score"] if z_select is not None else ref["score"]
        kept_mask = np.zeros(n, dtype=bool)
        kept_mask[sel] = True
        # (1) the sharp rule: given the score error asserted above, every candidate that any score vector
        # within that error must keep is kept, and every one it must drop is dropped
        err = Hp.TERM_REL_ERR * scale
        if frag_select is not None:
            err = np.where(frag_select, np.inf, err)
        must_keep, must_drop = Hp.decidable_selection(z_ref, err, k)
        if (must_keep & ~kept_mask).any() or (must_drop & kept_mask).any():
            skip_now = fragile() if frag_select is None else frag_select
            must_keep, must_drop = Hp.decidable_selection(z_ref, np.where(skip_now, np.inf, err), k)
        wrong = int((must_keep & ~kept_mask).sum()), int((must_drop & kept_mask).sum())
        assert wrong == (0, 0), f"{tag}: kept set vs oracle: {wrong[0]} missing, {wrong[1]} extra"
        free_sharp = int((~(must_keep | must_drop)).sum())
        # (2) the contract's band around the oracle's k-th score (much wider at these magnitudes)
        skip = frag_select if frag_select is not None else (frag_cache[0] if frag_cache else np.zeros(n, dtype=bool))
        mk, md, free = Hp.check_kept_against_oracle(sel, z_ref, k, skip)
        if mk or md:
            skip = fragile() if frag_select is None else frag_select
            mk, md, free = Hp.check_kept_against_oracle(sel, z_ref, k, skip)
        assert mk == 0 and md == 0, f"{tag}: kept set vs oracle: {mk} missing, {md} extra (free {free})"
        # and against the oracle's own list: the two may differ only in candidates the sharp rule leaves open
        theirs = ref["kept"][:k]
        odd = np.array(sorted(set(sel.tolist()) ^ set(theirs.tolist())), dtype=np.int64)
        loose = ~(must_keep | must_drop)[odd]
        assert loose.all(), f"{tag}: differs from the oracle's kept list at {odd[~loose][:8]}"
        np.testing.assert_array_equal(kept_gpu[k:], ref["kept"][k:], err_msg=f"{tag}: observation rows vs oracle")
        if kout is not None and np.array_equal(kept_gpu, ref["kept"]):
            np.testing.assert_array_equal(kout, ref["k_out"], err_msg=f"{tag}: K_out vs oracle")
            np.testing.assert_array_equal(vout, ref["v_out"], err_msg=f"{tag}: V_out vs oracle")
        if kout is not None:
            np.testing.assert_array_equal(kout, kb[kept_gpu], err_msg=f"{tag}: K_out")
            np.testing.assert_array_equal(vout, vb[kept_gpu], err_msg=f"{tag}: V_out")
        if tally is not None:
            tally.free_sharp += free_sharp
            tally.free_band += free
            tally.k += k
    if tally is not None:
        tally.heads += 1
        tally.fragile += int(frag_cache[0].sum()) if frag_cache else 0
    return int(frag_cache[0].sum()) if frag_cache else 0


def head_mean_fp32(z):
    """Mean over the heads of z [H, n] as the shared-selection kernel forms it: fp32 running sum over
    ascending h, times fp32(1 / H)."""
    s = np.zeros(z.shape[1], dtype=np.float32)
    for h in range(z.shape[0]):
        s = s + z[h].astype(np.float32)
    return s * np.float32(1.0 / z.shape[0])


def check_outputs(w, q, k, v, heads, idx_h, score_h, ko_h, vo_h, tag, flags=0, parts=None, pooled=False,
                  max_free=None):
    """Compare the listed (p, h) heads of host copies of rkv_compress outputs (of any entry point that
    produces them) with the oracle.  `pooled`: q, k, v are exactly synth.make_batch(w) of a seeded
    workload, so the oracle may run in worker processes that draw the same inputs themselves."""
    shared = bool(flags & rkv.RKV_FLAG_SHARED_SELECTION)
    gqa = ("softmax_max" if flags & rkv.RKV_FLAG_GQA_SOFTMAX_THEN_MAX else
           "softmax_mean" if flags & rkv.RKV_FLAG_GQA_SOFTMAX_THEN_MEAN else "max_logits")
    transposed = bool(flags & rkv.RKV_FLAG_RECENCY_TRANSPOSED)
    variant = dict(pool_after_mean=bool(flags & rkv.RKV_FLAG_POOL_AFTER_MEAN), shared_selection=shared, gqa=gqa,
                   recency_transposed=transposed)
    prm = Hp.oracle_params(w, **variant)
    frag_of = Hp.fragile_tokens_transposed if transposed else Hp.fragile_rows
    G = w.group
    tally = Tally()
    if shared:
        n = w.n_cand
        for p in sorted({p for (p, _) in heads}):
            refs = O.compress_problem(q[p], k[p], v[p], prm)
            frag_any = np.zeros(n, dtype=bool)
            for h in range(w.kv_heads):
                frag_any |= frag_of(O.decode_bf16(k[p, h, :n]), float(np.float32(w.sim_threshold)), w.beta, w.eps)
            zbar = head_mean_fp32(score_h[p])
            for h in range(w.kv_heads):
                assert np.array_equal(idx_h[p, h], idx_h[p, 0]), f"{tag}[p{p}]: heads hold different kept lists"
                extra = {}
                if parts is not None:
                    extra = dict(imp=parts[0][p, h], red=parts[1][p, h], msim=parts[2][p, h])
                check_head(w, refs[h], score_h[p, h], idx_h[p, h], ko_h[p, h], vo_h[p, h], k[p, h], v[p, h],
                           f"{tag}[p{p},h{h}]", z_select=zbar, frag_select=frag_any, transposed=transposed,
                           tally=tally, **extra)
        say(f"{tag}: shared selection matches: {tally.line()}")
        return tally
    if pooled:
        refs = Hp.oracle_heads(w, heads, **variant)
    else:
        refs = (((p, h), O.compress_head(q[p, h * G:(h + 1) * G], k[p, h], v[p, h], prm)) for (p, h) in heads)
    for (p, h), ref in refs:
        extra = {}
        if parts is not None:
            extra = dict(imp=parts[0][p, h], red=parts[1][p, h], msim=parts[2][p, h])
        check_head(w, ref, score_h[p, h], idx_h[p, h], ko_h[p, h], vo_h[p, h], k[p, h], v[p, h],
                   f"{tag}[p{p},h{h}]", transposed=transposed, tally=tally, **extra)
        if tally.heads % 256 == 0:
            say(f"{tag}: {tally.heads} of {len(heads)} heads checked")
    assert tally.heads == len(heads)
    say(f"{tag}: all match: {tally.line()}")
    if max_free is not None:
        # the comparison of the kept lists has teeth: what the asserted score error leaves undecidable is a
        # small, stated share of the selections
        assert tally.free_sharp <= max_free * tally.k, tally.line()
    return tally


def run_fused(w, q, k, v, heads, tag, check_parts=False, flags=0, pooled=False, max_free=None):
    """q,k,v: uint16 [P,...].  Runs rkv_compress (and optionally every stand-alone entry point) and
    checks the listed (p, h) heads against the oracle.  With RKV_FLAG_SHARED_SELECTION every head of
    the problems named in `heads` is checked."""
    P = k.shape[0]
    shp = shape_of(w, P)
    shp.flags = flags
    say(f"{tag}: rkv_compress P={P} H={w.kv_heads} N={w.n_tokens} budget={w.budget} G={w.group} "
        f"alpha={w.alpha} W={w.pool_w} beta={w.beta} T={w.sim_threshold} lam={w.lam}")
    qd, kd, vd = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    st, ko, vo, idx, score = rkv.rkv_compress(shp, qd, kd, vd, want_idx=True, want_score=True)
    torch.cuda.synchronize()
    assert st == rkv.RKV_OK
    parts = None
    if check_parts:
        say(f"{tag}: stand-alone entry points")
        imp = rkv.rkv_score_importance(shp, qd, kd)
        red, msim = rkv.rkv_score_redundancy(shp, kd, want_mean_sim=True)
        kept2, score2 = rkv.rkv_select_topk(shp, imp, red, want_score=True)
        ko2, vo2 = rkv.rkv_compact(shp, kd, vd, kept2)
        torch.cuda.synchronize()
        assert torch.equal(kept2, idx) and torch.equal(score2, score), f"{tag}: fused != staged"
        assert torch.equal(ko2, ko) and torch.equal(vo2, vo)
        parts = (imp.cpu().numpy(), red.cpu().numpy(), msim.cpu().numpy())
    check_outputs(w, q, k, v, heads, idx.cpu().numpy(), score.cpu().numpy(), host_bits(ko), host_bits(vo), tag,
                  flags=flags, parts=parts, pooled=pooled, max_free=max_free)
    return idx, score, ko, vo


# ------------------------------------------------------------------------------ configs
def test_cfg1_tiny_all_entry_points():
    w = synth.CONFIGS["cfg1_tiny"]
    q, k, v = synth.make_batch(w)
    run_fused(w, q, k, v, [(0, 0), (0, 1)], "cfg1", check_parts=True)


ADVERSARIAL = [
    # N, budget, kv_heads, G, alpha, W, beta, T, lam
    (203, 120, 2, 4, 8, 4, 1, 0.5, 0.1),      # ragged: n = 195 is no multiple of any tile
    (129, 100, 1, 1, 8, 0, 0, 0.5, 0.1),      # MHA, no pooling, nothing forgiven
    (300, 40, 2, 5, 8, 1, 2, 0.3, 0.1),       # G = 5 (40 query rows -> two MFMA row tiles)
    (260, 250, 2, 4, 1, 2, 8, 0.95, 0.5),     # alpha = 1, few evictions
    (452, 300, 1, 5, 12, 7, 1, 1.0, 0.0),     # 60 query rows, T = 1 (never exceeded), lambda = 0
    (577, 320, 3, 2, 8, 4, 4, 0.0, 1.0),      # T = 0: every positive similarity is a hit; lambda = 1
    (65, 17, 2, 4, 8, 4, 1, 0.5, 0.1),        # smaller than one tile
    (1030, 999, 1, 4, 8, 16, 3, 0.8, 0.05),   # wide pooling window
    (300, 200, 1, 1, 64, 3, 1, 0.5, 0.1),     # alpha = 64, the largest observation window (MHA)
    (390, 257, 1, 2, 32, 0, 64, 0.4, 0.2),    # G * alpha = 64 rows, beta larger than any hit count
    (700, 650, 1, 4, 8, 400, 1, 0.5, 0.3),    # pooling window wider than the cache
    (2100, 1900, 1, 4, 8, 4, 2, 0.5, 0.1),    # more than one staging block in the pooling stage
    (500, 300, 2, 2, 16, 3, 1, 0.5, 0.1),     # alpha = 16, G = 2: the pre-pass's register path, 8 values per lane
    (333, 200, 1, 1, 32, 2, 1, 0.5, 0.2),     # alpha = 32, MHA: register path, 16 values per lane
    (420, 300, 2, 1, 8, 4, 1, 0.5, 0.1),      # alpha = 8, MHA: register path with a single head per group
    (150, 100, 1, 2, 8, 4, 1, 0.5, 0.1),      # n = 142: the last chunk's third and fourth 32-key groups are empty
    (410, 300, 2, 3, 16, 3, 1, 0.5, 0.1),     # alpha = 16, G = 3: register path over two query row tiles
    (410, 300, 1, 8, 8, 4, 1, 0.5, 0.1),      # alpha = 8, G = 8: 64 query rows, register path over two row tiles
    (2300, 2000, 1, 4, 8, 1000, 1, 0.5, 0.1),  # the widest pooling window (2W = 2000): few columns per staging block
    (1100, 900, 1, 1, 64, 120, 1, 0.5, 0.1),   # alpha = 64 with 2W = 240: 56 columns per staging block, 19 blocks
    (900, 700, 1, 2, 8, 3, 1, 0.5, 0.1),       # W odd: the pooling window is not a multiple of four entries
    (5000, 4600, 2, 4, 8, 4, 1, 0.5, 0.1),     # two heads of 4992 candidates: one large staging block each
    (600, 9, 2, 4, 8, 4, 1, 0.5, 0.1),         # a single candidate is kept (k = 1)
    (600, 599, 2, 4, 8, 4, 1, 0.5, 0.1),       # a single candidate is evicted (k = n - 1)
    (140, 139, 1, 2, 8, 2, 2, 0.5, 0.9),       # the same within one and a bit tiles
]


@pytest.mark.parametrize("case", ADVERSARIAL, ids=lambda c: f"N{c[0]}_b{c[1]}_G{c[3]}_a{c[4]}_W{c[5]}_beta{c[6]}_T{c[7]}")
def test_adversarial_shapes(case):
    N, budget, H, G, alpha, W, beta, T, lam = case
    w = synth.Workload("adv", 2, H, H * G, N, budget, alpha=alpha, pool_w=W, beta=beta, sim_threshold=T,
                       lam=lam, seed=77 + N, recipe="rowcopy", redundancy=0.35, copy_noise=0.15)
    q, k, v = synth.make_batch(w)
    run_fused(w, q, k, v, [(p, h) for p in range(2) for h in range(H)], f"adv{N}", check_parts=True)


VARIANT_SHAPES = [
    # N, budget, kv_heads, G, alpha, W, beta, T, lam
    (203, 120, 2, 4, 8, 4, 1, 0.5, 0.1),
    (452, 300, 3, 5, 12, 7, 1, 0.6, 0.3),
    (300, 200, 1, 1, 63, 3, 1, 0.5, 0.1),      # alpha + 1 = 64 rows in the pooling stage
    (700, 650, 2, 4, 8, 400, 1, 0.5, 0.3),     # pooling window wider than the cache
    (2100, 1900, 4, 2, 8, 4, 2, 0.5, 0.1),     # more than one staging block
    (260, 250, 5, 1, 4, 0, 0, 0.5, 0.5),       # no pooling, five heads averaged
    (390, 257, 2, 2, 32, 2, 1, 0.4, 0.2),      # G * alpha = 64 logit rows per head
    (600, 500, 1, 1, 63, 128, 1, 0.5, 0.1),    # (alpha + 1) * 2W = 16384: the largest window the mean-then-pool order takes
]
VARIANT_FLAGS = {"mean_then_pool": 2, "shared": 4, "both": 6, "gqa_softmax_max": 8, "gqa_softmax_mean": 16,
                 "gqa_softmax_max_mean_then_pool_shared": 14, "gqa_softmax_mean_mean_then_pool": 18,
                 "recency_transposed": 32, "recency_transposed_shared_skip_saturated": 37}


@pytest.mark.parametrize("variant", sorted(VARIANT_FLAGS))
@pytest.mark.parametrize("case", VARIANT_SHAPES, ids=lambda c: f"N{c[0]}_H{c[2]}_G{c[3]}_a{c[4]}_W{c[5]}")
def test_pseudo_code_variants(case, variant):
    """The places where the paper's pseudo-code or appendix differ from its equations: mean over the
    query rows before the pooling, one selection per problem from the head-averaged score, the
    query heads of a group merged after their softmax (max or mean), and the keep-recent rule
    charged to the recent partner instead of the token itself."""
    N, budget, H, G, alpha, W, beta, T, lam = case
    flags = VARIANT_FLAGS[variant]
    assert (rkv.RKV_FLAG_POOL_AFTER_MEAN, rkv.RKV_FLAG_SHARED_SELECTION, rkv.RKV_FLAG_GQA_SOFTMAX_THEN_MAX,
            rkv.RKV_FLAG_GQA_SOFTMAX_THEN_MEAN, rkv.RKV_FLAG_RECENCY_TRANSPOSED, rkv.RKV_FLAG_SKIP_SATURATED) == (2, 4, 8, 16, 32, 1)
    w = synth.Workload("var", 2, H, H * G, N, budget, alpha=alpha, pool_w=W, beta=beta, sim_threshold=T,
                       lam=lam, seed=500 + N, recipe="rowcopy", redundancy=0.35, copy_noise=0.15)
    q, k, v = synth.make_batch(w)
    run_fused(w, q, k, v, [(p, h) for p in range(2) for h in range(H)], f"{variant}{N}", check_parts=True, flags=flags)


TRIANGULAR_SHAPES = [c for c in ADVERSARIAL if c[6] == 1] + [
    # N, budget, kv_heads, G, alpha, W, beta, T, lam
    (392, 300, 2, 4, 8, 4, 1, 0.5, 0.1),      # exactly one row block (384 candidates)
    (393, 300, 2, 4, 8, 4, 1, 0.9, 0.1),      # one candidate in a second row block
    (1300, 1100, 3, 4, 8, 4, 1, 0.0, 0.1),    # T = 0: every positive similarity counts
    (1300, 1100, 1, 4, 8, 4, 1, 1.0, 0.1),    # T = 1: nothing ever counts
]


@pytest.mark.parametrize("case", TRIANGULAR_SHAPES, ids=lambda c: f"N{c[0]}_b{c[1]}_G{c[3]}_a{c[4]}_W{c[5]}_T{c[7]}")
def test_triangular_scan_gives_the_default_rule(case):
    """RKV_FLAG_TRIANGULAR_SCAN is another schedule of the similarity pass (entries with j < i only, each
    reported to both of its tokens), not another rule: its results are compared with the same oracle."""
    N, budget, H, G, alpha, W, beta, T, lam = case
    w = synth.Workload("tri", 2, H, H * G, N, budget, alpha=alpha, pool_w=W, beta=beta, sim_threshold=T,
                       lam=lam, seed=300 + N, recipe="rowcopy", redundancy=0.35, copy_noise=0.15)
    q, k, v = synth.make_batch(w)
    run_fused(w, q, k, v, [(p, h) for p in range(2) for h in range(H)], f"tri{N}", check_parts=True,
              flags=rkv.RKV_FLAG_TRIANGULAR_SCAN)


def test_triangular_scan_on_benchmark_shapes():
    """cfg2 at T = 0.95 (entries above T are rare: the case the schedule is for) and at T = 0.5, cfg3's long
    heads, all heads of the problems drawn against the oracle; and the scores next to the default schedule's."""
    for w in (synth.scaled(synth.CONFIGS["cfg2_llama8b_b1024"], num_problems=4, sim_threshold=0.95),
              synth.scaled(synth.CONFIGS["cfg2_llama8b_b1024"], num_problems=2),
              synth.scaled(synth.CONFIGS["cfg3_llama8b_b4096"], num_problems=1, sim_threshold=0.9)):
        q, k, v = synth.make_batch(w)
        heads = [(p, h) for p in range(w.num_problems) for h in range(w.kv_heads)]
        idx, score, ko, vo = run_fused(w, q, k, v, heads, f"tri_{w.name}_T{w.sim_threshold}", flags=rkv.RKV_FLAG_TRIANGULAR_SCAN)
        st, ko2, vo2, idx2, score2 = rkv.rkv_compress(shape_of(w, w.num_problems), dev_bf16(q), dev_bf16(k), dev_bf16(v), want_score=True)
        torch.cuda.synchronize()
        a, b = score.cpu().numpy().astype(np.float64), score2.cpu().numpy().astype(np.float64)
        assert np.max(np.abs(a - b) / (np.abs(b) + 1e-12)) < 1e-4       # same rule; the last operations differ in order


def test_pseudo_code_variants_cfg2_full_size():
    """Both variants at the benchmark's launch shape; four problems (32 heads) against the oracle."""
    w = synth.CONFIGS["cfg2_llama8b_b1024"]
    q, k, v = synth.make_batch(w)
    flags = rkv.RKV_FLAG_POOL_AFTER_MEAN | rkv.RKV_FLAG_SHARED_SELECTION
    run_fused(w, q, k, v, [(p, 0) for p in (0, 9, 18, 31)], "cfg2_variants", flags=flags)
    run_fused(w, q, k, v, [(p, h) for p in (3, 30) for h in range(8)], "cfg2_gqa_softmax_max",
              flags=rkv.RKV_FLAG_GQA_SOFTMAX_THEN_MAX)
    run_fused(w, q, k, v, [(p, h) for p in (5, 17) for h in range(8)], "cfg2_gqa_softmax_mean",
              flags=rkv.RKV_FLAG_GQA_SOFTMAX_THEN_MEAN)
    idx1, score1, *_ = run_fused(w, q, k, v, [(p, h) for p in (1, 2, 29) for h in range(8)], "cfg2_recency_transposed",
                                 flags=rkv.RKV_FLAG_RECENCY_TRANSPOSED)
    # integer accumulation of the charged similarities: the result does not depend on the arrival order
    idx2, score2, *_ = run_fused(w, q, k, v, [(11, 4)], "cfg2_recency_transposed_again", flags=rkv.RKV_FLAG_RECENCY_TRANSPOSED)
    assert torch.equal(idx1, idx2) and torch.equal(score1, score2)


def test_cfg2_llama8b_full_size_all_heads():
    w = synth.CONFIGS["cfg2_llama8b_b1024"]
    q, k, v = synth.make_batch(w, workers=Hp.oracle_workers())
    run_fused(w, q, k, v, [(p, h) for p in range(w.num_problems) for h in range(w.kv_heads)], "cfg2", pooled=True, max_free=0.02)


def test_cfg2_high_threshold():
    """T = 0.95: only true near-duplicates exceed the threshold, most rows never saturate."""
    w = synth.scaled(synth.CONFIGS["cfg2_llama8b_b1024"], sim_threshold=0.95, num_problems=4)
    q, k, v = synth.make_batch(w)
    run_fused(w, q, k, v, [(p, h) for p in range(4) for h in range(0, 8, 3)], "cfg2_T095", check_parts=True)


def test_cfg3_llama8b_budget4096_full_size_all_heads():
    """All 32 x 8 = 256 heads of the configuration against the oracle (worker processes)."""
    w = synth.CONFIGS["cfg3_llama8b_b4096"]
    q, k, v = synth.make_batch(w, workers=Hp.oracle_workers())
    run_fused(w, q, k, v, [(p, h) for p in range(w.num_problems) for h in range(w.kv_heads)], "cfg3", pooled=True, max_free=0.02)


def test_cfg4_qwen14b_full_size_all_heads():
    """The configuration as written: 16 sequences x 48 layers = 768 problems, each drawn from its own seed
    (redundancy level per sequence), one launch; all 6144 heads against the oracle."""
    w = synth.CONFIGS["cfg4_qwen14b_b2048_bs16"]
    q, k, v = synth.make_batch(w, workers=Hp.oracle_workers())
    assert k.shape[0] == w.num_problems == 768
    heads = [(p, h) for p in range(w.num_problems) for h in range(w.kv_heads)]
    idx, score, ko, vo = run_fused(w, q, k, v, heads, "cfg4", pooled=True, max_free=0.02)
    _self_consistent_everywhere(w, k, v, idx, score, ko, vo, "cfg4")


def test_cfg5_long_trace_full_size_all_heads():
    """4 sequences x 32 layers = 128 problems of N = 8320, each from its own seed, one launch; all 1024
    heads against the oracle."""
    w = synth.CONFIGS["cfg5_llama8b_b8192_bs4"]
    q, k, v = synth.make_batch(w, workers=Hp.oracle_workers())
    assert k.shape[0] == w.num_problems == 128
    heads = [(p, h) for p in range(w.num_problems) for h in range(w.kv_heads)]
    idx, score, ko, vo = run_fused(w, q, k, v, heads, "cfg5", pooled=True, max_free=0.02)
    _self_consistent_everywhere(w, k, v, idx, score, ko, vo, "cfg5")


def _self_consistent_everywhere(w, k, v, idx, score, ko, vo, tag):
    """What can be said of every head without the oracle: the kept list is the exact top-k of the head's
    own scores (ties towards the larger index) followed by the observation rows, and the compacted rows
    are those rows of the inputs, bit for bit."""
    n, ksel = w.n_cand, w.k_sel
    P, H = idx.shape[:2]
    for p in range(P):
        idx_h, z_h = idx[p].cpu().numpy(), score[p].cpu().numpy()
        ko_h, vo_h = host_bits(ko[p]), host_bits(vo[p])
        for h in range(H):
            np.testing.assert_array_equal(idx_h[h, :ksel], Hp.exact_topk(z_h[h], ksel), err_msg=f"{tag}[p{p},h{h}]")
            np.testing.assert_array_equal(idx_h[h, ksel:], np.arange(n, w.n_tokens))
            assert np.array_equal(ko_h[h], k[p, h][idx_h[h]]) and np.array_equal(vo_h[h], v[p, h][idx_h[h]]), f"{tag}[p{p},h{h}]"
    say(f"{tag}: all {P * H} heads keep the exact top-k of their own scores and hold the gathered rows")


# --------------------------------------------------------------------------- properties
def test_bit_identical_on_repeat_and_on_another_stream():
    w = synth.scaled(synth.CONFIGS["cfg2_llama8b_b1024"], num_problems=3)
    q, k, v = synth.make_batch(w)
    shp = shape_of(w, 3)
    qd, kd, vd = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    say("repeat: default stream twice, then a side stream")
    a = rkv.rkv_compress(shp, qd, kd, vd, want_score=True)
    b = rkv.rkv_compress(shp, qd, kd, vd, want_score=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        c = rkv.rkv_compress(shp, qd, kd, vd, want_score=True)
    side.synchronize()
    torch.cuda.synchronize()
    for other in (b, c):
        for x, y in zip(a[1:], other[1:]):
            assert torch.equal(x, y)


def test_results_do_not_depend_on_how_the_similarity_pass_is_scheduled():
    """With few heads the column scan of every row block is shared by several workgroups and the finalize
    kernel finishes the mean similarity; with many heads one workgroup does it all.  Both finish it with
    the same sequence of rounded operations, so a problem gives the same bits alone and inside a batch."""
    w = synth.CONFIGS["cfg2_llama8b_b1024"]
    q, k, v = synth.make_batch(w, workers=Hp.oracle_workers())
    qd, kd, vd = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    say("full batch (one workgroup per row block) vs two problems alone (split column scan)")
    full = shape_of(w, w.num_problems)
    red_a, msim_a = rkv.rkv_score_redundancy(full, kd, want_mean_sim=True)
    out_a = rkv.rkv_compress(full, qd, kd, vd, want_score=True)
    few = shape_of(w, 2)
    red_b, msim_b = rkv.rkv_score_redundancy(few, kd[5:7].contiguous(), want_mean_sim=True)
    out_b = rkv.rkv_compress(few, qd[5:7].contiguous(), kd[5:7].contiguous(), vd[5:7].contiguous(), want_score=True)
    torch.cuda.synchronize()
    assert torch.equal(msim_a[5:7], msim_b) and torch.equal(red_a[5:7], red_b)
    for x, y in zip(out_a[1:], out_b[1:]):
        assert torch.equal(x[5:7], y)


def test_strided_cache_views():
    """K/V given as views of a larger [P, H, N_alloc, d] allocation (static cache with spare rows)."""
    w = synth.scaled(synth.CONFIGS["cfg1_tiny"], num_problems=2, kv_heads=2)
    q, k, v = synth.make_batch(w)
    shp = shape_of(w, 2)
    qd = dev_bf16(q)
    big_k = torch.zeros((2, 2, w.n_tokens + 40, 128), dtype=torch.bfloat16, device="cuda")
    big_v = torch.zeros((2, 2, w.n_tokens + 72, 128), dtype=torch.bfloat16, device="cuda")
    big_k[:, :, :w.n_tokens] = dev_bf16(k)
    big_v[:, :, :w.n_tokens] = dev_bf16(v)
    say("strided views")
    a = rkv.rkv_compress(shp, qd, big_k[:, :, :w.n_tokens], big_v[:, :, :w.n_tokens], want_score=True)
    b = rkv.rkv_compress(shp, qd, dev_bf16(k), dev_bf16(v), want_score=True)
    torch.cuda.synchronize()
    for x, y in zip(a[1:], b[1:]):
        assert torch.equal(x, y)


def test_strided_observation_queries():
    """q_obs given as a view of a query cache laid out [P, alpha, q_heads, d] (and with spare heads): the
    strides in rkv_params reach every entry point that reads or writes the queries."""
    w = synth.scaled(synth.CONFIGS["cfg1_tiny"], num_problems=2, kv_heads=2, q_heads=10)      # G = 5: two query row tiles
    q, k, v = synth.make_batch(w)
    shp = shape_of(w, 2)
    qd, kd, vd = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    cache = torch.zeros((2, w.alpha, w.q_heads + 3, 128), dtype=torch.bfloat16, device="cuda")
    qview = cache[:, :, :w.q_heads].permute(0, 2, 1, 3)            # [P, q_heads, alpha, d], nothing contiguous but d
    qview.copy_(qd)
    assert not qview.is_contiguous()
    say("strided q_obs")
    a = rkv.rkv_compress(shp, qd, kd, vd, want_score=True)
    b = rkv.rkv_compress(shp, qview, kd, vd, want_score=True)
    ia, ib = rkv.rkv_score_importance(shp, qd, kd), rkv.rkv_score_importance(shp, qview, kd)
    torch.cuda.synchronize()
    assert torch.equal(ia, ib)
    for x, y in zip(a[1:], b[1:]):
        assert torch.equal(x, y)
    # append through the strides: the new query rows land in their slot of the strided cache only
    newq = dev_bf16(synth.f32_to_bf16_bits(np.random.default_rng(8).standard_normal((2, w.q_heads, 128)).astype(np.float32)))
    newk = torch.zeros((2, w.kv_heads, 128), dtype=torch.bfloat16, device="cuda")
    before = cache.clone()
    rkv.rkv_cache_append(shp, kd.clone(), vd.clone(), qview, newk, newk, newq, 5, 3)
    torch.cuda.synchronize()
    assert torch.equal(cache[:, 3, :w.q_heads], newq)
    cache[:, 3, :w.q_heads] = before[:, 3, :w.q_heads]
    assert torch.equal(cache, before)


def test_exact_duplicates_only_one_copy_survives():
    """m exact copies of one key among otherwise orthogonal keys, lambda = 0, m - 1 evictions:
    the older copies go and the newest stays (tie-break towards the recent token)."""
    m, alpha, n = 4, 8, 120
    N = n + alpha
    kf = np.zeros((1, 1, N, 128), dtype=np.float32)
    pos = [5, 40, 77, 101]
    free = iter(range(1, 128))
    for i in range(N):
        if i in pos:
            kf[0, 0, i, 0] = 2.0
        else:
            kf[0, 0, i, next(free) if i < 120 else 127 - (i - 120)] = 1.0 + 0.01 * i
    rng = np.random.default_rng(5)
    q = synth.f32_to_bf16_bits(rng.standard_normal((1, 4, alpha, 128)).astype(np.float32))
    k = synth.f32_to_bf16_bits(kf)
    v = synth.f32_to_bf16_bits(rng.standard_normal((1, 1, N, 128)).astype(np.float32))
    w = synth.Workload("dups", 1, 1, 4, N, n - (m - 1) + alpha, alpha=alpha, pool_w=0, beta=1,
                       sim_threshold=0.5, lam=0.0)
    idx, score, ko, vo = run_fused(w, q, k, v, [(0, 0)], "dups")
    kept = set(idx[0, 0].cpu().numpy().tolist())
    assert [p in kept for p in pos] == [False, False, False, True]
    # with the rule charged to the recent partner the same outcome needs no tie-break: the newest
    # copy has strictly the lowest redundancy of the four, the second newest the next lowest
    idx, score, ko, vo = run_fused(w, q, k, v, [(0, 0)], "dups_transposed", flags=rkv.RKV_FLAG_RECENCY_TRANSPOSED)
    kept = set(idx[0, 0].cpu().numpy().tolist())
    assert [p in kept for p in pos] == [False, False, False, True]
    z = score[0, 0].cpu().numpy()
    assert z[101] > z[77] > z[40] and abs(z[40] - z[5]) < 1e-7 and abs(z[101] - z[0]) < 1e-6


def test_lambda_one_is_attention_only_selection():
    w = synth.scaled(synth.CONFIGS["cfg1_tiny"], lam=1.0)
    q, k, v = synth.make_batch(w)
    shp = shape_of(w, 1)
    qd, kd, vd = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    say("lambda = 1")
    imp = rkv.rkv_score_importance(shp, qd, kd)
    st, ko, vo, idx, score = rkv.rkv_compress(shp, qd, kd, vd, want_score=True)
    torch.cuda.synchronize()
    assert torch.equal(imp, score)
    for h in range(w.kv_heads):
        np.testing.assert_array_equal(idx[0, h, :w.k_sel].cpu().numpy(), Hp.exact_topk(imp[0, h].cpu().numpy(), w.k_sel))


def test_select_topk_ties_and_maximum_size():
    """rkv_select_topk alone: heavy ties, all-equal scores, and the largest supported N."""
    for (N, budget, levels) in [(32768, 20000, 7), (32768, 32000, 1), (5000, 4999, 3), (600, 9, 2)]:
        alpha = 8
        n = N - alpha
        shp = rkv.Shape(num_problems=1, kv_heads=3, q_heads=3, n_tokens=N, budget=budget, alpha=alpha, lam=0.25)
        g = torch.Generator().manual_seed(N + levels)
        imp = torch.randint(0, levels, (1, 3, n), generator=g).float() / 64.0
        red = torch.randint(0, levels, (1, 3, n), generator=g).float() / 64.0
        say(f"select N={N} budget={budget} levels={levels}")
        kept, score = rkv.rkv_select_topk(shp, imp.cuda(), red.cuda(), want_score=True)
        torch.cuda.synchronize()
        z = score.cpu().numpy()
        zr = np.float32(0.25) * imp.numpy() - (np.float32(1.0) - np.float32(0.25)) * red.numpy()
        np.testing.assert_allclose(z, zr, rtol=1e-6, atol=1e-9)
        for h in range(3):
            kh = kept[0, h].cpu().numpy()
            np.testing.assert_array_equal(kh[:budget - alpha], Hp.exact_topk(z[0, h], budget - alpha))
            np.testing.assert_array_equal(kh[budget - alpha:], np.arange(n, N))


def test_compact_arbitrary_indices():
    P, H, N, budget = 2, 3, 500, 333
    shp = rkv.Shape(num_problems=P, kv_heads=H, q_heads=H, n_tokens=N, budget=budget)
    g = torch.Generator().manual_seed(3)
    k = torch.randn((P, H, N, 128), generator=g).to(torch.bfloat16).cuda()
    v = torch.randn((P, H, N, 128), generator=g).to(torch.bfloat16).cuda()
    idx = torch.randint(0, N, (P, H, budget), generator=g, dtype=torch.int32)
    idx[0, 0, 0] = -5          # clamped to 0
    idx[1, 2, 7] = N + 100     # clamped to N - 1
    say("compact")
    ko, vo = rkv.rkv_compact(shp, k, v, idx.cuda())
    torch.cuda.synchronize()
    ci = idx.clamp(0, N - 1).long().cuda()
    ref_k = torch.gather(k, 2, ci[..., None].expand(-1, -1, -1, 128))
    ref_v = torch.gather(v, 2, ci[..., None].expand(-1, -1, -1, 128))
    assert torch.equal(ko, ref_k) and torch.equal(vo, ref_v)


def test_not_triggered_leaves_outputs_untouched():
    shp = rkv.Shape(num_problems=1, kv_heads=2, q_heads=8, n_tokens=256, budget=256)
    k = torch.randn((1, 2, 256, 128)).to(torch.bfloat16).cuda()
    q = torch.randn((1, 8, 8, 128)).to(torch.bfloat16).cuda()
    ko = torch.full((1, 2, 256, 128), 7.0, dtype=torch.bfloat16, device="cuda")
    vo = ko.clone()
    say("not triggered")
    st, ko2, vo2, idx, _ = rkv.rkv_compress(shp, q, k, k, k_out=ko, v_out=vo)
    torch.cuda.synchronize()
    assert st == rkv.RKV_NOT_TRIGGERED
    assert bool((ko == 7.0).all()) and bool((vo == 7.0).all())


# ------------------------------------------------------------------------- degenerate inputs
def _custom(kf, qf, vf, **kw):
    """float32 arrays [P,H,N,d], [P,Hq,alpha,d] -> workload + bf16 bit arrays."""
    P, H, N, d = kf.shape
    w = synth.Workload("custom", P, H, qf.shape[1], N, kw.pop("budget"), alpha=qf.shape[2], **kw)
    return w, synth.f32_to_bf16_bits(qf), synth.f32_to_bf16_bits(kf), synth.f32_to_bf16_bits(vf)


def test_smallest_problem():
    """n = 2 candidates, k = 1 selected."""
    rng = np.random.default_rng(21)
    kf = rng.standard_normal((3, 2, 10, 128)).astype(np.float32)
    qf = rng.standard_normal((3, 8, 8, 128)).astype(np.float32)
    w, q, k, v = _custom(kf, qf, kf[::-1].copy(), budget=9, pool_w=4, beta=1, sim_threshold=0.5, lam=0.1)
    run_fused(w, q, k, v, [(p, h) for p in range(3) for h in range(2)], "tiny", check_parts=True)


def test_all_keys_identical():
    """Every pair is a hit (S = 1 up to eps); beta = 2 forgives the two most recent partners of each row."""
    rng = np.random.default_rng(22)
    row = rng.standard_normal(128).astype(np.float32)
    kf = np.tile(row, (1, 1, 300, 1)).astype(np.float32)
    qf = rng.standard_normal((1, 4, 8, 128)).astype(np.float32)
    vf = rng.standard_normal((1, 1, 300, 128)).astype(np.float32)
    w, q, k, v = _custom(kf, qf, vf, budget=200, pool_w=2, beta=2, sim_threshold=0.9, lam=0.0)
    idx, score, ko, vo = run_fused(w, q, k, v, [(0, 0)], "identical", check_parts=True)
    # all scores equal -> the most recent candidates are kept
    np.testing.assert_array_equal(idx[0, 0].cpu().numpy(), np.arange(100, 300))


def test_zero_rows_and_large_magnitudes():
    rng = np.random.default_rng(23)
    kf = rng.standard_normal((1, 2, 260, 128)).astype(np.float32)
    kf[0, 0, [0, 17, 100, 251]] = 0.0                 # zero keys: similarity 0 to everything (eps keeps it finite)
    kf[0, 1, 40:60] *= 3.0e4                          # large rows
    kf[0, 1, 70:75] *= 1.0e-6                         # tiny rows
    kf[0, 1, 200] = kf[0, 1, 50] * 2.0                # exact direction duplicate at another scale
    qf = rng.standard_normal((1, 8, 8, 128)).astype(np.float32)
    vf = rng.standard_normal((1, 2, 260, 128)).astype(np.float32)
    w, q, k, v = _custom(kf, qf, vf, budget=180, pool_w=4, beta=1, sim_threshold=0.5, lam=0.1)
    run_fused(w, q, k, v, [(0, 0), (0, 1)], "zeros", check_parts=True)


def test_empty_batch_is_a_no_op():
    shp = rkv.Shape(num_problems=0, kv_heads=8, q_heads=32, n_tokens=1152, budget=1024)
    k = torch.empty((0, 8, 1152, 128), dtype=torch.bfloat16, device="cuda")
    q = torch.empty((0, 32, 8, 128), dtype=torch.bfloat16, device="cuda")
    say("empty batch")
    st, ko, vo, idx, _ = rkv.rkv_compress(shp, q, k, k)
    torch.cuda.synchronize()
    assert st == rkv.RKV_OK and ko.shape == (0, 8, 1024, 128) and idx.shape == (0, 8, 1024)


def _gradual(name, N, budget, P, H, beta, T, red, noise, seed):
    """Gaussian keys, a fraction `red` of the rows noisy copies of earlier rows: a row meets its partners
    anywhere in the scan, so the number of open rows falls gradually (several gathering stages)."""
    return synth.Workload(name, P, H, 4 * H, N, budget, beta=beta, sim_threshold=T, seed=seed, recipe="rowcopy",
                          redundancy=red, copy_noise=noise)


SKIP_CASES = [
    # workload, extra flags
    (synth.scaled(synth.CONFIGS["cfg2_llama8b_b1024"], num_problems=4), 0),             # few heads: column scan split over workgroups
    (synth.CONFIGS["cfg2_llama8b_b1024"], 0),                                            # full size: narrow last row blocks, listed last
    (synth.scaled(synth.CONFIGS["cfg2_llama8b_b1024"], beta=3), 0),
    (synth.scaled(synth.CONFIGS["cfg2_llama8b_b1024"], num_problems=2, sim_threshold=0.95, beta=2), 0),
    (synth.scaled(synth.CONFIGS["cfg2_llama8b_b1024"], num_problems=8), 32),            # other direction of the keep-recent rule
    (synth.scaled(synth.CONFIGS["cfg3_llama8b_b4096"], num_problems=3), 0),
    (synth.scaled(synth.CONFIGS["cfg5_llama8b_b8192_bs4"], num_problems=1), 0),
    (synth.CONFIGS["cfg1_tiny"], 0),
    (_gradual("gradual_b1", 1500, 1300, 40, 8, 1, 0.5, 0.9, 0.3, 501), 0),              # 1920 workgroups, six row blocks
    (_gradual("gradual_b2", 1500, 1300, 2, 2, 2, 0.5, 0.95, 0.3, 502), 0),              # beta = 2: rows move with one partner met
    (_gradual("gradual_narrow", 1400, 1200, 3, 2, 2, 0.5, 0.8, 0.3, 503), 0),           # last row block narrow (112 rows)
    (_gradual("gradual_tr", 1400, 1200, 2, 2, 3, 0.5, 0.9, 0.3, 504), 32),
    (_gradual("gradual_split", 2100, 1900, 1, 2, 1, 0.5, 0.9, 0.3, 505), 0),            # beta = 1, few heads: split scan
    (_gradual("gradual_small", 300, 200, 2, 2, 2, 0.5, 0.7, 0.3, 506), 0),              # two row blocks, the second with 36 rows
    (_gradual("none_similar", 1200, 1000, 2, 2, 1, 0.9, 0.0, 0.3, 507), 4),             # nothing is ever met: no row leaves
]


@pytest.mark.parametrize("w,flags", SKIP_CASES, ids=lambda x: x.name + f"_P{x.num_problems}_beta{x.beta}" if hasattr(x, "name") else f"flags{x}")
def test_skip_saturated_flag_gives_bit_identical_results(w, flags):
    """RKV_FLAG_SKIP_SATURATED only leaves out similarity tiles that cannot change a result, whatever
    the order in which rows are done, moved to other waves or written out early."""
    P = w.num_problems
    q, k, v = synth.make_batch(w)
    qd, kd, vd = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    dense = shape_of(w, P)
    dense.flags = flags
    skip = shape_of(w, P)
    skip.flags = flags | rkv.RKV_FLAG_SKIP_SATURATED
    say(f"skip-saturated vs dense: {w.name} P={P} H={w.kv_heads} N={w.n_tokens} T={w.sim_threshold} beta={w.beta} flags={flags}")
    a = rkv.rkv_compress(dense, qd, kd, vd, want_score=True)
    b = rkv.rkv_compress(skip, qd, kd, vd, want_score=True)
    ra, ma = rkv.rkv_score_redundancy(dense, kd, want_mean_sim=True)
    rb, mb = rkv.rkv_score_redundancy(skip, kd, want_mean_sim=True)
    torch.cuda.synchronize()
    assert torch.equal(ma, mb), f"mean similarity differs in {(ma != mb).sum().item()} entries"
    assert torch.equal(ra, rb)
    for x, y in zip(a[1:], b[1:]):
        assert torch.equal(x, y)
    if w.name.startswith("gradual"):
        # the case does what it is for: some rows are done early, some late, some never
        n = w.n_cand
        kc = O.decode_bf16(k[0, 0][:n])
        norm = np.sqrt((kc * kc).sum(1, keepdims=True)); kbar = kc / (norm + w.eps)
        hits = (kbar @ kbar.T - np.eye(n)) > w.sim_threshold
        done_at = np.full(n, -1)
        for i in range(n):
            cols = np.nonzero(hits[i])[0]
            if len(cols) >= w.beta:
                done_at[i] = cols[-w.beta]                      # the column at which row i has met beta partners
        assert (done_at < 0).sum() >= 8 and (done_at >= n - 128).sum() >= 8 and ((done_at >= 0) & (done_at < n // 2)).sum() >= 8


def test_largest_supported_cache_against_the_row_wise_oracle():
    """N = 32768 (the largest supported): 256 column tiles, 128 row blocks.  The n x n matrix does not fit
    in memory, so the oracle takes Eq. 5-6 one row of S at a time (all 32760 rows, dealt to worker
    processes) and everything after it (softmax, importance, joint score, selection) as usual; every
    output of the GPU is then compared as in the other tests."""
    N, budget, alpha = 32768, 32640, 8
    w = synth.Workload("max", 1, 1, 4, N, budget, alpha=alpha, seed=91, recipe="clusters", n_clusters=4096,
                       cluster_sigma=0.25, pool_w=4, beta=1, sim_threshold=0.8, lam=0.1)
    q, k, v = synth.make_batch(w)
    # Planted rows that tell "most recent partner" from any other choice: token i is an exact copy of an
    # old token (similarity 1) and has a loosely similar partner (cosine 0.81) at a larger index, many
    # column tiles away.  The rule forgives the recent, loose partner; forgiving the old exact copy
    # instead would move the mean similarity by 0.19 / n.  The planted direction is orthogonal to the sum
    # of all normalised keys, so the row's mean similarity is small and the tolerance below stays near
    # its absolute part, a third of that shift.
    rng = np.random.default_rng(92)
    kall = O.decode_bf16(k[0, 0][:w.n_cand])
    usum = (kall / np.sqrt((kall * kall).sum(1, keepdims=True))).sum(0)
    usum /= np.linalg.norm(usum)
    planted = []
    for (i, j_old, j_recent) in [(15000, 200, 31000), (25000, 100, 25900), (7, 3, 32500)]:
        base = rng.standard_normal(128)
        base -= (base @ usum) * usum
        noise = rng.standard_normal(128)
        noise -= (noise @ usum) * usum
        noise -= (noise @ base) / (base @ base) * base
        noise *= np.linalg.norm(base) / np.linalg.norm(noise)
        k[0, 0, i] = k[0, 0, j_old] = synth.f32_to_bf16_bits(base.astype(np.float32))
        k[0, 0, j_recent] = synth.f32_to_bf16_bits((base + 0.72 * noise).astype(np.float32))
        planted.append(i)
    shp = shape_of(w, 1)
    qd, kd, vd = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    say("max size: rkv_score_importance + rkv_score_redundancy + rkv_compress N=32768")
    imp = rkv.rkv_score_importance(shp, qd, kd)
    red, msim = rkv.rkv_score_redundancy(shp, kd, want_mean_sim=True)
    st, ko, vo, idx, score = rkv.rkv_compress(shp, qd, kd, vd, want_score=True)
    torch.cuda.synchronize()
    n = w.n_cand
    T = float(np.float32(w.sim_threshold))
    kc = O.decode_bf16(k[0, 0][:n])
    say("max size: the oracle, all rows of the similarity matrix one at a time")
    sbar = Hp.mean_similarity_all_rows(k[0, 0][:n], T, w.beta, w.eps)
    # the planted structure is what it claims to be, and the sampled rows of the earlier form of this test
    norm = np.sqrt((kc * kc).sum(1, keepdims=True)); kbar = kc / (norm + w.eps)
    got = msim[0, 0].cpu().numpy()
    for i in planted:
        srow = kbar @ kbar[i]; srow[i] = 0.0
        hits = np.nonzero(srow > w.sim_threshold)[0]
        assert len(hits) == 2 and srow[hits[0]] > 0.999 and 0.805 < srow[hits[1]] < 0.82 and hits[1] > i
        assert (srow[hits[0]] - srow[hits[1]]) / n > 2.5 * (2e-6 + 1e-3 * abs(sbar[i]))
        assert abs(got[i] - sbar[i]) <= 2e-6 + 1e-3 * abs(sbar[i]), f"row {i}: gpu {got[i]} oracle {sbar[i]}"
    # the rest of the step from the oracle's own functions on that mean similarity
    R = O.softmax_rows(sbar[None, :])[0]
    I = O.importance(O.decode_bf16(q[0]), kc, w.pool_w)
    Z = O.selection_score(I, R, float(np.float32(w.lam)))
    keep = O.select_topk(Z, w.k_sel)
    kept = np.concatenate([keep, np.arange(n, N, dtype=np.int64)])
    ref = dict(importance=I, mean_sim=sbar, redundancy=R, score=Z, kept=kept, k_out=k[0, 0][kept], v_out=v[0, 0][kept])
    # a row is exempt only if one of its similarities sits within the fp32 band around T: look for such rows
    # among those that disagree (none is expected)
    bad = np.nonzero(~Hp.close(got, sbar, rel=1e-3, abs_=2e-6))[0]
    for i in bad:
        srow = kbar @ kbar[i]; srow[i] = 0.0
        assert np.any(np.abs(srow - w.sim_threshold) <= Hp.SIM_BAND) and i not in planted, f"row {i}: gpu {got[i]} oracle {sbar[i]}"
    assert len(bad) <= 4
    ok = np.ones(n, dtype=bool)
    ok[bad] = False
    assert Hp.close(imp[0, 0].cpu().numpy(), I).all(), "importance"
    assert Hp.close(red[0, 0].cpu().numpy()[ok], R[ok]).all(), "redundancy"
    z = score[0, 0].cpu().numpy()
    assert Hp.close(z[ok], Z[ok]).all(), "score"
    lam = float(np.float32(w.lam))
    scale = lam * np.abs(I) + (1 - lam) * np.abs(R)
    rel = (np.abs(z - Z) / (scale + 1e-12))[ok].max()
    assert rel < Hp.TERM_REL_ERR, rel
    kept_gpu = idx[0, 0].cpu().numpy()
    np.testing.assert_array_equal(kept_gpu[:w.k_sel], Hp.exact_topk(z, w.k_sel))
    np.testing.assert_array_equal(kept_gpu[w.k_sel:], np.arange(n, N))
    must_keep, must_drop = Hp.decidable_selection(Z, np.where(ok, Hp.TERM_REL_ERR * scale, np.inf), w.k_sel)
    mask = np.zeros(n, dtype=bool)
    mask[kept_gpu[:w.k_sel]] = True
    assert not (must_keep & ~mask).any() and not (must_drop & mask).any()
    free = int((~(must_keep | must_drop)).sum())
    say(f"max size: scores match on all {n} candidates (error relative to the terms {rel:.1e}); "
        f"{free} selections undecidable within that error, {len(bad)} threshold-fragile rows")
    assert free <= 0.02 * w.k_sel
    np.testing.assert_array_equal(host_bits(ko)[0, 0], k[0, 0][kept_gpu])
    np.testing.assert_array_equal(host_bits(vo)[0, 0], v[0, 0][kept_gpu])
    if np.array_equal(kept_gpu, ref["kept"]):
        np.testing.assert_array_equal(host_bits(ko)[0, 0], ref["k_out"])
    r = red[0, 0].cpu().numpy().astype(np.float64)
    assert abs(r.sum() - 1.0) < 1e-4                      # softmax over the candidates (Eq. 6)


# ------------------------------------------------------------------------------ decode loop
@pytest.mark.parametrize("inplace", [False, True], ids=["two_buffers", "inplace"])
def test_decode_loop_bookkeeping_and_per_event_parity(inplace):
    """A synthetic decode run through DecodeCache: appended rows land where they should, the step
    triggers every B_buffer tokens once the cache is full, and every compression event matches the
    oracle run on the cache contents the GPU held at that moment."""
    from paper_2505_24133_amd.decode import DecodeCache
    P, H, G, alpha, budget, buffer = 2, 2, 4, 8, 96, 32
    N = budget + buffer
    shp = rkv.Shape(num_problems=P, kv_heads=H, q_heads=H * G, n_tokens=N, budget=budget, alpha=alpha,
                    pool_w=2, beta=1, sim_threshold=0.5, lam=0.1)
    w = synth.Workload("loop", P, H, H * G, N, budget, alpha=alpha, pool_w=2, beta=1, sim_threshold=0.5, lam=0.1)
    prm = Hp.oracle_params(w)
    cache = DecodeCache(shp, inplace=inplace)
    rng = np.random.default_rng(5)
    steps = N + 3 * buffer + 5
    history_k = []
    events = 0
    for t in range(steps):
        kf = rng.standard_normal((P, H, 128)).astype(np.float32)
        if t > 10 and t % 3 == 0:                       # repetitive "reasoning": re-emit an earlier key, noisily
            kf = history_k[int(rng.integers(0, t))] + 0.05 * rng.standard_normal((P, H, 128)).astype(np.float32)
        history_k.append(kf)
        vf = rng.standard_normal((P, H, 128)).astype(np.float32)
        qf = rng.standard_normal((P, H * G, 128)).astype(np.float32)
        kb, vb, qb = synth.f32_to_bf16_bits(kf), synth.f32_to_bf16_bits(vf), synth.f32_to_bf16_bits(qf)
        will_fire = cache.length + 1 == N
        before_k = host_bits(cache.k) if will_fire else None
        before_v = host_bits(cache.v) if will_fire else None
        pos = cache.length
        say(f"decode step {t}: length {cache.length}{' -> compress' if will_fire else ''}")
        fired = cache.append(dev_bf16(kb), dev_bf16(vb), dev_bf16(qb))
        torch.cuda.synchronize()
        assert fired == will_fire
        if not fired:
            np.testing.assert_array_equal(host_bits(cache.k)[:, :, pos], kb)
            np.testing.assert_array_equal(host_bits(cache.v)[:, :, pos], vb)
            assert cache.length == pos + 1
        else:
            events += 1
            before_k[:, :, pos] = kb
            before_v[:, :, pos] = vb
            q_now = host_bits(cache.q_cache)
            np.testing.assert_array_equal(q_now[:, :, t % alpha], qb)      # newest query is in its slot
            kept = cache.kept_idx.cpu().numpy()
            after_k, after_v = host_bits(cache.k), host_bits(cache.v)
            assert cache.length == budget
            for p in range(P):
                for h in range(H):
                    ref = O.compress_head(q_now[p, h * G:(h + 1) * G], before_k[p, h], before_v[p, h], prm)
                    check_head(w, ref, None, kept[p, h], after_k[p, h, :budget], after_v[p, h, :budget],
                               before_k[p, h], before_v[p, h], f"event{events}[p{p},h{h}]")
    assert events == cache.compressions == 1 + 3
    assert cache.tokens_seen == steps and cache.length == budget + 5


INPLACE_SHAPES = [
    # P, H, N, budget
    (2, 2, 384, 256),        # two column slices per row (few heads)
    (1, 1, 65, 17),          # less than one tile
    (3, 2, 5000, 4100),      # several tiles, ragged last tile
    (1, 2, 32768, 1000),     # shifts far larger than a tile
    (40, 8, 1152, 1024),     # whole rows per workgroup (many heads)
]


def _ascending_lists(rng, P, H, N, budget, pattern):
    """kept lists [P, H, budget], strictly ascending, of the given eviction pattern."""
    out = np.empty((P, H, budget), dtype=np.int32)
    for p in range(P):
        for h in range(H):
            if pattern == "front":        # the first N - budget rows are evicted: every row moves by the full shift
                out[p, h] = np.arange(N - budget, N)
            elif pattern == "back":       # nothing moves
                out[p, h] = np.arange(budget)
            elif pattern == "late":       # one eviction close to the end: almost every row stays
                cut = max(budget - 3, 0)
                out[p, h] = np.concatenate([np.arange(cut), np.arange(N - (budget - cut), N)])
            else:                         # random subset
                out[p, h] = np.sort(rng.choice(N, size=budget, replace=False))
    return out


@pytest.mark.parametrize("pattern", ["random", "front", "back", "late"])
@pytest.mark.parametrize("case", INPLACE_SHAPES, ids=lambda c: f"P{c[0]}_H{c[1]}_N{c[2]}_b{c[3]}")
def test_compact_inplace_moves_rows_without_losing_any(case, pattern):
    """In-place compaction against the definition (rows kept[r] of the cache as it was, bit for bit)
    for eviction patterns that stress the overlap of source and destination rows; rows behind the
    budget keep their old content."""
    P, H, N, budget = case
    rng = np.random.default_rng(N + budget)
    shp = rkv.Shape(num_problems=P, kv_heads=H, q_heads=H, n_tokens=N, budget=budget)
    kb = rng.integers(0, 1 << 16, size=(P, H, N, 128), dtype=np.uint16)
    vb = rng.integers(0, 1 << 16, size=(P, H, N, 128), dtype=np.uint16)
    kept = _ascending_lists(rng, P, H, N, budget, pattern)
    say(f"rkv_compact_inplace P={P} H={H} N={N} budget={budget} pattern={pattern}")
    kd, vd = dev_bf16(kb), dev_bf16(vb)
    rkv.rkv_compact_inplace(shp, kd, vd, torch.from_numpy(kept).cuda())
    torch.cuda.synchronize()
    k_after, v_after = host_bits(kd), host_bits(vd)
    pi, hi = np.arange(P)[:, None, None], np.arange(H)[None, :, None]
    np.testing.assert_array_equal(k_after[:, :, :budget], kb[pi, hi, kept])
    np.testing.assert_array_equal(v_after[:, :, :budget], vb[pi, hi, kept])
    np.testing.assert_array_equal(k_after[:, :, budget:], kb[:, :, budget:])
    np.testing.assert_array_equal(v_after[:, :, budget:], vb[:, :, budget:])


def test_compress_inplace_equals_compress():
    """The fused step with in-place compaction gives the kept list, scores and rows of rkv_compress,
    also on strided views of a larger cache allocation."""
    w = synth.scaled(synth.CONFIGS["cfg2_llama8b_b1024"], num_problems=3)
    q, k, v = synth.make_batch(w)
    shp = shape_of(w, 3)
    qd = dev_bf16(q)
    big_k = torch.zeros((3, w.kv_heads, w.n_tokens + 40, 128), dtype=torch.bfloat16, device="cuda")
    big_v = torch.zeros_like(big_k)
    kview, vview = big_k[:, :, 7:7 + w.n_tokens], big_v[:, :, 7:7 + w.n_tokens]
    kview.copy_(dev_bf16(k))
    vview.copy_(dev_bf16(v))
    say("rkv_compress then rkv_compress_inplace on strided views, cfg2 shape P=3")
    st, ko, vo, idx, score = rkv.rkv_compress(shp, qd, kview, vview, want_idx=True, want_score=True)
    st2, idx2, score2 = rkv.rkv_compress_inplace(shp, qd, kview, vview, want_idx=True, want_score=True)
    torch.cuda.synchronize()
    assert st == st2 == rkv.RKV_OK
    assert torch.equal(idx, idx2) and torch.equal(score, score2)
    assert torch.equal(kview[:, :, :w.budget], ko) and torch.equal(vview[:, :, :w.budget], vo)
    np.testing.assert_array_equal(host_bits(kview[:, :, w.budget:]), k[:, :, w.budget:])
    assert not big_k[:, :, :7].any() and not big_k[:, :, 7 + w.n_tokens:].any()      # nothing outside the view
    # not triggered: the cache is left alone
    calm = rkv.Shape(num_problems=3, kv_heads=w.kv_heads, q_heads=w.q_heads, n_tokens=w.n_tokens, budget=w.n_tokens)
    before = kview.clone()
    st3, *_ = rkv.rkv_compress_inplace(calm, qd, kview, vview)
    torch.cuda.synchronize()
    assert st3 == rkv.RKV_NOT_TRIGGERED and torch.equal(before, kview)


def test_hip_graph_replays_match_eager():
    """rkv_compress captured into a HIP graph (the library enqueues kernels only: no allocation, no
    memset, no host synchronisation) and replayed on fresh inputs, with eager work between the
    replays; every replay must equal the eager call on the same inputs."""
    w = synth.scaled(synth.CONFIGS["cfg1_tiny"], num_problems=3)
    shp = shape_of(w, 3)
    batches = [synth.make_batch(synth.scaled(w, seed=900 + i)) for i in range(3)]
    qs, ks, vs = (torch.empty_like(dev_bf16(x)) for x in batches[0])
    ws = rkv.make_workspace(shp)
    ko = torch.empty((3, w.kv_heads, w.budget, 128), dtype=torch.bfloat16, device="cuda")
    vo = torch.empty_like(ko)
    idx = torch.empty((3, w.kv_heads, w.budget), dtype=torch.int32, device="cuda")
    score = torch.empty((3, w.kv_heads, w.n_cand), dtype=torch.float32, device="cuda")

    def call():
        st = rkv.rkv_compress(shp, qs, ks, vs, ws=ws, k_out=ko, v_out=vo, kept_idx=idx, score=score)[0]
        assert st == rkv.RKV_OK

    say("graph capture of rkv_compress, cfg1 shape P=3")
    qs.copy_(dev_bf16(batches[0][0])), ks.copy_(dev_bf16(batches[0][1])), vs.copy_(dev_bf16(batches[0][2]))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call()                                       # first call outside the capture (one-time kernel set-up)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for r, (q, k, v) in enumerate(batches + batches[:1]):
        say(f"replay {r}")
        qs.copy_(dev_bf16(q)), ks.copy_(dev_bf16(k)), vs.copy_(dev_bf16(v))
        ko.zero_(), vo.zero_(), idx.zero_(), score.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = (ko.clone(), vo.clone(), idx.clone(), score.clone())
        st, ko2, vo2, idx2, score2 = rkv.rkv_compress(shp, dev_bf16(q), dev_bf16(k), dev_bf16(v), want_idx=True, want_score=True)
        torch.cuda.synchronize()
        assert torch.equal(got[2], idx2) and torch.equal(got[3], score2), f"replay {r}: indices or scores differ"
        assert torch.equal(got[0], ko2) and torch.equal(got[1], vo2), f"replay {r}: compacted rows differ"


def _paged_copy(rng, dense, page_size, spare=3):
    """dense [P, H, N, d] -> (pool [pages, H, page_size, d], table [P, ceil(N / page_size)]): pages are
    dealt in a random order, `spare` unused pages hold a marker, the tail of the last page of a
    problem is left as marker too."""
    P, H, N, d = dense.shape
    per = (N + page_size - 1) // page_size
    order = rng.permutation(P * per + spare)
    table = order[:P * per].reshape(P, per).astype(np.int32)
    pool = np.full((P * per + spare, H, page_size, d), 0x7FC0, dtype=np.uint16)      # bf16 NaN marker
    for p in range(P):
        for b in range(per):
            rows = dense[p, :, b * page_size:(b + 1) * page_size]
            pool[table[p, b], :, :rows.shape[1]] = rows
    return pool, table


def _unpage(pool, table, N):
    P, per = table.shape
    ps = pool.shape[2]
    return np.concatenate([pool[table[:, b]] for b in range(per)], axis=2)[:, :, :N]


@pytest.mark.parametrize("page_size", [16, 32, 64, 128])
def test_paged_cache_equals_contiguous(page_size):
    """The same K/V held in a page pool behind a block table: every entry point gives bit for bit
    what it gives on the contiguous cache (which the other tests check against the oracle), the
    in-place form leaves the kept rows in the first pages of each problem and touches nothing else,
    and a row appended through the table lands in its page."""
    w = synth.scaled(synth.CONFIGS["cfg1_tiny"], num_problems=3, n_tokens=363, budget=250, kv_heads=2, q_heads=8)
    q, k, v = synth.make_batch(w)
    rng = np.random.default_rng(page_size)
    kp, table = _paged_copy(rng, k, page_size)
    vp, _ = _paged_copy(np.random.default_rng(page_size), v, page_size)              # same table (same seed)
    shp = shape_of(w, 3)
    qd, kd, vd = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    say(f"paged cache, page_size={page_size}: dense reference run")
    st, ko, vo, idx, score = rkv.rkv_compress(shp, qd, kd, vd, want_idx=True, want_score=True)
    imp = rkv.rkv_score_importance(shp, qd, kd)
    red, msim = rkv.rkv_score_redundancy(shp, kd, want_mean_sim=True)
    torch.cuda.synchronize()
    import dataclasses
    pshp = dataclasses.replace(shp, page_size=page_size, block_table=torch.from_numpy(table).cuda())
    kpd, vpd = dev_bf16(kp), dev_bf16(vp)
    say(f"paged cache, page_size={page_size}: paged entry points")
    st2, ko2, vo2, idx2, score2 = rkv.rkv_compress(pshp, qd, kpd, vpd, want_idx=True, want_score=True)
    imp2 = rkv.rkv_score_importance(pshp, qd, kpd)
    red2, msim2 = rkv.rkv_score_redundancy(pshp, kpd, want_mean_sim=True)
    ko3, vo3 = rkv.rkv_compact(pshp, kpd, vpd, idx2)
    torch.cuda.synchronize()
    assert st2 == rkv.RKV_OK
    assert torch.equal(idx, idx2) and torch.equal(score, score2)
    assert torch.equal(ko, ko2) and torch.equal(vo, vo2) and torch.equal(ko, ko3) and torch.equal(vo, vo3)
    assert torch.equal(imp, imp2) and torch.equal(red, red2) and torch.equal(msim, msim2)
    np.testing.assert_array_equal(host_bits(kpd), kp)                                 # inputs untouched
    # and the paged entry points' own outputs against the oracle, every head
    check_outputs(w, q, k, v, [(p, h) for p in range(3) for h in range(w.kv_heads)], idx2.cpu().numpy(), score2.cpu().numpy(),
                  host_bits(ko2), host_bits(vo2), f"paged{page_size}",
                  parts=(imp2.cpu().numpy(), red2.cpu().numpy(), msim2.cpu().numpy()))
    # in place: kept rows move to the front of each problem's token order
    say(f"paged cache, page_size={page_size}: in place")
    st3, idx3, _ = rkv.rkv_compress_inplace(pshp, qd, kpd, vpd)
    torch.cuda.synchronize()
    assert st3 == rkv.RKV_OK and torch.equal(idx3, idx)
    k_after, v_after = host_bits(kpd), host_bits(vpd)
    np.testing.assert_array_equal(_unpage(k_after, table, w.n_tokens)[:, :, :w.budget], host_bits(ko))
    np.testing.assert_array_equal(_unpage(v_after, table, w.n_tokens)[:, :, :w.budget], host_bits(vo))
    np.testing.assert_array_equal(_unpage(k_after, table, w.n_tokens)[:, :, w.budget:], k[:, :, w.budget:])
    used = np.zeros(kp.shape[0], dtype=bool)
    used[table.ravel()] = True
    np.testing.assert_array_equal(k_after[~used], kp[~used])                          # spare pages untouched
    last = table[:, -1]
    tail = w.n_tokens - (table.shape[1] - 1) * page_size
    np.testing.assert_array_equal(k_after[last][:, :, tail:], kp[last][:, :, tail:])  # slots past N untouched
    # append through the table
    newk = dev_bf16(synth.f32_to_bf16_bits(rng.standard_normal((3, 2, 128)).astype(np.float32)))
    newv = dev_bf16(synth.f32_to_bf16_bits(rng.standard_normal((3, 2, 128)).astype(np.float32)))
    newq = dev_bf16(synth.f32_to_bf16_bits(rng.standard_normal((3, 8, 128)).astype(np.float32)))
    qring = qd.clone()
    pos = w.budget + 1
    rkv.rkv_cache_append(pshp, kpd, vpd, qring, newk, newv, newq, pos, 5)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(_unpage(host_bits(kpd), table, w.n_tokens)[:, :, pos], host_bits(newk))
    np.testing.assert_array_equal(_unpage(host_bits(vpd), table, w.n_tokens)[:, :, pos], host_bits(newv))
    np.testing.assert_array_equal(host_bits(qring)[:, :, 5], host_bits(newq))


def test_shared_workspace_across_shapes():
    """One oversized workspace reused by calls of different shapes: nothing read is left over from
    an earlier call."""
    big = synth.scaled(synth.CONFIGS["cfg2_llama8b_b1024"], num_problems=2)
    small = synth.Workload("small", 1, 2, 8, 203, 120, seed=5, recipe="rowcopy", redundancy=0.3, copy_noise=0.1)
    ws = rkv.make_workspace(shape_of(big, 2))
    ref = {}
    for w in (big, small):
        q, k, v = synth.make_batch(w)
        ref[w.name] = (dev_bf16(q), dev_bf16(k), dev_bf16(v))
    outs = {}
    say("shared workspace: big, small, big, small")
    for rnd in range(2):
        for w in (big, small):
            qd, kd, vd = ref[w.name]
            o = rkv.rkv_compress(shape_of(w, w.num_problems), qd, kd, vd, ws=ws, want_score=True)
            torch.cuda.synchronize()
            if w.name in outs:
                for x, y in zip(outs[w.name][1:], o[1:]):
                    assert torch.equal(x, y)
            outs[w.name] = tuple(t.clone() if isinstance(t, torch.Tensor) else t for t in o)
    # and both agree with a call that owns a fresh workspace
    for w in (big, small):
        qd, kd, vd = ref[w.name]
        o = rkv.rkv_compress(shape_of(w, w.num_problems), qd, kd, vd, want_score=True)
        torch.cuda.synchronize()
        for x, y in zip(outs[w.name][1:], o[1:]):
            assert torch.equal(x, y)


def test_bench_prints_one_json_line_with_the_agreed_fields(repo_root):
    """bench.py on the GPU, a few steps: one JSON line with the throughput, the dominant kernel's
    roofline entry and the CPU oracle's rate."""
    import json
    import subprocess
    import sys
    say("bench.py --steps 3 (child process)")
    r = subprocess.run([sys.executable, "bench.py", "--steps", "3", "--warmup", "1", "--no-other-modes", "--no-workloads", "--cpu-seconds", "1"],
                       cwd=repo_root, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["config"]["workload"] == "cfg2_llama8b_b1024" and d["data"] == "synthetic" and d["vs_baseline"] is None
    assert d["value"] > 0 and abs(d["value"] * d["ms_per_step"] - 1000.0) < 1.0
    roof = d["roofline"]
    assert roof["bound"] == "mfma" and roof["unit"] == "TFLOP/s" and roof["peak"] == 2500.0
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9 and 0.05 < roof["frac"] < 1.0
    assert roof["traffic"] is None or roof["traffic"] > 0
    dev = d["device"]
    assert dev["device_copy_GB/s"] > 500 and dev["published_peaks"]["hbm_GB/s"] == 8000.0
    assert dev["clocks_under_load"] is None or 100 < dev["clocks_under_load"]["sclk_mhz"] <= 2600
    cold = d["cold"]
    assert cold["sets_rotated"] >= 2 and cold["bytes_between_reuse"] > 4 * (256 << 20) and cold["ms_per_step"] > 0
    assert set(cold["stages"]) == set(d["stages"])
    cpu = d["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["value"] > 0 and cpu["cores"] >= 1 and cpu["unit"] == d["unit"] and cpu["sample"]


def _random_case(seed):
    """A supported shape drawn at random (seeded): odd group sizes and windows, beta beyond the number of
    hits, thresholds at both ends, budgets from k = 1 to k = n - 1."""
    rng = np.random.default_rng(1000 + seed)
    alpha = int(rng.choice([1, 2, 3, 5, 8, 8, 8, 9, 12, 16, 16, 24, 32, 40, 64]))
    G = int(rng.integers(1, 64 // alpha + 1))
    G = min(G, 8)
    H = int(rng.integers(1, 4))
    n = int(rng.integers(alpha + 2, 1500))
    N = n + alpha
    budget = int(rng.integers(alpha + 1, N))
    W = int(rng.choice([0, 1, 2, 3, 4, 4, 5, 8, 16, 33]))
    while W > 0 and (alpha + 1) * 2 * W > 16384:
        W //= 2
    beta = int(rng.choice([0, 1, 1, 1, 2, 3, 7]))
    T = float(rng.choice([0.0, 0.3, 0.5, 0.5, 0.8, 0.95, 1.0]))
    lam = float(rng.choice([0.0, 0.05, 0.1, 0.1, 0.5, 0.9]))
    recipe = str(rng.choice(["rowcopy", "spans", "clusters"]))
    red = float(rng.uniform(0.1, 0.7))
    return synth.Workload(f"rnd{seed}", 2, H, H * G, N, budget, alpha=alpha, pool_w=W, beta=beta, sim_threshold=T,
                          lam=lam, seed=5000 + seed, recipe=recipe, redundancy=red, copy_noise=0.1,
                          outlier_channels=int(rng.choice([0, 4])), n_clusters=int(rng.choice([4, 16, 64])))


@pytest.mark.parametrize("seed", range(24))
def test_random_supported_shapes(seed):
    w = _random_case(seed)
    q, k, v = synth.make_batch(w)
    run_fused(w, q, k, v, [(p, h) for p in range(2) for h in range(w.kv_heads)], w.name, check_parts=True)


@pytest.mark.parametrize("seed", range(100, 116))
def test_random_supported_shapes_with_variant_flags(seed):
    """The same with a random combination of the variant flags (pooling order, shared selection, either
    App. A.2 group merge, the other direction of the keep-recent rule, the exact shortcut)."""
    w = _random_case(seed)
    rng = np.random.default_rng(9000 + seed)
    flags = int(rng.choice([0, rkv.RKV_FLAG_GQA_SOFTMAX_THEN_MAX, rkv.RKV_FLAG_GQA_SOFTMAX_THEN_MEAN]))
    for bit in (rkv.RKV_FLAG_SKIP_SATURATED, rkv.RKV_FLAG_POOL_AFTER_MEAN, rkv.RKV_FLAG_SHARED_SELECTION,
                rkv.RKV_FLAG_RECENCY_TRANSPOSED):
        if rng.random() < 0.5:
            flags |= bit
    if (flags & rkv.RKV_FLAG_POOL_AFTER_MEAN) and w.pool_w > 0 and (w.alpha + 1) * 2 * w.pool_w > 16384:
        flags &= ~rkv.RKV_FLAG_POOL_AFTER_MEAN
    q, k, v = synth.make_batch(w)
    run_fused(w, q, k, v, [(p, h) for p in range(2) for h in range(w.kv_heads)], f"{w.name}_flags{flags}", flags=flags)
