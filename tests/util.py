"""Helpers shared by the tests: oracle argument packing and the parity rules."""
from __future__ import annotations

import numpy as np

from oracle import hisa_oracle as O

# Acceptance tolerances of the benchmark definition (relative score error; swaps at the threshold).
RTOL = {"f32": 1e-5, "bf16": 2e-2, "fp8_e4m3": 2e-2}

# Regression bounds per arithmetic path, relative to the row's largest |score| A.  The acceptance
# tolerances above are three to five orders of magnitude wider than what the kernels produce, so a
# lost term of the contraction would pass them; these bounds sit a factor 20-50 above the worst error
# the arithmetic is expected to make and far below what any dropped or halved term produces:
#   bf16 keys   products of two bf16 numbers are exact in fp32; what is left is the fp32 accumulation
#               of d = 128 products and H = 64 gated terms: observed 2e-7 * A;
#   fp8 keys    the stored e4m3 codes against the two-term e4m3 form of the bf16 query (exact but for
#               elements 2^-9 below their head's largest) on the fp8 MFMA, whose accumulation is
#               coarser: observed 2e-5 * A rms, 6e-5 * A worst;
#   fp32        FMA dot products in four partial sums: observed 3e-6 * A.
DESIGN_RTOL = {"f32": 1e-5, "bf16": 1e-5, "fp8_e4m3": 3e-4}


def oracle_args(wl, *, keys=True):
    a = dict(q=wl.q, q_dtype=wl.q_dtype, w=wl.w, q_seq=wl.q_seq, q_pos=wl.positions(), q_lo=wl.q_lo)
    if keys:
        a.update(keys=wl.keys, k_dtype=wl.k_dtype, k_scale=wl.k_scale)
    return a


def oracle_hisa(wl, queries=None, pooled=None, m=None, k=None):
    return O.hisa_indexer(**oracle_args(wl), seq_len=wl.seq_len, B=wl.B, m=wl.m if m is None else m,
                          k=wl.k if k is None else k, pooled_dtype=wl.pooled_dtype,
                          queries=queries, pooled=pooled)


def oracle_flat(wl, queries=None, k=None, return_scores=False):
    return O.dsa_flat_indexer_topk(**oracle_args(wl), k=wl.k if k is None else k, queries=queries,
                                   return_scores=return_scores)


def rtol_for(wl):
    return max(RTOL[wl.q_dtype], RTOL[wl.k_dtype])


def design_rtol_for(wl, pooled=False):
    """Regression bound of the path that scores `wl`'s token keys (pooled=True: its pooled keys,
    which are bf16 -- or fp32 -- whatever the token keys are)."""
    if pooled:
        return DESIGN_RTOL[wl.pooled_dtype]
    return max(DESIGN_RTOL[wl.q_dtype], DESIGN_RTOL[wl.k_dtype])


def check_scores(got, want, rtol, what="", design_rtol=None):
    """|got - want| <= rtol * max(|want|, A) per row, A = the row's largest finite |want|;
    slots that are -inf in the oracle must be -inf (or untouched NaN-free -inf) in `got`.
    design_rtol: additionally |got - want| <= design_rtol * A (the regression bound of the path).
    Returns the largest |got - want| / A."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if want.size == 0:                       # nothing to compare (a query that sees no key)
        return 0.0
    fin = np.isfinite(want)
    assert np.array_equal(np.isneginf(got), np.isneginf(want)), f"{what}: -inf mask differs"
    A = np.where(fin, np.abs(want), 0.0).max(axis=-1, keepdims=True)
    bound = rtol * np.maximum(np.abs(np.where(fin, want, 0.0)), A)
    err = np.abs(np.where(fin, got, 0.0) - np.where(fin, want, 0.0))
    bad = err > bound
    assert not bad.any(), (f"{what}: {bad.sum()} scores out of tolerance; worst "
                           f"{(err / np.maximum(bound, 1e-300)).max():.3g} x bound")
    worst = float((err / np.maximum(A, 1e-300)).max())
    if design_rtol is not None:
        assert worst <= design_rtol, (f"{what}: score error {worst:.3g} x the row maximum exceeds the "
                                      f"regression bound {design_rtol:.3g} of this arithmetic path")
    return worst


def check_set(got_ids, want_ids, cand_ids, cand_scores, rtol, what="", design_rtol=None):
    """The selection rule of the benchmark definition: the two index sets have the same size and
    every id in their symmetric difference has an oracle score within rtol * |tau| of the oracle's
    threshold tau (its worst selected score; a threshold of zero gets the floor 1e-3 * rtol * A, A =
    max |score| over the candidates).  design_rtol: additionally such an id lies within
    2 * design_rtol * A of tau (both scores of a swapped pair may be off by the path's regression
    bound).  cand_ids / cand_scores: every candidate id with its oracle score.  Also checked: ids
    unique, ascending, -1 padding at the end only, every id a candidate.  Returns the number of swaps."""
    got_ids = np.asarray(got_ids)
    n_valid = int((got_ids >= 0).sum())
    g = got_ids[:n_valid]
    assert np.all(got_ids[n_valid:] == -1) and np.all(g >= 0), f"{what}: padding is not a suffix of -1"
    assert np.all(np.diff(g) > 0), f"{what}: ids not strictly ascending"
    wv = np.asarray(want_ids)
    wv = wv[wv >= 0]
    assert g.size == wv.size, f"{what}: {g.size} valid ids, oracle has {wv.size}"
    cand_ids = np.asarray(cand_ids)
    cand_scores = np.asarray(cand_scores, dtype=np.float64)
    assert np.all(np.isin(g, cand_ids)), f"{what}: ids outside the candidate set"
    diff = np.setxor1d(g, wv)
    if diff.size == 0:
        return 0
    order = np.argsort(cand_ids)
    sid, ssc = cand_ids[order], cand_scores[order]
    sc_diff = ssc[np.searchsorted(sid, diff)]
    tau = ssc[np.searchsorted(sid, wv)].min()
    A = np.abs(cand_scores).max()
    tol = rtol * max(abs(tau), 1e-3 * A)
    if design_rtol is not None:
        tol = min(tol, 2.0 * design_rtol * A)
    worst = np.abs(sc_diff - tau).max()
    assert worst <= tol, (f"{what}: {diff.size} ids differ from the oracle's set and one lies "
                          f"{worst:.3g} from the threshold {tau:.6g} (allowed {tol:.3g})")
    return int(diff.size // 2)
