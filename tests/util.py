"""Helpers shared by the tests: oracle argument packing and the parity rules."""
from __future__ import annotations

import numpy as np

from oracle import hisa_oracle as O

RTOL = {"f32": 1e-5, "bf16": 2e-2, "fp8_e4m3": 2e-2}


def oracle_args(wl, *, keys=True):
    a = dict(q=wl.q, q_dtype=wl.q_dtype, w=wl.w, q_seq=wl.q_seq, q_pos=wl.positions())
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


def check_scores(got, want, rtol, what=""):
    """|got - want| <= rtol * max(|want|, A) per row, A = the row's largest finite |want|;
    slots that are -inf in the oracle must be -inf (or untouched NaN-free -inf) in `got`."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    fin = np.isfinite(want)
    assert np.array_equal(np.isneginf(got), np.isneginf(want)), f"{what}: -inf mask differs"
    A = np.where(fin, np.abs(want), 0.0).max(axis=-1, keepdims=True)
    bound = rtol * np.maximum(np.abs(np.where(fin, want, 0.0)), A)
    err = np.abs(np.where(fin, got - want, 0.0))
    bad = err > bound
    assert not bad.any(), (f"{what}: {bad.sum()} scores out of tolerance; worst "
                           f"{(err / np.maximum(bound, 1e-300)).max():.3g} x bound")
    return float((err / np.maximum(A, 1e-300)).max())


def check_set(got_ids, want_ids, id_scores, rtol, what="", universe=None):
    """The selection rule of the benchmark definition: the two index sets have the same size and
    every id in their symmetric difference has an oracle score within rtol * max(|tau|, A) of the
    oracle's threshold tau (its worst selected score).  id_scores: dict-like id -> oracle score
    for every candidate; A = max |score| over the candidates.  Also checks uniqueness and that
    every got id is a candidate."""
    g = np.asarray(got_ids)
    g = g[g >= 0]
    wv = np.asarray(want_ids)
    wv = wv[wv >= 0]
    assert len(set(g.tolist())) == g.size, f"{what}: duplicate ids"
    assert g.size == wv.size, f"{what}: {g.size} valid ids, oracle has {wv.size}"
    sg, sw = set(g.tolist()), set(wv.tolist())
    if universe is not None:
        assert sg <= universe, f"{what}: ids outside the candidate set: {sorted(sg - universe)[:8]}"
    if sg == sw:
        return 0
    diff = sg ^ sw
    sc = id_scores
    allv = np.array([sc[i] for i in (universe if universe is not None else sw | sg)])
    A = np.abs(allv).max()
    tau = min(sc[i] for i in sw)
    tol = rtol * max(abs(tau), A)
    for i in diff:
        assert i in sc, f"{what}: id {i} is not a candidate"
        assert abs(sc[i] - tau) <= tol, (f"{what}: id {i} score {sc[i]!r} differs from threshold "
                                         f"{tau!r} by more than {tol:.3g}")
    return len(diff)
