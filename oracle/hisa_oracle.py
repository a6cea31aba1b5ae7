"""CPU oracle for the HISA hierarchical indexer and the flat DSA indexer.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP library is
checked against; only tests/, the smoke check and the benchmark's cpu_baseline leg may import it.
It shares no code with the HIP path and imports nothing from the product package.

Everything is written out from the paper's definitions, in IEEE double:

  Eq. 1   I_{t,s} = sum_j w_{t,j} * ReLU(q_{t,j} . k_s)                    (DSA token score)
  Eq. 2   T_t     = TopK(I_{t,:}, k)                                        (flat DSA selection)
  Eq. 4   pooled key of block b = mean of the block's indexing keys        (Algorithm 1, pooling loop)
  Eq. 5   J_{t,b} = sum_j w_{t,j} * ReLU(q_{t,j} . pooled_b)                (Stage 1 score)
  Eq. 6   C_t     = TopK(J_{t,:}, m), first and last visible block forced   (Section 4.1, Stage 1)
  Eq. 7   Omega_t = union of the kept blocks' tokens
  Eq. 8-9 Eq. 1 restricted to Omega_t, then TopK(., k)                      (Stage 2)

A library matmul (numpy, float64) serves as the contraction step; selection is a full sort.

Readings taken where the paper is silent (each is listed in the design notes of the repository):
  * positions are 0-based; query at position p sees keys s <= p (Section 4.1, boundary behaviour:
    in the short-prefix regime the whole prefix is selected, which includes the query's own key);
  * the forced first block and the block containing the query count inside the budget m (Section
    4.1, boundary behaviour, counts m*B candidates at most), so |C_t| = min(m, #visible blocks);
  * a partial block is averaged over the tokens it holds; the pooled cache is a stored tensor, so
    the mean is rounded once (nearest-even) to the pooled dtype and Stage 1 reads the rounded value;
  * TopK orders by score descending, ties by lower index; with fewer candidates than the budget
    everything is selected and the output is padded with -1;
  * -0 counts as +0;
  * packed sequences (Section 4.1's remark on blocks that straddle two sequences): a query may
    carry a first visible position lo (its sequence's first token in the packed stream; 0 if not
    given) and then sees the keys lo <= s <= p.  Blocks stay multiples of B of the packed stream; a
    block that holds tokens of two sequences is pooled over everything it stores; the visible
    blocks are lo // B .. p // B, of which the first and the last are forced, and Stage 2 masks
    the tokens below lo.

Stored formats: "f32" float32; "bf16" uint16 bit patterns (upper half of a float32); "fp8_e4m3"
uint8 OCP e4m3fn codes with one float32 scale per token, key = scale * decode(code).
"""
from __future__ import annotations

import numpy as np

F32, BF16, FP8 = "f32", "bf16", "fp8_e4m3"


# ----------------------------------------------------------------------------- stored formats
def fp8_e4m3fn_table() -> np.ndarray:
    """All 256 OCP e4m3fn values from the format definition: 1 sign, 4 exponent (bias 7),
    3 mantissa bits; exponent field 0 is subnormal (m/8 * 2^-6); S.1111.111 is NaN; no infinities."""
    tab = np.empty(256, dtype=np.float64)
    for c in range(256):
        s = -1.0 if (c >> 7) else 1.0
        e = (c >> 3) & 0xF
        mant = c & 0x7
        if e == 0xF and mant == 0x7:
            tab[c] = np.nan
        elif e == 0:
            tab[c] = s * (mant / 8.0) * 2.0 ** (-6)
        else:
            tab[c] = s * (1.0 + mant / 8.0) * 2.0 ** (e - 7)
    return tab


_FP8_TABLE = fp8_e4m3fn_table()


def decode(bits: np.ndarray, dtype: str, scale: np.ndarray | None = None) -> np.ndarray:
    """Stored bits -> float64, exactly."""
    if dtype == F32:
        assert bits.dtype == np.float32
        return bits.astype(np.float64)
    if dtype == BF16:
        assert bits.dtype == np.uint16
        return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    if dtype == FP8:
        assert bits.dtype == np.uint8
        x = _FP8_TABLE[bits]
        if scale is not None:
            x = x * scale.astype(np.float64)[..., None]
        return x
    raise ValueError(dtype)


def encode(x: np.ndarray, dtype: str) -> np.ndarray:
    """float64 -> stored bits with ONE round-to-nearest-even (pooled-cache storage)."""
    x = np.asarray(x, dtype=np.float64)
    if dtype == F32:
        return x.astype(np.float32)
    if dtype == BF16:
        # bf16 keeps 8 significant bits; quantum = 2^(e-8) with frexp's e, floored at the
        # subnormal quantum 2^-133.  np.rint rounds half to even.
        _, e = np.frexp(x)
        qe = np.maximum(e - 8, -133)
        r = np.ldexp(np.rint(np.ldexp(x, -qe)), qe)
        f = r.astype(np.float32)            # exact: r has <= 8 significant bits
        assert np.all(f.astype(np.float64) == r)
        return (f.view(np.uint32) >> 16).astype(np.uint16)
    raise ValueError(dtype)


# ----------------------------------------------------------------------------- Eq. 4: pooling
def pool_blocks(keys: np.ndarray, k_dtype: str, k_scale, seq_len: np.ndarray, B: int,
                pooled_dtype: str, mode: str = "mean") -> np.ndarray:
    """Eq. 4 / Algorithm 1 pooling loop.  keys [n_seq, s_max, d] stored bits -> pooled stored bits
    [n_seq, s_max/B, d].  Block b of sequence n holds tokens bB .. min((b+1)B, seq_len[n]) - 1;
    blocks with no token are written as zeros.  mode "mean" is the paper's method; "max" is the
    per-dimension maximum the paper names as a possible other Pool (Section 4.1 writes Pool
    generically; its closing discussion lists max-pooling as future work)."""
    assert mode in ("mean", "max")
    n_seq, s_max, d = keys.shape
    assert s_max % B == 0
    M = s_max // B
    out = np.zeros((n_seq, M, d), dtype=np.float64)
    for n in range(n_seq):
        L = int(seq_len[n])
        for b in range(-(-L // B)):
            lo, hi = b * B, min((b + 1) * B, L)
            sc = None if k_scale is None else k_scale[n, lo:hi]
            kb = decode(keys[n, lo:hi], k_dtype, sc)
            out[n, b] = kb.sum(axis=0) / float(hi - lo) if mode == "mean" else kb.max(axis=0)
    return encode(out, pooled_dtype)


# ----------------------------------------------------------------------------- Eq. 1 / 5: score
def score(q_t: np.ndarray, w_t: np.ndarray, keys: np.ndarray) -> np.ndarray:
    """Eq. 1 (Eq. 5 when `keys` are pooled keys).  q_t [H, d], w_t [H], keys [n, d], float64.
    Returns [n]: sum_j w_j * max(0, q_j . k_s)."""
    dots = q_t @ keys.T                      # [H, n]
    return w_t @ np.maximum(dots, 0.0) + 0.0  # "+ 0.0": -0 -> +0


def top_select(scores: np.ndarray, ids: np.ndarray, budget: int) -> np.ndarray:
    """TopK of Eqs. 2, 6, 9: the `budget` best by (score descending, id ascending); everything if
    there are no more than `budget` entries.  Returns the chosen ids in ascending order."""
    if scores.size <= budget:
        return np.sort(ids)
    order = np.lexsort((ids, -scores))       # last key is primary
    return np.sort(ids[order[:budget]])


# ----------------------------------------------------------------------------- Stage 1
def select_blocks(J: np.ndarray, m: int, b0: int = 0) -> np.ndarray:
    """Eq. 6 with the causal rule and the forced blocks (Section 4.1, Stage 1).
    J holds the scores of the visible blocks b0 .. b_t.  Block b0 (first) and block b_t (the one
    containing the query) are always kept and count inside the budget m.  Returns block ids."""
    n_vis = J.size
    if n_vis <= m:
        return b0 + np.arange(n_vis, dtype=np.int64)
    assert m >= 2, "m >= 2 is needed to hold the two forced blocks"
    last = n_vis - 1
    inner = np.arange(1, last, dtype=np.int64)
    kept = top_select(J[1:last], inner, m - 2)
    return b0 + np.sort(np.concatenate([[0], kept, [last]]).astype(np.int64))


def hisa_block_score_topk(*, q, q_dtype, w, q_seq, q_pos, pooled, pooled_dtype, B, m,
                          queries=None, q_lo=None):
    """Stage 1 for the listed queries.  pooled: stored bits [n_seq, M, d].  q_lo: first visible
    position per query (None: 0).
    Returns (block_idx [n, m] int32 ascending then -1, J [n, M] float64 with -inf for invisible
    blocks)."""
    T = q.shape[0]
    queries = np.arange(T) if queries is None else np.asarray(queries)
    M = pooled.shape[1]
    block_idx = np.full((queries.size, m), -1, dtype=np.int32)
    Jout = np.full((queries.size, M), -np.inf, dtype=np.float64)
    for i, t in enumerate(queries):
        n = 0 if q_seq is None else int(q_seq[t])
        b_t = int(q_pos[t]) // B
        b_0 = 0 if q_lo is None else int(q_lo[t]) // B
        if b_t < b_0:
            continue                          # the query sees no key
        qt = decode(q[t], q_dtype)
        pk = decode(pooled[n, b_0:b_t + 1], pooled_dtype)
        J = score(qt, w[t].astype(np.float64), pk)
        Jout[i, b_0:b_t + 1] = J
        C = select_blocks(J, m, b_0)
        block_idx[i, :C.size] = C
    return block_idx, Jout


# ----------------------------------------------------------------------------- Stage 2
def candidate_tokens(C: np.ndarray, pos: int, B: int, lo: int = 0) -> np.ndarray:
    """Eq. 7 with the causal mask: tokens of the kept blocks that the query can see
    (lo <= s <= pos), ascending."""
    toks = (C[:, None] * B + np.arange(B, dtype=np.int64)[None, :]).reshape(-1)
    return toks[(toks <= pos) & (toks >= lo)]


def hisa_token_refine_topk(*, q, q_dtype, w, q_seq, q_pos, keys, k_dtype, k_scale, B, m,
                           block_idx, k, queries=None, q_lo=None):
    """Stage 2 (Eqs. 8-9) for the listed queries; block_idx [n, m] is aligned with `queries`.
    Returns (topk_idx [n, k] int32 ascending then -1, topk_scores [n, k] float64 (nan padding),
    cand_scores [n, m*B] float64, slot c = (kept block c//B, offset c%B), -inf where masked)."""
    T = q.shape[0]
    queries = np.arange(T) if queries is None else np.asarray(queries)
    topk_idx = np.full((queries.size, k), -1, dtype=np.int32)
    topk_scores = np.full((queries.size, k), np.nan, dtype=np.float64)
    cand_scores = np.full((queries.size, m * B), -np.inf, dtype=np.float64)
    for i, t in enumerate(queries):
        n = 0 if q_seq is None else int(q_seq[t])
        pos = int(q_pos[t])
        lo = 0 if q_lo is None else int(q_lo[t])
        C = block_idx[i][block_idx[i] >= 0].astype(np.int64)
        toks = candidate_tokens(C, pos, B, lo)
        sc = None if k_scale is None else k_scale[n, toks]
        kc = decode(keys[n, toks], k_dtype, sc)
        I = score(decode(q[t], q_dtype), w[t].astype(np.float64), kc)
        if toks.size:                         # slot of token s: its kept block's rank * B + s % B
            rank = np.searchsorted(C, toks // B)
            cand_scores[i, rank * B + toks % B] = I
        sel = top_select(I, toks, k)
        topk_idx[i, :sel.size] = sel
        lookup = dict(zip(toks.tolist(), I.tolist()))
        topk_scores[i, :sel.size] = [lookup[s] for s in sel.tolist()]
    return topk_idx, topk_scores, cand_scores


def hisa_indexer(*, q, q_dtype, w, q_seq, q_pos, keys, k_dtype, k_scale, seq_len, B, m, k,
                 pooled_dtype, queries=None, pooled=None, q_lo=None):
    """Algorithm 1 end to end for the listed queries.  Returns dict with pooled, block_idx, J,
    topk_idx, topk_scores, cand_scores."""
    if pooled is None:
        pooled = pool_blocks(keys, k_dtype, k_scale, seq_len, B, pooled_dtype)
    block_idx, J = hisa_block_score_topk(q=q, q_dtype=q_dtype, w=w, q_seq=q_seq, q_pos=q_pos,
                                         pooled=pooled, pooled_dtype=pooled_dtype, B=B, m=m,
                                         queries=queries, q_lo=q_lo)
    topk_idx, topk_scores, cand = hisa_token_refine_topk(
        q=q, q_dtype=q_dtype, w=w, q_seq=q_seq, q_pos=q_pos, keys=keys, k_dtype=k_dtype,
        k_scale=k_scale, B=B, m=m, block_idx=block_idx, k=k, queries=queries, q_lo=q_lo)
    return dict(pooled=pooled, block_idx=block_idx, J=J, topk_idx=topk_idx,
                topk_scores=topk_scores, cand_scores=cand)


# ----------------------------------------------------------------------------- flat DSA (Eqs. 1-2)
def dsa_flat_indexer_topk(*, q, q_dtype, w, q_seq, q_pos, keys, k_dtype, k_scale, k,
                          queries=None, return_scores=False, chunk=16384, q_lo=None):
    """Eqs. 1-2 over the whole causal prefix lo_t <= s <= pos_t (lo_t = 0 unless q_lo is given).
    Returns (topk_idx [n, k] int32 ascending then -1, topk_scores [n, k] float64) and, if asked,
    the list of full score rows (row i covers the positions lo_t .. pos_t)."""
    T = q.shape[0]
    queries = np.arange(T) if queries is None else np.asarray(queries)
    topk_idx = np.full((queries.size, k), -1, dtype=np.int32)
    topk_scores = np.full((queries.size, k), np.nan, dtype=np.float64)
    rows = []
    for i, t in enumerate(queries):
        n = 0 if q_seq is None else int(q_seq[t])
        pos = int(q_pos[t])
        qt = decode(q[t], q_dtype)
        wt = w[t].astype(np.float64)
        first = 0 if q_lo is None else int(q_lo[t])
        I = np.empty(max(pos + 1 - first, 0), dtype=np.float64)
        for lo in range(first, pos + 1, chunk):   # chunked only to bound the float64 copy of the keys
            hi = min(lo + chunk, pos + 1)
            sc = None if k_scale is None else k_scale[n, lo:hi]
            I[lo - first:hi - first] = score(qt, wt, decode(keys[n, lo:hi], k_dtype, sc))
        sel = top_select(I, np.arange(first, pos + 1, dtype=np.int64), k)
        topk_idx[i, :sel.size] = sel
        topk_scores[i, :sel.size] = I[sel - first]
        if return_scores:
            rows.append(I)
    if return_scores:
        return topk_idx, topk_scores, rows
    return topk_idx, topk_scores


# ----------------------------------------------------------------------------- Eq. 12 diagnostic
def iou(a: np.ndarray, b: np.ndarray) -> float:
    """Eq. 12: |A & B| / |A | B| over the valid (>= 0) entries of two index rows."""
    sa, sb = set(a[a >= 0].tolist()), set(b[b >= 0].tolist())
    u = len(sa | sb)
    return 1.0 if u == 0 else len(sa & sb) / u
