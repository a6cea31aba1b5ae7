"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without a GPU.

Each test targets a mistake that would otherwise go unnoticed: a wrong sign or index, a dropped
gate, a transposed operand, a wrong tie rule, a forced block outside the budget, a wrong divisor.
"""
import json
import os

import numpy as np
import pytest
import torch

from oracle import hisa_oracle as O
from paper_2603_28458_amd import workloads as W
from tests.util import oracle_args, oracle_flat, oracle_hisa

HERE = os.path.dirname(os.path.abspath(__file__))


# ------------------------------------------------------------------ stored formats
def test_fp8_table_matches_library_decode_on_all_codes():
    codes = torch.arange(256, dtype=torch.uint8)
    lib = codes.view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    tab = O.fp8_e4m3fn_table()
    assert np.array_equal(np.isnan(lib), np.isnan(tab))
    ok = ~np.isnan(lib)
    assert np.array_equal(lib[ok], tab[ok])
    assert tab[0x7E] == 448.0 and tab[0x01] == 2.0 ** -9 and tab[0x08] == 2.0 ** -6


def test_bf16_decode_and_encode_match_library_cast():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-6, 6, 20000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e-39, -7.1e-40]])
    x32 = x.astype(np.float32)
    lib_bits = torch.from_numpy(x32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    # fp32 -> bf16 in the library is one RNE rounding of an fp32 value; so is encode() on it.
    assert np.array_equal(O.encode(x32.astype(np.float64), "bf16"), lib_bits)
    back = torch.from_numpy(lib_bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(O.decode(lib_bits, "bf16"), back.astype(np.float64))


def test_bf16_encode_rounds_a_double_once():
    # 1 + 2^-8 + 2^-30 lies just above the bf16 halfway point 1 + 2^-8: one rounding goes up,
    # rounding through fp32 first (-> exactly halfway -> even) would go down.
    x = np.array([1.0 + 2.0 ** -8 + 2.0 ** -30])
    assert O.decode(O.encode(x, "bf16"), "bf16")[0] == 1.0 + 2.0 ** -7


# ------------------------------------------------------------------ Eq. 4
@pytest.mark.parametrize("k_dtype", ["f32", "bf16", "fp8_e4m3"])
def test_pooled_keys_are_block_means(k_dtype):
    wl = W.make_workload("p", seq_len=200, T=8, H=2, d=16, B=32, m=2, k=8, q_dtype="f32" if k_dtype == "f32" else "bf16",
                         k_dtype=k_dtype, pooled_dtype="f32", seed=5)
    pooled = O.pool_blocks(wl.keys, wl.k_dtype, wl.k_scale, wl.seq_len, wl.B, "f32")
    if k_dtype == "fp8_e4m3":
        kf = torch.from_numpy(wl.keys).view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
        kf = kf * wl.k_scale.astype(np.float64)[..., None]
    elif k_dtype == "bf16":
        kf = torch.from_numpy(wl.keys.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy().astype(np.float64)
    else:
        kf = wl.keys.astype(np.float64)
    assert pooled.shape == (1, 7, 16)
    for b in range(7):
        hi = min(200, (b + 1) * 32)
        want = np.mean(kf[0, b * 32:hi], axis=0)          # partial block: divide by the count (8)
        np.testing.assert_allclose(pooled[0, b].astype(np.float64), want, rtol=1e-6, atol=1e-7)


def test_max_pool_variant_pins():
    # per-dimension maximum: identical keys give that key; never below the mean; a one-token block is
    # the token; equals a pure-Python maximum; fp8 keys are compared after dequantisation
    keys = np.zeros((1, 64, 4), dtype=np.float32)
    keys[0] = [1.5, -2.25, 0.0, 7.0]
    assert np.array_equal(O.pool_blocks(keys, "f32", None, np.array([64]), 16, "f32", mode="max")[0],
                          np.tile([1.5, -2.25, 0.0, 7.0], (4, 1)).astype(np.float32))
    rng = np.random.default_rng(17)
    keys = rng.standard_normal((2, 48, 8)).astype(np.float32)
    lens = np.array([48, 33])
    mx = O.pool_blocks(keys, "f32", None, lens, 16, "f32", mode="max")
    mean = O.pool_blocks(keys, "f32", None, lens, 16, "f32", mode="mean")
    assert np.all(mx[0] >= mean[0]) and np.all(mx[1, :3] >= mean[1, :3])
    assert np.array_equal(mx[1, 2], keys[1, 32])                     # one token present in block 2
    for n in range(2):
        for b in range(-(-int(lens[n]) // 16)):
            for i in range(8):
                want = max(float(keys[n, s, i]) for s in range(16 * b, min(16 * b + 16, int(lens[n]))))
                assert mx[n, b, i] == np.float32(want)
    wl = W.make_workload("mx8", seq_len=64, T=64, H=2, d=16, B=16, m=2, k=16, q_dtype="bf16", k_dtype="fp8_e4m3",
                         pooled_dtype="f32", seed=18)
    deq = O.decode(wl.keys, "fp8_e4m3", wl.k_scale)[0]
    got = O.pool_blocks(wl.keys, "fp8_e4m3", wl.k_scale, wl.seq_len, 16, "f32", mode="max")[0]
    assert np.array_equal(got, deq.reshape(4, 16, 16).max(axis=1).astype(np.float32))


def test_pool_of_identical_keys_is_that_key_and_empty_blocks_are_zero():
    keys = np.zeros((2, 64, 4), dtype=np.float32)
    keys[0, :, :] = [1.5, -2.25, 0.0, 7.0]
    keys[1, :20, :] = [0.5, 0.5, -1.0, 3.0]
    pooled = O.pool_blocks(keys, "f32", None, np.array([64, 20]), 16, "f32")
    assert np.array_equal(pooled[0], np.tile([1.5, -2.25, 0.0, 7.0], (4, 1)).astype(np.float32))
    assert np.array_equal(pooled[1, 0], [0.5, 0.5, -1.0, 3.0])
    assert np.array_equal(pooled[1, 1], [0.5, 0.5, -1.0, 3.0])     # 4 tokens present, mean over 4
    assert np.array_equal(pooled[1, 2:], np.zeros((2, 4), dtype=np.float32))


# ------------------------------------------------------------------ Eq. 1 / Eq. 5
def test_single_head_unit_gate_positive_dots_is_inner_product_search():
    rng = np.random.default_rng(1)
    q = np.abs(rng.standard_normal((1, 8)))
    K = np.abs(rng.standard_normal((50, 8)))
    s = O.score(q, np.ones(1), K)
    np.testing.assert_allclose(s, (K @ q[0]), rtol=1e-14)


def test_score_homogeneity_head_permutation_and_relu():
    rng = np.random.default_rng(2)
    q = rng.standard_normal((6, 16))
    w = rng.standard_normal(6)                # gates of either sign
    K = rng.standard_normal((40, 16))
    s = O.score(q, w, K)
    np.testing.assert_allclose(O.score(3.5 * q, w, K), 3.5 * s, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(O.score(q, 0.25 * w, K), 0.25 * s, rtol=1e-13, atol=1e-13)
    perm = rng.permutation(6)
    np.testing.assert_allclose(O.score(q[perm], w[perm], K), s, rtol=1e-13, atol=1e-13)
    # independent evaluation, term by term
    ref = np.array([sum(w[j] * max(0.0, float(np.dot(q[j], K[i]))) for j in range(6)) for i in range(40)])
    np.testing.assert_allclose(s, ref, rtol=1e-13, atol=1e-13)
    # the gate multiplies AFTER the ReLU: a negative gate on a negative dot contributes 0
    assert O.score(np.array([[1.0]]), np.array([-2.0]), np.array([[-3.0]]))[0] == 0.0
    assert O.score(np.array([[1.0]]), np.array([-2.0]), np.array([[3.0]]))[0] == -6.0


def test_all_dots_nonpositive_gives_zero_scores_and_lowest_indices():
    q = np.ones((3, 4), dtype=np.float32)
    keys = -np.abs(np.random.default_rng(3).standard_normal((1, 64, 4))).astype(np.float32)
    idx, sc = O.dsa_flat_indexer_topk(q=q[None], q_dtype="f32", w=np.ones((1, 3), np.float32), q_seq=None,
                                      q_pos=np.array([63]), keys=keys, k_dtype="f32", k_scale=None, k=10)
    assert np.array_equal(idx[0], np.arange(10))
    assert np.all(sc[0] == 0.0)


# ------------------------------------------------------------------ hand-worked example
def test_hand_worked_example():
    g = json.load(open(os.path.join(HERE, "golden", "hand_example.json")))
    keys = np.array(g["keys"], dtype=np.float32)[None]
    q = np.array(g["q"], dtype=np.float32)[None]
    w = np.array(g["w"], dtype=np.float32)[None]
    L, B = g["L"], g["B"]
    pooled = O.pool_blocks(keys, "f32", None, np.array([L]), B, "f32")
    assert np.array_equal(pooled[0], np.array(g["pooled"], dtype=np.float32))
    _, _, rows = O.dsa_flat_indexer_topk(q=q, q_dtype="f32", w=w, q_seq=None, q_pos=np.array([L - 1]), keys=keys,
                                         k_dtype="f32", k_scale=None, k=3, return_scores=True)
    assert rows[0].tolist() == g["token_scores"]
    for c in g["cases"]:
        pos = np.array([c["pos"]])
        r = O.hisa_indexer(q=q, q_dtype="f32", w=w, q_seq=None, q_pos=pos, keys=keys, k_dtype="f32", k_scale=None,
                           seq_len=np.array([L]), B=B, m=c["m"], k=c["k"], pooled_dtype="f32")
        nb = c["pos"] // B + 1
        assert r["J"][0, :nb].tolist() == g["block_scores"][:nb]
        assert np.all(np.isneginf(r["J"][0, nb:]))
        bi = r["block_idx"][0]
        assert bi[bi >= 0].tolist() == c["blocks"], c
        ti = r["topk_idx"][0]
        assert ti[ti >= 0].tolist() == c["hisa"], c
        # Eq. 8 in the slot layout of the candidate-score output (kept block rank * B + offset)
        want_cand = [-np.inf if v == "-inf" else float(v) for v in c["cand_scores"]]
        assert r["cand_scores"][0].tolist() == want_cand, c
        fi, _ = O.dsa_flat_indexer_topk(q=q, q_dtype="f32", w=w, q_seq=None, q_pos=pos, keys=keys, k_dtype="f32",
                                        k_scale=None, k=c["k"])
        assert fi[0][fi[0] >= 0].tolist() == c["flat"], c


# ------------------------------------------------------------------ brute force on tiny inputs
def _brute_force(wl, t, m, k):
    """Algorithm 1 and Eqs. 1-2 with Python floats, loops and sorted(); shares nothing with the
    oracle except the stored inputs (fp32 here)."""
    K = wl.keys[0].astype(float).tolist()
    Q = wl.q[t].astype(float).tolist()
    Wt = wl.w[t].astype(float).tolist()
    pos = int(wl.positions()[t])
    B, d, H = wl.B, wl.d, wl.H

    def sc(vec):
        tot = 0.0
        for j in range(H):
            dot = 0.0
            for i in range(d):
                dot += Q[j][i] * vec[i]
            if dot > 0:
                tot += Wt[j] * dot
        return tot

    L = int(wl.seq_len[0])
    flat = sorted(range(pos + 1), key=lambda s: (-sc(K[s]), s))[:k]
    b_t = pos // B
    pooled = []
    for b in range(b_t + 1):
        toks = range(b * B, min((b + 1) * B, L))
        v = [float(np.float32(sum(K[s][i] for s in toks) / len(toks))) for i in range(d)]
        pooled.append(v)
    if b_t + 1 <= m:
        C = list(range(b_t + 1))
    else:
        inner = sorted(range(1, b_t), key=lambda b: (-sc(pooled[b]), b))[:m - 2]
        C = sorted([0, b_t] + inner)
    cand = [s for b in C for s in range(b * B, (b + 1) * B) if s <= pos]
    hisa = sorted(cand, key=lambda s: (-sc(K[s]), s))[:k]
    return C, sorted(hisa), sorted(flat)


def test_brute_force_on_tiny_inputs():
    wl = W.make_workload("bf", seq_len=77, T=77, H=3, d=5, B=8, m=4, k=12, q_dtype="f32", k_dtype="f32", seed=11)
    r = oracle_hisa(wl)
    f, _ = oracle_flat(wl)
    for t in range(wl.T):
        C, hisa, flat = _brute_force(wl, t, wl.m, wl.k)
        bi = r["block_idx"][t]
        assert bi[bi >= 0].tolist() == C, t
        ti = r["topk_idx"][t]
        assert ti[ti >= 0].tolist() == hisa, t
        assert f[t][f[t] >= 0].tolist() == flat, t


# ------------------------------------------------------------------ regimes of Section 4.1
def _small(seed=21, **kw):
    p = dict(seq_len=300, T=300, H=4, d=16, B=16, m=5, k=24, q_dtype="f32", k_dtype="f32", seed=seed)
    p.update(kw)
    return W.make_workload("s", **p)


def test_m_covering_all_blocks_reproduces_flat_dsa():
    wl = _small(m=19)                      # 19 blocks of 16 cover 300 tokens
    r = oracle_hisa(wl)
    f, fs = oracle_flat(wl)
    assert np.array_equal(r["topk_idx"], f)
    np.testing.assert_array_equal(r["topk_scores"], fs)


def test_queries_inside_the_capacity_mB_match_flat_and_short_prefixes_select_everything():
    wl = _small()
    r = oracle_hisa(wl)
    f, _ = oracle_flat(wl)
    pos = wl.positions()
    for t in range(wl.T):
        if pos[t] + 1 <= wl.m * wl.B:      # regime 2: all visible blocks kept
            assert np.array_equal(r["topk_idx"][t], f[t]), t
        if pos[t] + 1 <= wl.k:             # regime 1: dense
            assert r["topk_idx"][t][:pos[t] + 1].tolist() == list(range(pos[t] + 1))
            assert np.all(r["topk_idx"][t][pos[t] + 1:] == -1)
    # the boundaries themselves: pos+1 in {k, k+1, mB, mB+1}, block edges
    for p in (wl.k - 1, wl.k, wl.m * wl.B - 1, wl.m * wl.B):
        n_valid = int((r["topk_idx"][p] >= 0).sum())
        assert n_valid == min(wl.k, p + 1)


def test_block_size_one_makes_stage_one_equal_token_scoring():
    # B = 1: pooled key = token key, J = I; with m >= k + 2 every flat top-k token survives Stage 1.
    wl = _small(B=1, m=40, k=24, seq_len=120, T=120)
    r = oracle_hisa(wl)
    f, _ = oracle_flat(wl)
    assert np.array_equal(r["topk_idx"], f)


def test_forced_blocks_budget_and_order():
    wl = _small()
    r = oracle_hisa(wl)
    pos = wl.positions()
    for t in range(wl.T):
        bi = r["block_idx"][t]
        v = bi[bi >= 0]
        b_t = pos[t] // wl.B
        assert v.size == min(wl.m, b_t + 1)              # forced blocks are inside the budget
        assert v[0] == 0 and v[-1] == b_t                # first block and own block always kept
        assert np.all(np.diff(v) > 0) and np.all(bi[v.size:] == -1)
        assert v.max() <= b_t                            # causal: nothing after the own block
        # the free slots hold the best-scoring inner blocks
        if b_t + 1 > wl.m:
            J = r["J"][t]
            inner_kept = [b for b in v if b not in (0, b_t)]
            inner_dropped = [b for b in range(1, b_t) if b not in v]
            assert min(J[inner_kept]) >= max(J[inner_dropped])


def test_hisa_differs_from_flat_only_through_dropped_blocks():
    # Failure-case analysis (Appendix C): inside a kept block the score is DSA's own, so every flat
    # winner that lies in Omega_t is also a HISA winner, and if all flat winners lie in Omega_t the
    # two sets are equal.
    wl = _small(seed=33)
    r = oracle_hisa(wl)
    f, _ = oracle_flat(wl)
    n_diff = 0
    for t in range(wl.T):
        bi = r["block_idx"][t]
        kept = set(bi[bi >= 0].tolist())
        flat = set(f[t][f[t] >= 0].tolist())
        hisa = set(r["topk_idx"][t][r["topk_idx"][t] >= 0].tolist())
        inside = {s for s in flat if s // wl.B in kept}
        assert inside <= hisa, t
        if inside == flat:
            assert hisa == flat, t
        else:
            n_diff += 1
        assert len(hisa) == min(wl.k, len([s for b in kept for s in range(b * wl.B, (b + 1) * wl.B)
                                           if s <= wl.positions()[t]]))
    assert n_diff > 0                                     # the case is actually exercised


def test_selected_scores_dominate_unselected_candidates_and_work_counts():
    wl = _small(seed=34)
    r = oracle_hisa(wl)
    for t in range(wl.T):
        cs = r["cand_scores"][t]
        n_cand = int(np.isfinite(cs).sum())
        assert n_cand <= wl.m * wl.B                      # Eq. 10: at most mB token scores
        assert int(np.isfinite(r["J"][t]).sum()) <= -(-wl.s_max // wl.B)
        ts = r["topk_scores"][t]
        ts = ts[~np.isnan(ts)]
        if n_cand > wl.k:
            rest = np.sort(cs[:n_cand])[: n_cand - wl.k]
            assert ts.min() >= rest.max()


def test_positive_rescaling_of_a_query_leaves_every_set_unchanged():
    wl = _small(seed=35)
    r1 = oracle_hisa(wl)
    wl.q = (wl.q * np.float32(4.0)).astype(np.float32)    # exact in fp32
    wl.w = (wl.w * np.float32(0.5)).astype(np.float32)
    r2 = oracle_hisa(wl)
    assert np.array_equal(r1["block_idx"], r2["block_idx"])
    assert np.array_equal(r1["topk_idx"], r2["topk_idx"])


def test_decode_layout_and_subset_of_queries():
    wl = W.make_workload("dec", n_seq=3, seq_len=[100, 64, 37], T=3, H=4, d=16, B=16, m=3, k=20, q_dtype="bf16",
                         k_dtype="bf16", mode="decode", seed=8)
    r = oracle_hisa(wl)
    for t in range(3):
        ti = r["topk_idx"][t]
        assert ti[ti >= 0].max() <= wl.seq_len[t] - 1
    sub = oracle_hisa(wl, queries=[2, 0])
    assert np.array_equal(sub["topk_idx"][0], r["topk_idx"][2])
    assert np.array_equal(sub["topk_idx"][1], r["topk_idx"][0])


# ------------------------------------------------------------------ packed sequences (first visible position)
def _varlen(lens, seed=31, **kw):
    p = dict(n_seq=len(lens), seq_len=lens, T=int(sum(lens)), H=3, d=8, B=8, m=4, k=10, q_dtype="f32",
             k_dtype="f32", mode="varlen", seed=seed)
    p.update(kw)
    return W.make_workload("v", **p)


def test_packed_sequences_on_block_boundaries_equal_the_padded_layout():
    # every sequence a multiple of B long: the packed stream's blocks are the sequences' own blocks,
    # so each query must keep the same blocks and tokens, shifted by its sequence's start
    wl = _varlen([40, 16, 64, 8])
    pk = W.pack(wl)
    a, b = oracle_hisa(wl), oracle_hisa(pk)
    fa, _ = oracle_flat(wl)
    fb, _ = oracle_flat(pk)
    lo = pk.q_lo.astype(np.int64)
    for t in range(wl.T):
        for x, y, unit in ((a["block_idx"][t], b["block_idx"][t], wl.B), (a["topk_idx"][t], b["topk_idx"][t], 1),
                           (fa[t], fb[t], 1)):
            assert np.array_equal(np.where(x >= 0, x + lo[t] // unit, -1), y), t
    np.testing.assert_array_equal(a["topk_scores"], b["topk_scores"])


def test_zero_first_position_is_the_plain_indexer():
    wl = _small()
    r0 = oracle_hisa(wl)
    wl.q_lo = np.zeros(wl.T, dtype=np.int32)
    r1 = oracle_hisa(wl)
    for key in ("block_idx", "topk_idx", "J", "cand_scores"):
        np.testing.assert_array_equal(r0[key], r1[key])


def _brute_force_packed(pk, t):
    """Section 4.1 on a packed stream with Python floats, loops and sorted(): blocks of the stream,
    pooled over everything they hold, visible blocks lo // B .. pos // B with both ends forced,
    tokens lo .. pos of the kept blocks."""
    K = pk.keys[0].astype(float).tolist()
    Q = pk.q[t].astype(float).tolist()
    Wt = pk.w[t].astype(float).tolist()
    pos, lo = int(pk.q_pos[t]), int(pk.q_lo[t])
    B, d, H, m, k = pk.B, pk.d, pk.H, pk.m, pk.k
    L = int(pk.seq_len[0])

    def sc(vec):
        tot = 0.0
        for j in range(H):
            dot = sum(Q[j][i] * vec[i] for i in range(d))
            if dot > 0:
                tot += Wt[j] * dot
        return tot

    b0, b1 = lo // B, pos // B
    pooled = {}
    for b in range(b0, b1 + 1):
        toks = range(b * B, min((b + 1) * B, L))
        pooled[b] = [float(np.float32(sum(K[s][i] for s in toks) / len(toks))) for i in range(d)]
    if b1 - b0 + 1 <= m:
        C = list(range(b0, b1 + 1))
    else:
        inner = sorted(range(b0 + 1, b1), key=lambda b: (-sc(pooled[b]), b))[:m - 2]
        C = sorted([b0, b1] + inner)
    cand = [s for b in C for s in range(b * B, (b + 1) * B) if lo <= s <= pos]
    hisa = sorted(sorted(cand, key=lambda s: (-sc(K[s]), s))[:k])
    flat = sorted(sorted(range(lo, pos + 1), key=lambda s: (-sc(K[s]), s))[:k])
    return C, hisa, flat


def test_packed_sequences_with_straddling_blocks_brute_force_and_invariants():
    wl = _varlen([37, 5, 61, 19, 3], seed=32)           # starts 0, 37, 42, 103, 122: blocks straddle
    pk = W.pack(wl)
    r = oracle_hisa(pk)
    f, _ = oracle_flat(pk)
    lo, pos = pk.q_lo.astype(np.int64), pk.q_pos.astype(np.int64)
    assert np.any(lo % pk.B != 0)
    for t in range(pk.T):
        C, hisa, flat = _brute_force_packed(pk, t)
        bi = r["block_idx"][t][r["block_idx"][t] >= 0]
        ti = r["topk_idx"][t][r["topk_idx"][t] >= 0]
        assert bi.tolist() == C and ti.tolist() == hisa and f[t][f[t] >= 0].tolist() == flat, t
        # the first and the last visible block are kept, the budget holds, nothing outside [lo, pos]
        n_vis = pos[t] // pk.B - lo[t] // pk.B + 1
        assert bi[0] == lo[t] // pk.B and bi[-1] == pos[t] // pk.B and bi.size == min(pk.m, n_vis)
        assert ti.min() >= lo[t] and ti.max() <= pos[t] and ti.size == min(pk.k, pos[t] - lo[t] + 1)
        if n_vis <= pk.m:                                # every visible block kept: HISA = flat
            assert ti.tolist() == flat, t


def test_iou_definition():
    assert O.iou(np.array([1, 2, 3, -1]), np.array([2, 3, 4, 5])) == 2 / 5
    assert O.iou(np.array([1, 2]), np.array([2, 1])) == 1.0


def test_planted_mistakes_are_caught_by_the_pins():
    """The pins above are only worth something if a plausible slip fails them: plant three slips in
    copies of the oracle's arithmetic and check that the hand example / brute force disagree."""
    g = json.load(open(os.path.join(HERE, "golden", "hand_example.json")))
    K = np.array(g["keys"], dtype=np.float64)
    q = np.array(g["q"], dtype=np.float64)
    w = np.array(g["w"], dtype=np.float64)
    good = O.score(q, w, K)
    assert good.tolist() == g["token_scores"]
    gate_before_relu = np.maximum(w[:, None] * (q @ K.T), 0.0).sum(axis=0)
    dropped_gate = np.maximum(q @ K.T, 0.0).sum(axis=0)
    no_relu = w @ (q @ K.T)
    assert dropped_gate.tolist() != g["token_scores"]
    assert no_relu.tolist() != g["token_scores"]
    # gate-before-ReLU only shows with a negative gate (covered in the homogeneity test)
    assert gate_before_relu.tolist() == g["token_scores"]
    neg = O.score(np.array([[1.0]]), np.array([-2.0]), np.array([[3.0]]))[0]
    assert neg == -6.0 and max(-2.0 * 3.0, 0.0) != neg
    # higher index winning ties, or forced blocks outside the budget, both break the hand example
    assert sorted(sorted(range(6), key=lambda s: (-g["token_scores"][s], -s))[:5]) != g["cases"][3]["flat"]
    assert len(g["cases"][1]["blocks"]) == g["cases"][1]["m"]
