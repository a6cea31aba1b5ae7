"""Parity of the HIP library against the CPU oracle, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest
import torch

from paper_2603_28458_amd import workloads as W
from tests.parity import run_and_check, sample_queries

pytestmark = pytest.mark.gpu


def _run(wl, **kw):
    print(f"\n[parity] {wl.name}: T={wl.T} H={wl.H} d={wl.d} B={wl.B} m={wl.m} k={wl.k} "
          f"q={wl.q_dtype} k={wl.k_dtype} n_seq={wl.n_seq} s_max={wl.s_max} seed={wl.seed}", flush=True)
    st = run_and_check(wl, verbose=True, **kw)
    return st


def test_tiny_fp32_config_all_queries():
    st = _run(W.config("tiny_f32"))
    assert st["block_swaps"] == 0 and st["token_swaps"] == 0 and st["flat_swaps"] == 0


@pytest.mark.parametrize("k_dtype", ["bf16", "fp8_e4m3"])
def test_small_prefill_ragged_tail(k_dtype):
    # 1467 tokens: 11 full blocks of 128 and a ragged one of 59; several 64-key tiles per query
    wl = W.make_workload(f"small_{k_dtype}", seq_len=1467, T=1467, H=64, d=128, B=128, m=4, k=256,
                         q_dtype="bf16", k_dtype=k_dtype, n_needles=4, seed=101)
    _run(wl)


@pytest.mark.parametrize("B,m,k", [(32, 8, 128), (64, 6, 200), (256, 3, 512)])
def test_block_sizes(B, m, k):
    wl = W.make_workload(f"B{B}", seq_len=2100, T=2100, H=64, d=128, B=B, m=m, k=k, q_dtype="bf16",
                         k_dtype="bf16", seed=102 + B)
    _run(wl, queries=sample_queries(wl, 200))


@pytest.mark.parametrize("B,m", [(64, 128), (512, 16), (2048, 4)])
def test_ablation_block_shapes_at_fixed_candidate_budget(B, m):
    # Appendix C: (B, m) pairs with m*B = 8192 and k = 2048; 512 queries at the end of a 24K prefix
    wl = W.make_workload(f"abl_B{B}", seq_len=24576, T=512, H=64, d=128, B=B, m=m, k=2048, q_dtype="bf16",
                         k_dtype="bf16", seed=140 + m)
    _run(wl, queries=sample_queries(wl, 48))


@pytest.mark.parametrize("k_dtype", ["bf16", "fp8_e4m3"])
def test_more_than_8192_candidates(k_dtype):
    # m*B = 12800 (> 8192): the fused Stage 2 runs 8 waves per query; 320 queries at the end of 20000 keys
    wl = W.make_workload(f"cand12800_{k_dtype}", seq_len=20000, T=320, H=64, d=128, B=128, m=100, k=2048,
                         q_dtype="bf16", k_dtype=k_dtype, seed=145)
    _run(wl, queries=sample_queries(wl, 32))


def test_32_heads_and_fp8():
    wl = W.make_workload("H32", seq_len=900, T=900, H=32, d=128, B=128, m=3, k=300, q_dtype="bf16",
                         k_dtype="fp8_e4m3", seed=103)
    _run(wl, queries=sample_queries(wl, 150))


def test_chunk_against_longer_prefix():
    # 300 queries at the end of a 5000-token prefix (q_pos0 > 0); two-kernel and fused Stage 2
    wl = W.make_workload("chunk", seq_len=5000, T=300, H=64, d=128, B=128, m=8, k=512, q_dtype="bf16",
                         k_dtype="bf16", n_needles=3, seed=104)
    _run(wl)


@pytest.mark.parametrize("k_dtype", ["bf16", "fp8_e4m3"])
def test_decode_batch_ragged_lengths(k_dtype):
    wl = W.make_workload(f"decode_{k_dtype}", n_seq=5, seq_len=[4000, 3333, 129, 128, 1], T=5, H=64, d=128,
                         B=128, m=6, k=512, q_dtype="bf16", k_dtype=k_dtype, mode="decode", seed=105)
    _run(wl)


@pytest.mark.parametrize("H", [64, 32])
def test_decode_batch_with_thousands_of_blocks(H):
    # Stage 1 of a small batch runs in one launch (scores and kept ids stay in LDS): here with 3750
    # blocks per sequence (B = 32), beyond the 2048 that the deeper tile ring covers, ragged lengths,
    # one sequence shorter than a block
    wl = W.make_workload(f"decode_blocks_{H}", n_seq=4, seq_len=[120000, 65537, 40, 99999], T=4, H=H, d=128, B=32,
                         m=40, k=1024, q_dtype="bf16", k_dtype="bf16", mode="decode", n_needles=2, seed=141)
    _run(wl)


@pytest.mark.parametrize("k_dtype", ["bf16", "fp8_e4m3"])
def test_packed_varlen_prefill(k_dtype):
    # three sequences of different lengths prefilled in one call (each starts at a block boundary
    # of its own padded key array): per-query sequence ids and positions, fused Stage 2
    wl = W.make_workload(f"varlen_{k_dtype}", n_seq=3, seq_len=[700, 1300, 257], T=2257, H=64, d=128, B=128,
                         m=4, k=256, q_dtype="bf16", k_dtype=k_dtype, mode="varlen", seed=130)
    _run(wl, queries=sample_queries(wl, 200))


@pytest.mark.parametrize("k_dtype", ["bf16", "fp8_e4m3"])
def test_packed_sequences_with_straddling_blocks(k_dtype):
    # five sequences laid end to end in ONE key stream (Section 4.1: blocks straddle two sequences):
    # starts 0, 700, 2003, 2260, 2263 against B = 128; every query carries its sequence's start as
    # first visible position; two-kernel, fused and single-launch paths, and the flat indexer
    base = W.make_workload(f"pk_{k_dtype}", n_seq=5, seq_len=[700, 1303, 257, 3, 1500], T=3763, H=64, d=128,
                           B=128, m=4, k=256, q_dtype="bf16", k_dtype=k_dtype, mode="varlen", seed=131)
    wl = W.pack(base)
    starts = np.unique(wl.q_lo)
    edge = [int(np.nonzero(wl.q_pos == p)[0][0]) for s in starts for p in (s, s + 1) if np.any(wl.q_pos == p)]
    qs = np.unique(np.concatenate([sample_queries(wl, 200), np.array(edge, dtype=np.int64)]))
    _run(wl, queries=qs)


def test_packed_sequences_in_a_small_batch():
    # at most 256 queries: Stage 1 runs in one launch per batch (scores and kept ids stay in LDS); here
    # with four short sequences end to end in one key stream, blocks of 32 straddling their boundaries,
    # every query of the stream
    base = W.make_workload("pk_small", n_seq=4, seq_len=[70, 33, 101, 45], T=249, H=64, d=128, B=32, m=3, k=64,
                           q_dtype="bf16", k_dtype="bf16", mode="varlen", seed=134)
    _run(W.pack(base))


def test_packed_sequences_fp32_and_long_rows():
    # the fp32 path, and a stream long enough for the streaming top-k of the flat indexer
    base = W.make_workload("pk_f32", n_seq=4, seq_len=[100, 45, 300, 77], T=522, H=4, d=64, B=16, m=4, k=32,
                           q_dtype="f32", k_dtype="f32", mode="varlen", seed=132)
    _run(W.pack(base))
    base = W.make_workload("pk_long", n_seq=2, seq_len=[1001, 19003], T=20004, H=64, d=128, B=128, m=8, k=512,
                           q_dtype="bf16", k_dtype="bf16", mode="varlen", seed=133)
    wl = W.pack(base)
    qs = sample_queries(wl, 24)
    _run(wl, queries=qs, flat_queries=qs[::3])


def test_fp32_generic_shapes():
    wl = W.make_workload("f32_odd", seq_len=777, T=777, H=3, d=20, B=16, m=5, k=50, q_dtype="f32", k_dtype="f32",
                         seed=106)
    _run(wl, queries=sample_queries(wl, 200))
    wl = W.make_workload("f32_dec", n_seq=3, seq_len=[300, 17, 64], T=3, H=8, d=64, B=32, m=4, k=100, q_dtype="f32",
                         k_dtype="f32", mode="decode", seed=107)
    _run(wl)


def test_degenerate_inputs():
    # one token; k larger than every prefix; m covering everything (HISA == flat, Section 4.1)
    wl = W.make_workload("one", seq_len=1, T=1, H=64, d=128, B=128, m=2, k=256, q_dtype="bf16", k_dtype="bf16",
                         seed=108)
    _run(wl)
    wl = W.make_workload("allsel", seq_len=500, T=500, H=64, d=128, B=128, m=4, k=512, q_dtype="bf16",
                         k_dtype="bf16", seed=109)
    st = _run(wl)
    wl = W.make_workload("mcovers", seq_len=1024, T=1024, H=64, d=128, B=128, m=8, k=128, q_dtype="bf16",
                         k_dtype="bf16", seed=110)
    st = _run(wl)
    assert st["iou_hisa_flat"] == 1.0


def test_empty_sequence_in_a_decode_batch():
    # a sequence with no key at all: its query sees nothing, every output row is -1 padding
    wl = W.make_workload("empty_seq", n_seq=3, seq_len=[300, 0, 129], T=3, H=64, d=128, B=128, m=2, k=64,
                         q_dtype="bf16", k_dtype="bf16", mode="decode", seed=170)
    _run(wl)


def test_ties_and_zero_scores():
    # every dot product negative -> every score exactly 0 -> the lowest indices win everywhere
    wl = W.make_workload("zeros", seq_len=1500, T=1500, H=64, d=128, B=128, m=4, k=300, q_dtype="bf16",
                         k_dtype="bf16", seed=111)
    q = np.abs(W._bf16_bits_to_f32(wl.q))
    wl.q = W._to_bf16_bits(q)
    wl.keys = W._to_bf16_bits(-np.abs(W._bf16_bits_to_f32(wl.keys)))
    st = _run(wl, queries=sample_queries(wl, 100))
    assert st["token_swaps"] == 0 and st["flat_swaps"] == 0 and st["block_swaps"] == 0
    # duplicated keys: exact ties between distinct tokens
    wl = W.make_workload("dups", seq_len=1024, T=1024, H=64, d=128, B=128, m=4, k=200, q_dtype="bf16",
                         k_dtype="bf16", seed=112)
    wl.keys[0, 1::2] = wl.keys[0, 0::2]
    _run(wl, queries=sample_queries(wl, 100))


@pytest.mark.parametrize("k_dtype", ["bf16", "fp8_e4m3"])
def test_score_outliers_send_the_fused_topk_to_its_general_select(k_dtype):
    # The fused Stage 2 first tries a one-pass top-k whose bins span the row's own score range; one key
    # with 3000 times the usual norm inside the always-kept first block stretches that range until
    # nearly every candidate shares a bin, and the kernel must fall back to its general select.  A
    # second key of the same size with negative gates stretches the other end.
    wl = W.make_workload(f"outlier_{k_dtype}", seq_len=3000, T=3000, H=64, d=128, B=128, m=8, k=512, q_dtype="bf16",
                         k_dtype=k_dtype, seed=114)
    if k_dtype == "bf16":
        kf = W._bf16_bits_to_f32(wl.keys[0, 5]) * np.float32(3000.0)
        wl.keys[0, 5] = W._to_bf16_bits(kf)
    else:
        wl.k_scale[0, 5] *= np.float32(3000.0)           # the fp8 codes stay, the per-token scale grows
    _run(wl, queries=sample_queries(wl, 150))
    if k_dtype == "bf16":
        # gates of both signs: scores of both signs, the outlier's included.  (bf16 keys only: with signed
        # gates a score is a difference of large terms, and the fp8 path's error, which scales with the
        # terms, is then no longer small against the row maximum the regression bound is stated in.)
        wl.w = (wl.w - np.float32(0.5)).astype(np.float32)
        _run(wl, queries=sample_queries(wl, 150, seed=1))


def test_negative_gates():
    wl = W.make_workload("negw", seq_len=1300, T=1300, H=64, d=128, B=128, m=5, k=256, q_dtype="bf16",
                         k_dtype="bf16", seed=113)
    wl.w = (wl.w - np.float32(0.5)).astype(np.float32)
    _run(wl, queries=sample_queries(wl, 150))


def test_run_to_run_determinism():
    from paper_2603_28458_amd import hisa
    wl = W.make_workload("det", seq_len=3000, T=3000, H=64, d=128, B=128, m=8, k=512, q_dtype="bf16",
                         k_dtype="bf16", seed=114)
    Q, K = hisa.to_device(wl)
    outs = []
    for _ in range(2):
        pooled = hisa.hisa_pool_blocks(K, wl.B)
        bi, _ = hisa.hisa_block_score_topk(Q, K, pooled, hisa.HISA_BF16, wl.B, wl.m)
        ti, _, _ = hisa.hisa_token_refine_topk(Q, K, wl.B, wl.m, bi, wl.k)
        fi, _ = hisa.dsa_flat_indexer_topk(Q, K, wl.k)
        torch.cuda.synchronize()
        outs.append((pooled.clone(), bi.clone(), ti.clone(), fi.clone()))
    for a, b in zip(*outs):
        assert torch.equal(a, b)


def test_incremental_pooled_cache_matches_full_pool_and_oracle():
    # Section 4.1: the pooled cache is maintained while sequences grow (decode).  Grow three sequences
    # by different amounts (within a block, across one boundary, across several) and compare the
    # incrementally updated cache with a full re-pool (bit-exact) and with the oracle's block means.
    from oracle import hisa_oracle as O
    from paper_2603_28458_amd import hisa
    from tests.parity import _np
    from tests.util import check_scores
    for k_dtype in ("bf16", "fp8_e4m3"):
        wl = W.make_workload(f"append_{k_dtype}", n_seq=4, seq_len=[700, 1024, 333, 64], T=4, H=64, d=128, B=128,
                             m=4, k=128, q_dtype="bf16", k_dtype=k_dtype, mode="decode", seed=120)
        print(f"\n[parity] {wl.name}", flush=True)
        Q, K = hisa.to_device(wl)
        prev = np.array([650, 600, 0, 64], dtype=np.int32)          # last one: nothing appended
        K_prev = hisa.Keys(k=K.k, seq_len=torch.from_numpy(prev).cuda(), dtype=K.dtype, k_scale=K.k_scale)
        pooled = hisa.hisa_pool_blocks(K_prev, wl.B)                 # cache as of the previous lengths
        hisa.hisa_pool_append(K, wl.B, K_prev.seq_len, 450, pooled)  # bound >= every growth
        full = hisa.hisa_pool_blocks(K, wl.B)
        torch.cuda.synchronize()
        M = wl.s_max // wl.B
        for n in range(4):                                           # blocks that hold tokens now
            nb = -(-int(wl.seq_len[n]) // wl.B)
            assert torch.equal(pooled[n, :nb], full[n, :nb]), n
        want = O.pool_blocks(wl.keys, wl.k_dtype, wl.k_scale, wl.seq_len, wl.B, "bf16")
        check_scores(O.decode(_np(full), "bf16").reshape(-1, wl.d), O.decode(want, "bf16").reshape(-1, wl.d), 2e-2,
                     "pooled keys")
        # a growth beyond the stated bound is (by contract) not pooled: only the first blocks change
        pooled2 = hisa.hisa_pool_blocks(K_prev, wl.B)
        hisa.hisa_pool_append(K, wl.B, K_prev.seq_len, 0, pooled2)
        torch.cuda.synchronize()
        assert torch.equal(pooled2, hisa.hisa_pool_blocks(K_prev, wl.B))


def test_block_sparse_tokens_and_iou_diagnostic():
    # Block-Sparse baseline (Section 5) = all visible tokens of the kept blocks (Eq. 7 + causal mask),
    # and the IoU of Eq. 12 between HISA's and the flat indexer's selections.
    from oracle import hisa_oracle as O
    from paper_2603_28458_amd import hisa
    wl = W.make_workload("bsparse", seq_len=2500, T=2500, H=64, d=128, B=128, m=5, k=256, q_dtype="bf16",
                         k_dtype="bf16", seed=121)
    print(f"\n[parity] {wl.name}", flush=True)
    Q, K = hisa.to_device(wl)
    pooled = hisa.hisa_pool_blocks(K, wl.B)
    bi, _ = hisa.hisa_block_score_topk(Q, K, pooled, hisa.HISA_BF16, wl.B, wl.m)
    toks = hisa.hisa_block_sparse_tokens(Q, K, wl.B, wl.m, bi)
    ti, _, _ = hisa.hisa_token_refine_topk(Q, K, wl.B, wl.m, bi, wl.k)
    fi, _ = hisa.dsa_flat_indexer_topk(Q, K, wl.k)
    iou = hisa.hisa_index_iou(ti, fi)
    torch.cuda.synchronize()
    bi_h, toks_h, ti_h, fi_h, iou_h = (x.cpu().numpy() for x in (bi, toks, ti, fi, iou))
    pos = wl.positions()
    for t in range(0, wl.T, 7):
        C = bi_h[t][bi_h[t] >= 0].astype(np.int64)
        want = O.candidate_tokens(C, int(pos[t]), wl.B)
        row = toks_h[t]
        assert np.array_equal(row[:want.size], want), t
        assert np.all(row[want.size:] == -1), t
        assert abs(iou_h[t] - O.iou(ti_h[t], fi_h[t])) < 1e-6, t
    assert torch.all(hisa.hisa_index_iou(ti, ti) == 1.0)
    # hand-made rows: both empty (1 by convention), disjoint, nested, partial overlap, full rows of odd width
    kk = 70
    a = torch.full((5, kk), -1, dtype=torch.int32)
    b = torch.full((5, kk), -1, dtype=torch.int32)
    a[1, :3] = torch.tensor([1, 5, 9]); b[1, :2] = torch.tensor([2, 6])                 # disjoint: 0
    a[2, :3] = torch.tensor([1, 5, 9]); b[2, :5] = torch.tensor([0, 1, 5, 9, 12])       # nested: 3 / 5
    a[3, :3] = torch.tensor([1, 5, 9]); b[3, :4] = torch.tensor([5, 7, 9, 11])          # 2 / 5
    a[4] = torch.arange(0, 2 * kk, 2, dtype=torch.int32); b[4] = torch.arange(0, 3 * kk, 3, dtype=torch.int32)
    got = hisa.hisa_index_iou(a.cuda(), b.cuda()).cpu().numpy()
    want = [1.0, 0.0, 0.6, 0.4, O.iou(a[4].numpy(), b[4].numpy())]
    assert np.allclose(got, want, atol=1e-6), (got, want)
    # rows wider than the kernel stages in LDS (k > 4096), ragged valid lengths
    kw = 5000
    rng = np.random.default_rng(3)
    aw = np.full((6, kw), -1, dtype=np.int32)
    bw = np.full((6, kw), -1, dtype=np.int32)
    for r in range(6):
        na, nb = int(rng.integers(0, kw + 1)), int(rng.integers(0, kw + 1))
        aw[r, :na] = np.sort(rng.choice(20000, size=na, replace=False))
        bw[r, :nb] = np.sort(rng.choice(20000, size=nb, replace=False))
    got = hisa.hisa_index_iou(torch.from_numpy(aw).cuda(), torch.from_numpy(bw).cuda()).cpu().numpy()
    want = [O.iou(aw[r], bw[r]) for r in range(6)]
    assert np.allclose(got, want, atol=1e-6), (got, want)


def test_bad_device_side_metadata_stays_in_bounds():
    # seq_len, q_pos, q_lo and block_idx live on the device and cannot be validated by the host: the
    # kernels clamp them.  Whatever they hold, every call must finish and every index it writes
    # must be -1 or a position inside the padded key array.
    from paper_2603_28458_amd import hisa
    wl = W.make_workload("bad_meta", seq_len=2000, T=600, H=64, d=128, B=128, m=4, k=256, q_dtype="bf16",
                         k_dtype="bf16", seed=150)
    print(f"\n[parity] {wl.name}", flush=True)
    Q, K = hisa.to_device(wl)
    s_max, M = K.s_max, K.s_max // wl.B
    dev = Q.q.device

    def run_all(Qx, Kx, bi_in=None):
        pooled = hisa.hisa_pool_blocks(Kx, wl.B)
        bi, _ = hisa.hisa_block_score_topk(Qx, Kx, pooled, hisa.HISA_BF16, wl.B, wl.m)
        use = bi if bi_in is None else bi_in
        outs = [bi]
        outs.append(hisa.hisa_token_refine_topk(Qx, Kx, wl.B, wl.m, use, wl.k)[0])                      # fused
        outs.append(hisa.hisa_token_refine_topk(Qx, Kx, wl.B, wl.m, use, wl.k, want_cand_scores=True)[0])  # two kernels
        outs.append(hisa.hisa_block_sparse_tokens(Qx, Kx, wl.B, wl.m, use))
        outs.append(hisa.dsa_flat_indexer_topk(Qx, Kx, wl.k)[0])
        a_bi, a_ti, _ = hisa.hisa_indexer_topk(Qx, Kx, pooled, hisa.HISA_BF16, wl.B, wl.m, wl.k, want_block_idx=True)
        outs += [a_bi, a_ti]
        torch.cuda.synchronize()
        for j, o in enumerate(outs):
            o = o.cpu().numpy()
            hi = M if j in (0, 5) else s_max
            assert ((o == -1) | ((o >= 0) & (o < hi))).all(), f"output {j} out of range"

    # 1. sequence length far beyond the padded array
    K1 = hisa.Keys(K.k, torch.tensor([s_max + 5000], dtype=torch.int32, device=dev), K.dtype)
    run_all(Q, K1)
    # 2. positions below zero and far beyond the sequence
    pos = torch.arange(600, dtype=torch.int32, device=dev) + 1400
    pos[::3] = -7
    pos[1::3] = 10 ** 9
    Q2 = hisa.Queries(Q.q, Q.w, Q.dtype, q_pos=pos)
    run_all(Q2, K)
    # 2b. first visible positions below zero, past the query, and far beyond the sequence
    lo = torch.arange(600, dtype=torch.int32, device=dev) + 1000
    lo[::4] = -50
    lo[1::4] = 10 ** 9
    lo[2::4] += 500                      # past the query's own position: it sees nothing
    pos_ok = torch.arange(600, dtype=torch.int32, device=dev) + 1400
    run_all(hisa.Queries(Q.q, Q.w, Q.dtype, q_pos=pos_ok, q_lo=lo), K)
    run_all(hisa.Queries(Q.q, Q.w, Q.dtype, q_pos=pos, q_lo=lo), K)
    # 3. block ids that are negative, far too large, or repeated
    g = torch.Generator(device="cpu").manual_seed(3)
    bad = torch.randint(-100, 10 ** 6, (600, wl.m), generator=g, dtype=torch.int64).to(torch.int32)
    bad[:, 0] = 3
    bad[:, 1] = 3
    run_all(Q, K, bi_in=bad.to(dev))


@pytest.mark.parametrize("k_dtype,pooled_dtype", [("bf16", "bf16"), ("fp8_e4m3", "bf16"), ("f32", "f32")])
def test_max_pool_variant(k_dtype, pooled_dtype):
    # Eq. 4 with Pool = per-dimension maximum, ragged last block, several sequences; then Stage 1 on
    # the max-pooled keys against the oracle's Stage 1 on the same pooled bits
    from oracle import hisa_oracle as O
    from paper_2603_28458_amd import hisa
    from tests.util import check_scores, oracle_args, rtol_for
    f32 = k_dtype == "f32"
    wl = W.make_workload(f"maxpool_{k_dtype}", n_seq=3, seq_len=[1000, 517, 64], T=3, H=4 if f32 else 64,
                         d=64 if f32 else 128, B=64, m=4, k=64, q_dtype="f32" if f32 else "bf16", k_dtype=k_dtype,
                         pooled_dtype=pooled_dtype, mode="decode", seed=160)
    print(f"\n[parity] {wl.name}", flush=True)
    Q, K = hisa.to_device(wl)
    pd = hisa.DTYPE_CODE[pooled_dtype]
    got = hisa.hisa_pool_blocks_max(K, wl.B, pooled_dtype=pd)
    torch.cuda.synchronize()
    bits = got.view(torch.int16).cpu().numpy().view(np.uint16) if pooled_dtype == "bf16" else got.cpu().numpy()
    want = O.pool_blocks(wl.keys, wl.k_dtype, wl.k_scale, wl.seq_len, wl.B, pooled_dtype, mode="max")
    g = O.decode(bits, pooled_dtype).reshape(-1, wl.d)
    w_ = O.decode(want, pooled_dtype).reshape(-1, wl.d)
    if k_dtype == "fp8_e4m3":
        check_scores(g, w_, rtol_for(wl), "max-pooled keys")      # scale * code rounds once more in fp32
    else:
        assert np.array_equal(bits, want), "a maximum of stored values is exact"
    bi, J = hisa.hisa_block_score_topk(Q, K, got, pd, wl.B, wl.m, want_scores=True)
    torch.cuda.synchronize()
    o_bi, o_J = O.hisa_block_score_topk(**oracle_args(wl, keys=False), pooled=bits, pooled_dtype=pooled_dtype,
                                        B=wl.B, m=wl.m, queries=np.arange(wl.T))
    check_scores(J.cpu().numpy(), o_J, rtol_for(wl), "block scores on max-pooled keys")
