"""No call writes outside what it was handed: every output tensor and every workspace sits between
two bands of sentinel bytes, each entry point runs on one prefill and one decode shape, and the
bands are read back afterwards.  The workspace is exactly hisa_workspace_bytes long, so a kernel
that used one element more than the library asked for lands in a band."""
import pytest
import torch

from paper_2603_28458_amd import hisa
from paper_2603_28458_amd import workloads as W

pytestmark = pytest.mark.gpu

PAD = 8192
FILL = 0xA5


class Guarded:
    """nbytes of device memory with PAD sentinel bytes in front and behind."""

    def __init__(self, what, nbytes, device):
        self.what, self.nbytes = what, int(nbytes)
        self.buf = torch.full((2 * PAD + self.nbytes,), FILL, dtype=torch.uint8, device=device)

    def tensor(self, dtype, shape):
        return self.buf[PAD:PAD + self.nbytes].view(dtype).view(shape)

    def check(self):
        assert bool((self.buf[:PAD] == FILL).all()), f"{self.what}: bytes in FRONT of the buffer were written"
        assert bool((self.buf[PAD + self.nbytes:] == FILL).all()), f"{self.what}: bytes BEHIND the buffer were written"


def _guard(pool, what, dtype, shape, device):
    n = 1
    for s in shape:
        n *= s
    g = Guarded(what, n * torch.empty((), dtype=dtype).element_size(), device)
    pool.append(g)
    return g.tensor(dtype, shape)


def _run_all(wl, single_launch):
    print(f"\n[guards] {wl.name}: T={wl.T} n_seq={wl.n_seq} s_max={wl.s_max} B={wl.B} m={wl.m} k={wl.k} "
          f"k_dtype={wl.k_dtype}", flush=True)
    Q, K = hisa.to_device(wl)
    dev = Q.q.device
    pd = hisa.DTYPE_CODE[wl.pooled_dtype]
    T, M, B, m, k = wl.T, wl.s_max // wl.B, wl.B, wl.m, wl.k
    G = []
    i32, f32, u8 = torch.int32, torch.float32, torch.uint8

    def ws(op):
        """Exactly the bytes the header names as the call's minimum (Stage 1: T * s_max / B floats, Stage 2
        two-kernel path: T * m * B floats; flat: what hisa_workspace_bytes recommends), or no workspace."""
        n = hisa.hisa_workspace_bytes(op, Q, K, B if op != hisa.OP_FLAT_TOPK else 1, m if op != hisa.OP_FLAT_TOPK else 0, k)
        if op == hisa.OP_BLOCK_SCORE_TOPK:
            n = T * M * 4
        elif op == hisa.OP_TOKEN_REFINE_TOPK and n:
            n = T * m * B * 4
        return _guard(G, f"workspace of op {op}", u8, (n,), dev) if n else None

    pooled = _guard(G, "pooled", torch.bfloat16, (wl.n_seq, M, wl.d), dev)
    pooled.zero_()
    hisa.hisa_pool_blocks(K, B, pooled=pooled, pooled_dtype=pd)
    hisa.hisa_pool_blocks_max(K, B, pooled=_guard(G, "pooled (max)", torch.bfloat16, (wl.n_seq, M, wl.d), dev), pooled_dtype=pd)
    prev = torch.clamp(K.seq_len - 200, min=0).to(torch.int32)
    hisa.hisa_pool_append(K, B, prev, 200, pooled, pd)

    # Stage 1: workspace path, then the score-output path
    block_idx = _guard(G, "block_idx", i32, (T, m), dev)
    hisa.hisa_block_score_topk(Q, K, pooled, pd, B, m, block_idx=block_idx, ws=ws(hisa.OP_BLOCK_SCORE_TOPK))
    hisa.hisa_block_score_topk(Q, K, pooled, pd, B, m, block_idx=_guard(G, "block_idx (scores path)", i32, (T, m), dev),
                               block_scores=_guard(G, "block_scores", f32, (T, M), dev))
    # Stage 2: the path the shapes select (fused for T >= 256), then the two-kernel path with every output
    hisa.hisa_token_refine_topk(Q, K, B, m, block_idx, k, topk_idx=_guard(G, "topk_idx", i32, (T, k), dev),
                                ws=ws(hisa.OP_TOKEN_REFINE_TOPK))
    hisa.hisa_token_refine_topk(Q, K, B, m, block_idx, k, topk_idx=_guard(G, "topk_idx (+scores)", i32, (T, k), dev),
                                topk_scores=_guard(G, "topk_scores", f32, (T, k), dev), ws=ws(hisa.OP_TOKEN_REFINE_TOPK))
    hisa.hisa_token_refine_topk(Q, K, B, m, block_idx, k, topk_idx=_guard(G, "topk_idx (cand path)", i32, (T, k), dev),
                                topk_scores=_guard(G, "topk_scores (cand path)", f32, (T, k), dev),
                                cand_scores=_guard(G, "cand_scores", f32, (T, m * B), dev))
    if T * m * B * 4 <= hisa.STATIC_SCRATCH_BYTES or T >= 256:
        hisa.hisa_token_refine_topk_static(Q, K, B, m, block_idx, k, _guard(G, "topk_idx (static)", i32, (T, k), dev),
                                           _guard(G, "topk_scores (static)", f32, (T, k), dev))
    if single_launch:
        hisa.hisa_indexer_topk(Q, K, pooled, pd, B, m, k, block_idx=_guard(G, "block_idx (single launch)", i32, (T, m), dev),
                               topk_idx=_guard(G, "topk_idx (single launch)", i32, (T, k), dev),
                               topk_scores=_guard(G, "topk_scores (single launch)", f32, (T, k), dev))
    # flat baseline, Block-Sparse expansion, IoU
    flat_idx = _guard(G, "flat topk_idx", i32, (T, k), dev)
    hisa.dsa_flat_indexer_topk(Q, K, k, topk_idx=flat_idx, topk_scores=_guard(G, "flat topk_scores", f32, (T, k), dev),
                               ws=ws(hisa.OP_FLAT_TOPK))
    hisa.hisa_block_sparse_tokens(Q, K, B, m, block_idx, tokens=_guard(G, "block-sparse tokens", i32, (T, m * B), dev))
    hisa.hisa_index_iou(flat_idx, flat_idx, iou=_guard(G, "iou", f32, (T,), dev))
    torch.cuda.synchronize()
    for g in G:
        g.check()
    return len(G)


@pytest.mark.parametrize("k_dtype", ["bf16", "fp8_e4m3"])
def test_prefill_shape_leaves_the_guard_bands_intact(k_dtype):
    # ragged: 2891 = 22 blocks of 128 + 75; T >= 256 -> fused Stage 2, resident / prefill Stage 1
    wl = W.make_workload(f"guard_prefill_{k_dtype}", seq_len=2891, T=2891, H=64, d=128, B=128, m=7, k=513,
                         q_dtype="bf16", k_dtype=k_dtype, seed=401)
    assert _run_all(wl, single_launch=True) >= 18


def test_long_prefill_chunk_leaves_the_guard_bands_intact():
    # more than 512 blocks (Stage 1 through the shared-tile kernel) and rows long enough for the
    # streaming select of the flat indexer; 300 queries at the end of the context
    wl = W.make_workload("guard_long", seq_len=70001, T=300, H=64, d=128, B=128, m=16, k=1024, q_dtype="bf16",
                         k_dtype="bf16", seed=402)
    assert _run_all(wl, single_launch=True) >= 18


@pytest.mark.parametrize("k_dtype", ["bf16", "fp8_e4m3"])
def test_decode_shape_leaves_the_guard_bands_intact(k_dtype):
    wl = W.make_workload(f"guard_decode_{k_dtype}", n_seq=7, seq_len=[9000, 8191, 4097, 777, 129, 128, 1], T=7, H=64,
                         d=128, B=128, m=9, k=600, q_dtype="bf16", k_dtype=k_dtype, mode="decode", seed=403)
    assert _run_all(wl, single_launch=True) >= 18


def test_fp32_shape_leaves_the_guard_bands_intact():
    wl = W.make_workload("guard_f32", seq_len=1000, T=1000, H=4, d=64, B=64, m=4, k=130, q_dtype="f32", k_dtype="f32",
                         seed=404)
    Q, K = hisa.to_device(wl)
    dev = Q.q.device
    G = []
    T, M, B, m, k = wl.T, wl.s_max // wl.B, wl.B, wl.m, wl.k
    pooled = _guard(G, "pooled f32", torch.float32, (1, M, wl.d), dev)
    hisa.hisa_pool_blocks(K, B, pooled=pooled, pooled_dtype=hisa.HISA_F32)
    n1 = T * M * 4
    block_idx = _guard(G, "block_idx", torch.int32, (T, m), dev)
    hisa.hisa_block_score_topk(Q, K, pooled, hisa.HISA_F32, B, m, block_idx=block_idx,
                               ws=_guard(G, "ws1", torch.uint8, (n1,), dev))
    n2 = T * m * B * 4
    hisa.hisa_token_refine_topk(Q, K, B, m, block_idx, k, topk_idx=_guard(G, "topk_idx", torch.int32, (T, k), dev),
                                ws=_guard(G, "ws2", torch.uint8, (n2,), dev))
    nf = hisa.hisa_workspace_bytes(hisa.OP_FLAT_TOPK, Q, K, 1, 0, k)
    hisa.dsa_flat_indexer_topk(Q, K, k, topk_idx=_guard(G, "flat idx", torch.int32, (T, k), dev),
                               ws=_guard(G, "wsf", torch.uint8, (nf,), dev))
    torch.cuda.synchronize()
    for g in G:
        g.check()
