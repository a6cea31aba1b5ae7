"""hisa_token_refine_topk_static (the Stage 2 call that allocates nothing: its candidate scores go
through a static device array inside the library) against hisa_token_refine_topk with a caller
workspace, through the C ABI: two calls in a row on one GPU, the second on a smaller input, so that
whatever the first call left in the shared array must not leak into the second."""
import pytest
import torch

from paper_2603_28458_amd import hisa
from paper_2603_28458_amd import workloads as W
from tests.parity import _check_token_sets, _np, sample_queries
from tests.util import oracle_args, rtol_for
from oracle import hisa_oracle as O

pytestmark = pytest.mark.gpu


def _both(wl):
    """Stage 1 once, then Stage 2 through the workspace call and through the static call."""
    Q, K = hisa.to_device(wl)
    pd = hisa.DTYPE_CODE[wl.pooled_dtype]
    pooled = hisa.hisa_pool_blocks(K, wl.B, pooled_dtype=pd)
    block_idx, _ = hisa.hisa_block_score_topk(Q, K, pooled, pd, wl.B, wl.m)
    ref_idx, ref_sc, _ = hisa.hisa_token_refine_topk(Q, K, wl.B, wl.m, block_idx, wl.k, want_topk_scores=True)
    # outputs exist before the call under test: it must not need to allocate anything
    got_idx = torch.full((wl.T, wl.k), -7, dtype=torch.int32, device=Q.q.device)
    got_sc = torch.full((wl.T, wl.k), 123.0, dtype=torch.float32, device=Q.q.device)
    torch.cuda.synchronize()
    hisa.hisa_token_refine_topk_static(Q, K, wl.B, wl.m, block_idx, wl.k, got_idx, got_sc)
    torch.cuda.synchronize()
    return Q, K, block_idx, ref_idx, ref_sc, got_idx, got_sc


def _check(wl, tag):
    print(f"\n[no-alloc] {tag}: T={wl.T} n_seq={wl.n_seq} B={wl.B} m={wl.m} k={wl.k} k_dtype={wl.k_dtype} "
          f"seed={wl.seed}", flush=True)
    Q, K, block_idx, ref_idx, ref_sc, got_idx, got_sc = _both(wl)
    # same kernels, same fp32 scores, same tie rule: bit for bit
    assert torch.equal(got_idx, ref_idx), f"{tag}: index sets differ from hisa_token_refine_topk"
    assert torch.equal(got_sc.view(torch.int32), ref_sc.view(torch.int32)), f"{tag}: scores differ"
    # and against the oracle on the GPU's own block ids (Eqs. 8-9)
    qs = sample_queries(wl, 16)
    bi = _np(block_idx)
    o_ti, _, o_cand = O.hisa_token_refine_topk(**oracle_args(wl), B=wl.B, m=wl.m, block_idx=bi[qs], k=wl.k,
                                               queries=qs)
    _check_token_sets(wl, qs, bi, _np(got_idx), _np(got_sc), o_ti, o_cand, rtol_for(wl), tag)
    return got_idx


def test_static_scratch_two_calls_second_smaller():
    # two-kernel path (T < 256): the candidate scores really go through the static array
    big = W.make_workload("na_big", n_seq=6, seq_len=[6000, 5100, 4097, 3000, 129, 1], T=6, H=64, d=128, B=128,
                          m=12, k=1024, q_dtype="bf16", k_dtype="bf16", mode="decode", seed=310)
    small = W.make_workload("na_small", n_seq=3, seq_len=[900, 2050, 640], T=3, H=64, d=128, B=128, m=4, k=256,
                            q_dtype="bf16", k_dtype="fp8_e4m3", mode="decode", seed=311)
    _check(big, "first call")
    _check(small, "second call, smaller")
    _check(big, "third call, large again")


def test_static_scratch_fused_shape_and_limit():
    # T >= 256 with m*B <= 16384 takes the fused kernel (no scratch at all): same results
    wl = W.make_workload("na_fused", seq_len=1500, T=300, H=64, d=128, B=128, m=5, k=300, q_dtype="bf16",
                         k_dtype="bf16", seed=312)
    _check(wl, "fused shape")
    # beyond the array: 200 queries x 65536 candidates x 4 B = 50 MiB > 16 MiB -> refused, nothing launched
    Q, K = hisa.to_device(W.make_workload("na_lim", n_seq=1, seq_len=70000, T=200, H=64, d=128, B=128, m=512, k=512,
                                          q_dtype="bf16", k_dtype="bf16", seed=313))
    bi = torch.zeros((200, 512), dtype=torch.int32, device=Q.q.device)
    out = torch.full((200, 512), -7, dtype=torch.int32, device=Q.q.device)
    with pytest.raises(hisa.HisaError) as e:
        hisa.hisa_token_refine_topk_static(Q, K, 128, 512, bi, 512, out)
    assert e.value.status == 5
    torch.cuda.synchronize()
    assert bool((out == -7).all()), "a refused call must leave the output untouched"
