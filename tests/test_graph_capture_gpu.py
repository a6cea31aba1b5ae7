"""The library only enqueues kernels on the caller's stream (no allocation, no memset, no
synchronisation), so a serving loop can record a decode step into a HIP graph.  The test records
pooling + Stage 1 + Stage 2 + the single-launch indexer + the flat indexer of a small decode batch,
replays the graph several times with eager work and synchronisations of the program in between,
and compares every replay with the eager result bit for bit (the kernels are deterministic)."""
import pytest
import torch

from paper_2603_28458_amd import hisa, workloads as W

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("k_dtype", ["bf16", "fp8_e4m3"])
def test_graph_replays_match_eager(k_dtype):
    wl = W.make_workload(f"graph_{k_dtype}", n_seq=6, seq_len=[9000, 7777, 4100, 129, 128, 1], T=6, H=64,
                         d=128, B=128, m=8, k=512, q_dtype="bf16", k_dtype=k_dtype, mode="decode", seed=131)
    Q, K = hisa.to_device(wl)
    dev = Q.q.device
    pd = hisa.HISA_BF16
    M = K.s_max // wl.B
    pooled = torch.zeros((K.n_seq, M, K.d), dtype=torch.bfloat16, device=dev)
    bi = torch.empty((wl.T, wl.m), dtype=torch.int32, device=dev)
    ti = torch.empty((wl.T, wl.k), dtype=torch.int32, device=dev)
    si = torch.empty((wl.T, wl.k), dtype=torch.int32, device=dev)
    fi = torch.empty((wl.T, wl.k), dtype=torch.int32, device=dev)
    outs = (pooled, bi, ti, si, fi)

    def ws(op, m, k):
        return torch.empty(max(1, hisa.hisa_workspace_bytes(op, Q, K, wl.B, m, k)), dtype=torch.uint8, device=dev)

    ws1 = ws(hisa.OP_BLOCK_SCORE_TOPK, wl.m, 0)
    ws2 = ws(hisa.OP_TOKEN_REFINE_TOPK, wl.m, wl.k)
    wsf = ws(hisa.OP_FLAT_TOPK, 0, wl.k)

    def step():
        hisa.hisa_pool_blocks(K, wl.B, pooled=pooled, pooled_dtype=pd)
        hisa.hisa_block_score_topk(Q, K, pooled, pd, wl.B, wl.m, block_idx=bi, ws=ws1)
        hisa.hisa_token_refine_topk(Q, K, wl.B, wl.m, bi, wl.k, topk_idx=ti, ws=ws2)
        hisa.hisa_indexer_topk(Q, K, pooled, pd, wl.B, wl.m, wl.k, topk_idx=si)
        hisa.dsa_flat_indexer_topk(Q, K, wl.k, topk_idx=fi, ws=wsf)

    step()
    torch.cuda.synchronize()
    want = [o.clone() for o in outs]

    side = torch.cuda.Stream()                       # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                       # warm-up on the side stream, as capture requires
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()

    for replay in range(4):
        for o in outs:
            o.fill_(0 if o.dtype == torch.bfloat16 else -7)      # fill kernels, no memset nodes
        eager = torch.randn(1 << 18, device=dev).square().sum().item()   # the program's own eager work
        assert eager > 0
        graph.replay()
        torch.cuda.synchronize()
        for name, o, w in zip(("pooled", "block_idx", "topk_idx", "single_launch_idx", "flat_idx"), outs, want):
            assert torch.equal(o, w), f"replay {replay}: {name} differs from the eager result"
