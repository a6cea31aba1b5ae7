#!/usr/bin/env python3
"""Benchmark of the HISA indexer hot path on one MI355X.

One step = one pass of the whole path (block pooling, Stage 1 block filter, Stage 2 token
refinement: Algorithm 1 of the paper) over one batch of synthetic queries whose inputs are already
resident in HBM.  The default workload is the 64K-context prefill (B=128, m=64, k=2048, H=64,
d=128, bf16): the shape the headline metric "indexer queries/s at 64K context" is quoted on.
The flat DSA indexer (Eqs. 1-2) is timed at the same shape for the speedup ratio, the Stage 2
kernel is timed alone for the roofline figure, and the CPU oracle is timed on a bounded sample of
the same queries as a reported baseline.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_FP8_TFLOPS = 5000.0      # MI355X dense fp8 MFMA
PEAK_HBM_GBS = 8000.0


def algorithmic_pairs(wl):
    """(Stage 1 block scores, Stage 2 token scores, flat token scores) the method must compute:
    causal, selected, no padding (Eqs. 10-11 of the paper, counted exactly)."""
    pos = wl.positions()
    b_t = pos // wl.B
    stage1 = int((b_t + 1).sum())
    nblk = np.minimum(wl.m, b_t + 1)
    stage2 = int(((nblk - 1) * wl.B + (pos % wl.B) + 1).sum())
    flat = int((pos + 1).sum())
    return stage1, stage2, flat


def _iou(a, b):
    """Eq. 12 of the paper on two index rows (-1 = padding): a host-side diagnostic."""
    a, b = a[a >= 0], b[b >= 0]
    u = np.union1d(a, b).size
    return 1.0 if u == 0 else np.intersect1d(a, b).size / u


def time_region(fn, steps, warmup):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    return e0.elapsed_time(e1) / steps, wall


def measured_traffic(workload):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary
    (profiles/hbm_traffic_<workload>.txt: FETCH_SIZE and WRITE_SIZE scaled by a copy of known size);
    None if that workload has not been profiled."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch="):
            return float(line.split("=", 1)[1])
    return None


def cpu_baseline(wl, budget_s=20.0, seed=0):
    """The oracle as it stands, on the host cores, on a bounded uniform sample of the queries."""
    from oracle import hisa_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1])
    except Exception:
        cores = 1
    rng = np.random.default_rng(seed)
    pos = wl.positions()
    args = dict(q=wl.q, q_dtype=wl.q_dtype, w=wl.w, q_seq=wl.q_seq, q_pos=pos, keys=wl.keys,
                k_dtype=wl.k_dtype, k_scale=wl.k_scale, seq_len=wl.seq_len, B=wl.B, m=wl.m, k=wl.k,
                pooled_dtype=wl.pooled_dtype)
    t0 = time.perf_counter()
    pooled = O.pool_blocks(wl.keys, wl.k_dtype, wl.k_scale, wl.seq_len, wl.B, wl.pooled_dtype)
    t_pool = time.perf_counter() - t0
    done, spent, n = 0, 0.0, 8
    while spent < budget_s and done < wl.T:
        qs = rng.choice(wl.T, size=min(n, wl.T), replace=False)
        t0 = time.perf_counter()
        O.hisa_indexer(**args, queries=qs, pooled=pooled)
        spent += time.perf_counter() - t0
        done += qs.size
        n = min(n * 2, 256)
    return {"value": done / spent, "unit": "queries/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{done} queries drawn uniformly from the {wl.T} of the workload, Stage 1 + Stage 2 in "
                      f"float64 numpy ({spent:.1f} s); pooling all keys once took {t_pool:.2f} s extra"}


def needle_recall(wl, block_idx, topk_idx, flat_idx):
    """Synthetic-data diagnostic: a needle key is a scaled copy of one head of its target query, so
    the target query should keep the needle's block (Stage 1) and select the needle token."""
    pos = wl.positions()
    n = blk = tok = flat = 0
    for (_, p, t_star, _) in wl.needles:
        if p > pos[t_star]:
            continue
        n += 1
        blk += int((block_idx[t_star] == p // wl.B).any().item())
        tok += int((topk_idx[t_star] == p).any().item())
        flat += int((flat_idx[t_star] == p).any().item())
    return {"n": n, "block_kept_by_stage1": blk, "token_selected_by_hisa": tok, "token_selected_by_flat": flat}


def sweep(a, torch, hisa, W):
    """Kernel-latency shapes of the paper (Sec. 5.1, Fig. 2) and its (B, m) ablation shapes (App. C)."""
    shapes = []
    if a.sweep == "context":
        for L in (8192, 16384, 32768, 65536):
            shapes.append((L, 128, 64, "budget 8192"))
            shapes.append((L, 128, max(2, L // 128 // 4), "M:m = 4:1"))
    else:
        for B, m in ((64, 128), (128, 64), (256, 32), (512, 16), (1024, 8), (2048, 4)):
            shapes.append((65536, B, m, "m*B = 8192"))
        shapes.append((65536, 128, 16, "Block-Sparse shape (Stage 1 only is timed as block_sparse_ms)"))
    for i, (L, B, m, note) in enumerate(shapes):
        k = min(2048, m * B)
        wl = W.make_workload(f"sweep_{a.sweep}_{L}_{B}_{m}", seq_len=L, T=1024, H=64, d=128, B=B, m=m, k=k,
                             q_dtype=W.BF16, k_dtype=W.BF16, seed=W.BASE_SEED + 100 + i)
        Q, K = hisa.to_device(wl)
        pd = hisa.DTYPE_CODE[wl.pooled_dtype]
        dev = Q.q.device
        pooled = hisa.hisa_pool_blocks(K, B, pooled_dtype=pd)
        block_idx = torch.empty((wl.T, m), dtype=torch.int32, device=dev)
        topk_idx = torch.empty((wl.T, k), dtype=torch.int32, device=dev)
        flat_idx = torch.empty((wl.T, k), dtype=torch.int32, device=dev)
        tokens = torch.empty((wl.T, m * B), dtype=torch.int32, device=dev)
        ws1 = torch.empty(max(1, hisa.hisa_workspace_bytes(hisa.OP_BLOCK_SCORE_TOPK, Q, K, B, m, k)),
                          dtype=torch.uint8, device=dev)
        ws2 = torch.empty(max(1, hisa.hisa_workspace_bytes(hisa.OP_TOKEN_REFINE_TOPK, Q, K, B, m, k)),
                          dtype=torch.uint8, device=dev)
        wsf = torch.empty(hisa.hisa_workspace_bytes(hisa.OP_FLAT_TOPK, Q, K, 1, 0, k), dtype=torch.uint8, device=dev)

        def s1():
            hisa.hisa_block_score_topk(Q, K, pooled, pd, B, m, block_idx=block_idx, ws=ws1)

        def s2():
            hisa.hisa_token_refine_topk(Q, K, B, m, block_idx, k, topk_idx=topk_idx, ws=ws2)

        def bs():
            s1()
            hisa.hisa_block_sparse_tokens(Q, K, B, m, block_idx, tokens=tokens)

        def flat():
            hisa.dsa_flat_indexer_topk(Q, K, k, topk_idx=flat_idx, ws=wsf)

        ms1, _ = time_region(s1, a.steps, a.warmup)
        ms2, _ = time_region(s2, a.steps, a.warmup)
        msb, _ = time_region(bs, a.steps, a.warmup)
        msf, _ = time_region(flat, a.steps, a.warmup)
        iou = float(hisa.hisa_index_iou(topk_idx, flat_idx).mean().item())
        print(json.dumps({"sweep": a.sweep, "L": L, "T": wl.T, "B": B, "m": m, "k": k, "note": note,
                          "stage1_ms": ms1, "stage2_ms": ms2, "hisa_ms": ms1 + ms2, "block_sparse_ms": msb,
                          "flat_ms": msf, "flat_over_hisa": msf / (ms1 + ms2), "iou_hisa_vs_flat_mean": iou,
                          "steps": a.steps, "warmup": a.warmup}), flush=True)
        del Q, K, pooled, ws1, ws2, wsf, tokens
        torch.cuda.empty_cache()


def variant_line(name, steps, warmup, flat_steps, torch, hisa, W):
    """The same step on another variant of the headline configuration (BASELINE's 64K prefill has
    two: bf16 keys, and fp8 e4m3 keys with per-token scales), timed the same way, in short form."""
    wl = W.config(name)
    Q, K = hisa.to_device(wl)
    pd = hisa.DTYPE_CODE[wl.pooled_dtype]
    T, dev = wl.T, Q.q.device
    pooled = torch.zeros((wl.n_seq, wl.s_max // wl.B, wl.d), dtype=torch.bfloat16, device=dev)
    block_idx = torch.empty((T, wl.m), dtype=torch.int32, device=dev)
    topk_idx = torch.empty((T, wl.k), dtype=torch.int32, device=dev)
    ws1 = torch.empty(max(1, hisa.hisa_workspace_bytes(hisa.OP_BLOCK_SCORE_TOPK, Q, K, wl.B, wl.m, wl.k)),
                      dtype=torch.uint8, device=dev)
    ws2 = torch.empty(max(1, hisa.hisa_workspace_bytes(hisa.OP_TOKEN_REFINE_TOPK, Q, K, wl.B, wl.m, wl.k)),
                      dtype=torch.uint8, device=dev)
    ws_f = torch.empty(hisa.hisa_workspace_bytes(hisa.OP_FLAT_TOPK, Q, K, 1, 0, wl.k), dtype=torch.uint8, device=dev)

    def stage2():
        hisa.hisa_token_refine_topk(Q, K, wl.B, wl.m, block_idx, wl.k, topk_idx=topk_idx, ws=ws2)

    def step():
        hisa.hisa_pool_blocks(K, wl.B, pooled=pooled, pooled_dtype=pd)
        hisa.hisa_block_score_topk(Q, K, pooled, pd, wl.B, wl.m, block_idx=block_idx, ws=ws1)
        stage2()

    ms_step, _ = time_region(step, steps, warmup)
    ms_s2, _ = time_region(stage2, steps, 1)
    ms_flat, _ = time_region(lambda: hisa.dsa_flat_indexer_topk(Q, K, wl.k, topk_idx=topk_idx, ws=ws_f), flat_steps, 1)
    _, p2, _ = algorithmic_pairs(wl)
    fp8 = wl.k_dtype == "fp8_e4m3"
    peak = PEAK_FP8_TFLOPS if fp8 else PEAK_BF16_TFLOPS
    achieved = p2 * 2.0 * wl.H * wl.d / (ms_s2 * 1e-3) / 1e12
    return {"workload": name, "dtype": "fp8" if fp8 else "bf16", "value": T / (ms_step * 1e-3), "unit": "queries/s",
            "ms_per_step": ms_step, "stage2_ms": ms_s2,
            "roofline": {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                         "frac": achieved / peak, "traffic": measured_traffic(name)},
            "flat_ms": ms_flat, "speedup_vs_flat": ms_flat / ms_step}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="prefill64k_bf16")
    ap.add_argument("--flat-steps", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-flat", action="store_true")
    ap.add_argument("--sweep", choices=["context", "blocks"], default=None,
                    help="instead of the headline line, time the shapes of the paper's kernel-latency "
                         "figure (Sec. 5.1: 1024 queries at the end of 8K-64K contexts, m = 64 and M:m = 4:1) "
                         "or of its block-size ablation (App. C: (B, m) at m*B = 8192, and Block-Sparse "
                         "(128, 16)); one JSON line per shape")
    ap.add_argument("--profile-flat", action="store_true",
                    help="with --profile-mode: run the flat DSA indexer instead of the HISA step")
    ap.add_argument("--profile-mode", action="store_true",
                    help="for rocprofv3: run the step a few times plus a 256 MiB device copy (counter "
                         "calibration), print nothing else and exit")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the indexer shards by query with no exchange; "
              "nothing is exchanged between GPUs); --gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_28458_amd import hisa
    from paper_2603_28458_amd import workloads as W

    hisa.lib()                                  # fail loudly if the HIP library is not built
    torch.cuda.set_device(0)
    if a.sweep:
        sweep(a, torch, hisa, W)
        return
    wl = W.config(a.workload)
    Q, K = hisa.to_device(wl)
    pd = hisa.DTYPE_CODE[wl.pooled_dtype]
    T, M = wl.T, wl.s_max // wl.B
    dev = Q.q.device
    decode = wl.q_seq is not None

    pooled = torch.zeros((wl.n_seq, M, wl.d), dtype=torch.bfloat16 if pd == hisa.HISA_BF16 else torch.float32,
                         device=dev)
    block_idx = torch.empty((T, wl.m), dtype=torch.int32, device=dev)
    topk_idx = torch.empty((T, wl.k), dtype=torch.int32, device=dev)
    ws1 = torch.empty(max(1, hisa.hisa_workspace_bytes(hisa.OP_BLOCK_SCORE_TOPK, Q, K, wl.B, wl.m, wl.k)),
                      dtype=torch.uint8, device=dev)
    ws2 = torch.empty(max(1, hisa.hisa_workspace_bytes(hisa.OP_TOKEN_REFINE_TOPK, Q, K, wl.B, wl.m, wl.k)),
                      dtype=torch.uint8, device=dev)

    def pool():
        hisa.hisa_pool_blocks(K, wl.B, pooled=pooled, pooled_dtype=pd)

    def stage1():
        hisa.hisa_block_score_topk(Q, K, pooled, pd, wl.B, wl.m, block_idx=block_idx, ws=ws1)

    def stage2():
        hisa.hisa_token_refine_topk(Q, K, wl.B, wl.m, block_idx, wl.k, topk_idx=topk_idx, ws=ws2)

    def step():
        if not decode:          # decode: the pooled cache is precomputed (maintained with the KV cache)
            pool()
        stage1()
        stage2()

    pool()
    if a.profile_mode:
        if a.profile_flat:
            ws_f = torch.empty(hisa.hisa_workspace_bytes(hisa.OP_FLAT_TOPK, Q, K, 1, 0, wl.k), dtype=torch.uint8,
                               device=dev)
            for _ in range(max(1, a.steps)):
                hisa.dsa_flat_indexer_topk(Q, K, wl.k, topk_idx=topk_idx, ws=ws_f)
        else:
            for _ in range(max(1, a.steps)):
                step()
        src = torch.ones(64 << 20, dtype=torch.float32, device=dev)     # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"profile_mode": True, "workload": a.workload, "steps": a.steps,
                          "calibration_copy_bytes": src.numel() * 4}))
        return
    ms_step, wall_step = time_region(step, a.steps, a.warmup)
    ms_pool, _ = time_region(pool, a.steps, 1)
    ms_s1, _ = time_region(stage1, a.steps, 1)
    ms_s2, _ = time_region(stage2, a.steps, 1)     # Stage 2 alone: the dominant kernel

    p1, p2, pf = algorithmic_pairs(wl)
    flop_pair = 2.0 * wl.H * wl.d
    fused = wl.q_dtype == "bf16" and T >= 256 and wl.m * wl.B <= 16384
    if decode:
        kb = {"bf16": 2, "fp8_e4m3": 1, "f32": 4}[wl.k_dtype] * wl.d + (4 if wl.k_dtype == "fp8_e4m3" else 0)
        bytes_s2 = p2 * kb + T * (wl.H * wl.d * 2 + wl.H * 4 + wl.m * 4 + wl.k * 4) + 2 * p2 * 4
        roof = {"bound": "hbm", "achieved": bytes_s2 / (ms_s2 * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "kernel": "hisa_token_refine_topk (k_score_ranges + k_select)", "traffic": None}
    else:
        # fp8 keys are scored on the fp8 MFMA, twice per algorithmic flop (the bf16 query enters as
        # the sum of two e4m3 numbers): `achieved` stays the algorithmic rate, `peak` is that pipe's
        fp8 = wl.k_dtype == "fp8_e4m3" and wl.q_dtype == "bf16"
        roof = {"bound": "mfma", "achieved": p2 * flop_pair / (ms_s2 * 1e-3) / 1e12,
                "peak": PEAK_FP8_TFLOPS if fp8 else PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "kernel": "k_refine_fused" if fused else "k_score_ranges + k_select",
                "mfma": "fp8 e4m3 x e4m3, 2 executed flop per algorithmic flop" if fp8 else "bf16",
                "traffic": None}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["ms_per_launch"] = ms_s2
    kbytes = {"bf16": 2, "fp8_e4m3": 1, "f32": 4}[wl.k_dtype] * wl.d + (4 if wl.k_dtype == "fp8_e4m3" else 0)
    qbytes = wl.H * wl.d * (2 if wl.q_dtype == "bf16" else 4) + wl.H * 4
    # key tiles that reach the compute units (from L2 / Infinity Cache / HBM) for the pairs scored
    roof["tile_delivery_GBs"] = p2 * kbytes / (ms_s2 * 1e-3) / 1e9
    # bytes the step has to move through HBM at least: keys (those of kept blocks, at most all) and pooled keys once, the queries once
    # per stage, the block ids written and read, the top-k indices written
    hbm_bytes = (min(int(wl.seq_len.sum()), p2) * kbytes + int(wl.seq_len.sum()) // wl.B * wl.d * 2
                 + 2 * T * qbytes + 2 * T * wl.m * 4 + T * wl.k * 4)
    roof["traffic"] = measured_traffic(a.workload)
    # what this chip delivers to a kernel that does nothing else: a 1 GiB streaming copy and a loop
    # of MFMAs only (the library's probe kernels), for the fraction of the ATTAINABLE peak
    src = torch.empty(1 << 29, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    ms_copy, _ = time_region(lambda: hisa.hisa_probe_copy(src, dst), 5, 1)
    probe_out = torch.empty(512 * 256, dtype=torch.float32, device=dev)
    flop_box = []
    ms_mfma, _ = time_region(lambda: flop_box.append(hisa.hisa_probe_mfma(probe_out, 20000)), 3, 1)
    ms_mfma8, _ = time_region(lambda: flop_box.append(hisa.hisa_probe_mfma_fp8(probe_out, 10000)), 3, 1)
    attainable = {"hbm_copy_GBs": 2.0 * src.numel() / (ms_copy * 1e-3) / 1e9,
                  "mfma_bf16_TFLOPs": flop_box[0] / (ms_mfma * 1e-3) / 1e12,
                  "mfma_fp8_TFLOPs": flop_box[-1] / (ms_mfma8 * 1e-3) / 1e12}
    del src, dst
    if roof["bound"] == "hbm":
        roof["frac_of_attainable"] = roof["achieved"] / attainable["hbm_copy_GBs"]
    else:
        roof["frac_of_attainable"] = roof["achieved"] / (
            attainable["mfma_fp8_TFLOPs"] if roof["peak"] == PEAK_FP8_TFLOPS else attainable["mfma_bf16_TFLOPs"])

    out = {
        "metric": "indexer queries/s at 64K context (HISA: pool + Stage 1 + Stage 2)" if "64k" in a.workload
                  else f"indexer queries/s ({a.workload})",
        "value": T / (ms_step * 1e-3), "unit": "queries/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("fp8" if wl.k_dtype == "fp8_e4m3" else "bf16") if wl.q_dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": a.workload, "T": T, "L": int(wl.seq_len.max()), "n_seq": wl.n_seq, "H": wl.H,
                   "d": wl.d, "B": wl.B, "m": wl.m, "k": wl.k, "q_dtype": wl.q_dtype, "k_dtype": wl.k_dtype},
        "stage_ms": {"pool": ms_pool, "stage1": ms_s1, "stage2": ms_s2, "wall_ms_per_step": wall_step},
        "algorithmic": {"stage1_pairs": p1, "stage2_pairs": p2, "flat_pairs": pf, "flop_per_pair": flop_pair,
                        "hisa_tflop": (p1 + p2) * flop_pair / 1e12, "flat_tflop": pf * flop_pair / 1e12},
        "roofline": roof,
        "attainable": attainable,
        "hbm_step": {"algorithmic_bytes": hbm_bytes, "GBs": hbm_bytes / (ms_step * 1e-3) / 1e9,
                     "frac_of_peak": hbm_bytes / (ms_step * 1e-3) / 1e9 / PEAK_HBM_GBS},
    }

    if not a.no_flat:
        ws_f = torch.empty(hisa.hisa_workspace_bytes(hisa.OP_FLAT_TOPK, Q, K, 1, 0, wl.k), dtype=torch.uint8, device=dev)
        flat_idx = torch.empty((T, wl.k), dtype=torch.int32, device=dev)

        def flat():
            hisa.dsa_flat_indexer_topk(Q, K, wl.k, topk_idx=flat_idx, ws=ws_f)

        ms_flat, _ = time_region(flat, a.flat_steps, 1)
        out["flat"] = {"ms": ms_flat, "queries_per_s": T / (ms_flat * 1e-3),
                       "tflops": pf * flop_pair / (ms_flat * 1e-3) / 1e12,
                       "frac_of_mfma_peak": pf * flop_pair / (ms_flat * 1e-3) / 1e12 / roof.get("peak", PEAK_BF16_TFLOPS)
                       if roof["bound"] == "mfma" else
                       pf * flop_pair / (ms_flat * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
        out["speedup_vs_flat"] = ms_flat / ms_step
        # Eq. 12 over every query, computed by the library's own diagnostic kernel
        out["iou_hisa_vs_flat_mean"] = float(hisa.hisa_index_iou(topk_idx, flat_idx).mean().item())
        if wl.needles:
            out["needles"] = needle_recall(wl, block_idx, topk_idx, flat_idx)
        del ws_f

    if a.workload == "prefill64k_bf16" and not a.no_flat:
        del Q, K, pooled, block_idx, topk_idx, ws1, ws2
        torch.cuda.empty_cache()
        out["fp8_keys_variant"] = variant_line("prefill64k_fp8", a.steps, a.warmup, a.flat_steps, torch, hisa, W)
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
