#!/usr/bin/env python3
"""Benchmark of the HISA indexer hot path on one MI355X.

One step = one pass of the whole path (block pooling, Stage 1 block filter, Stage 2 token
refinement: Algorithm 1 of the paper) over one batch of synthetic queries whose inputs are already
resident in HBM.  The default workload is the 64K-context prefill (B=128, m=64, k=2048, H=64,
d=128, bf16): the shape the headline metric "indexer queries/s at 64K context" is quoted on.
The flat DSA indexer (Eqs. 1-2) is timed at the same shape for the speedup ratio, the Stage 2
kernel is timed alone for the roofline figure, and the CPU oracle is timed on a bounded, stratified
sample of the same queries as a reported baseline; the oracle's index sets for those queries are
compared with the GPU's (`cpu_baseline.mismatches`; the run exits non-zero if there is one).
The same line carries, in short form, the configuration's fp8-keys variant (`fp8_keys_variant`) and
the other four configurations of the benchmark definition (`all_configs`: tiny fp32 prefill, 16K
prefill, decode batch, 16K-query chunk at 1M context), each with its own roofline figure.

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


def measured_traffic(workload, lib_version):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary
    (profiles/hbm_traffic_<workload>.txt: FETCH_SIZE and WRITE_SIZE scaled by a copy of known size).
    The counters come from a separate profiling run, not from this one, so the figure is returned
    with the file it came from, and only if that file was taken on this version of the kernels
    (its `library_version=` line); otherwise (None, reason)."""
    rel = f"profiles/hbm_traffic_{workload}.txt"
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, f"no counter summary for this workload ({rel})"
    val, ver, kern = None, None, None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch="):
            val = float(line.split("=", 1)[1])
        elif line.startswith("library_version="):
            ver = line.split("=", 1)[1].strip()
        elif line.startswith("kernel="):
            kern = line.split("=", 1)[1].strip()
    if val is None or ver != lib_version:
        return None, f"{rel} was taken on library version {ver}, this is {lib_version}: not reported"
    return val, f"{rel} (rocprofv3 FETCH_SIZE + WRITE_SIZE of {kern}, library version {ver}; a separate run)"


def stratified_sample(wl, n, seed=0):
    """Query sample for the oracle: uniform over the queries, plus the regime boundaries of Section 4.1
    (pos + 1 in {k, k+1, mB, mB+1}), block edges, the first and last query and the needle targets."""
    rng = np.random.default_rng(seed)
    pos = wl.positions()
    pick = set(rng.choice(wl.T, size=min(n, wl.T), replace=False).tolist())
    pick |= {0, wl.T - 1}
    for p in (wl.k - 1, wl.k, wl.m * wl.B - 1, wl.m * wl.B, wl.B - 1, wl.B, 2 * wl.B - 1):
        hit = np.nonzero(pos == p)[0]
        if hit.size:
            pick.add(int(hit[0]))
    for (_, _, t_star, _) in wl.needles:
        pick.add(int(t_star))
    return np.array(sorted(pick), dtype=np.int64)


def _blas_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"] or [1]))
    except Exception:
        return 1


def _same_set_or_threshold_swaps(got, want, cand_ids, cand_scores, rtol):
    """The benchmark's index rule on one row: 'exact', 'swap' (the sets differ only by ids whose oracle
    score lies within rtol * |threshold| of the oracle's threshold) or 'mismatch'."""
    g, w = got[got >= 0], want[want >= 0]
    if g.size != w.size or np.any(np.diff(g) <= 0):
        return "mismatch"
    diff = np.setxor1d(g, w)
    if diff.size == 0:
        return "exact"
    order = np.argsort(cand_ids)
    sid, ssc = cand_ids[order], cand_scores[order]
    at = np.searchsorted(sid, diff)
    if np.any(at >= sid.size) or np.any(sid[np.minimum(at, sid.size - 1)] != diff):
        return "mismatch"                                   # an id that is not a candidate at all
    tau = ssc[np.searchsorted(sid, w)].min()
    tol = rtol * max(abs(tau), 1e-3 * np.abs(cand_scores).max())
    return "swap" if np.abs(ssc[at] - tau).max() <= tol else "mismatch"


def cpu_baseline(wl, gpu_block_idx, gpu_topk_idx, gpu_flat_idx, budget_s=14.0, single_s=5.0, flat_s=5.0):
    """The oracle as it stands, timed on the host cores over a stratified sample of the workload's
    queries (all BLAS threads, then one thread; HISA, then the flat indexer), and its index sets
    compared with what the GPU selected for the same queries."""
    from oracle import hisa_oracle as O
    try:
        from threadpoolctl import threadpool_limits
    except Exception:
        threadpool_limits = None
    rtol = 1e-5 if wl.q_dtype == "f32" else 2e-2
    pos = wl.positions()
    args = dict(q=wl.q, q_dtype=wl.q_dtype, w=wl.w, q_seq=wl.q_seq, q_pos=pos, keys=wl.keys,
                k_dtype=wl.k_dtype, k_scale=wl.k_scale)
    t0 = time.perf_counter()
    pooled = O.pool_blocks(wl.keys, wl.k_dtype, wl.k_scale, wl.seq_len, wl.B, wl.pooled_dtype)
    t_pool = time.perf_counter() - t0
    order = stratified_sample(wl, 8192)
    np.random.default_rng(1).shuffle(order)                 # any prefix of it is spread over the positions

    checked = dict(checked_queries=0, block_sets_equal=0, block_set_swaps=0, token_sets_exact=0,
                   token_set_swaps=0, mismatches=0)

    def compare(qs, res):
        for i, t in enumerate(qs):
            gb, ob = gpu_block_idx[t], res["block_idx"][i]
            checked["checked_queries"] += 1
            if np.array_equal(gb, ob):
                checked["block_sets_equal"] += 1
                o_ti, cand = res["topk_idx"][i], res["cand_scores"][i]
            else:
                b_t = int(pos[t]) // wl.B
                verdict = _same_set_or_threshold_swaps(gb, ob, np.arange(b_t + 1), res["J"][i, :b_t + 1], rtol)
                if verdict != "swap":
                    checked["mismatches"] += 1
                    continue
                checked["block_set_swaps"] += 1
                o_ti, _, cand = O.hisa_token_refine_topk(**args, B=wl.B, m=wl.m, block_idx=gb[None], k=wl.k,
                                                         queries=np.array([t]))
                o_ti, cand = o_ti[0], cand[0]
            C = gb[gb >= 0].astype(np.int64)
            toks = O.candidate_tokens(C, int(pos[t]), wl.B)
            slots = np.searchsorted(C, toks // wl.B) * wl.B + toks % wl.B
            verdict = _same_set_or_threshold_swaps(gpu_topk_idx[t], o_ti, toks, cand[slots], rtol)
            key = {"exact": "token_sets_exact", "swap": "token_set_swaps", "mismatch": "mismatches"}[verdict]
            checked[key] += 1

    def timed(budget, start, compare_rows):
        done, spent, n, at = 0, 0.0, 8, start
        while spent < budget and at < order.size:
            qs = order[at:at + n]
            t0 = time.perf_counter()
            res = O.hisa_indexer(**args, seq_len=wl.seq_len, B=wl.B, m=wl.m, k=wl.k, pooled_dtype=wl.pooled_dtype,
                                 queries=qs, pooled=pooled)
            spent += time.perf_counter() - t0
            if compare_rows:
                compare(qs, res)
            done += qs.size
            at += qs.size
            n = min(n * 2, 256)
        return done, spent, at

    done, spent, at = timed(budget_s, 0, True)
    out = {"value": done / spent, "unit": "queries/s", "cores": len(os.sched_getaffinity(0)),
           "blas_threads": _blas_threads(), "kind": "oracle",
           "sample": f"{done} of the workload's {wl.T} queries, stratified (uniform over positions + the regime "
                     f"boundaries of Section 4.1 + block edges + needle targets), Stage 1 + Stage 2 in float64 numpy "
                     f"({spent:.1f} s); pooling all keys once took {t_pool:.2f} s extra"}
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            # (a workload with few queries, the decode batch, has none left: the same ones again, unchecked)
            d1, s1, at = timed(single_s, at, True) if at < order.size else timed(single_s, 0, False)
        out["single_thread"] = {"value": d1 / s1, "unit": "queries/s",
                                "sample": f"{d1} {'further' if at > d1 else 'of the same'} queries ({s1:.1f} s)"}
    # the flat indexer (Eqs. 1-2) on a smaller sample: one query costs its whole causal prefix
    fdone, fspent, fexact, fswap, fbad = 0, 0.0, 0, 0, 0
    forder = stratified_sample(wl, 2048, seed=2)
    np.random.default_rng(3).shuffle(forder)
    while fspent < flat_s and fdone < forder.size:
        qs = forder[fdone:fdone + 8]
        t0 = time.perf_counter()
        f_idx, _, rows = O.dsa_flat_indexer_topk(**args, k=wl.k, queries=qs, return_scores=True)
        fspent += time.perf_counter() - t0
        fdone += qs.size
        if gpu_flat_idx is not None:
            for i, t in enumerate(qs):
                v = _same_set_or_threshold_swaps(gpu_flat_idx[t], f_idx[i], np.arange(rows[i].size), rows[i], rtol)
                fexact, fswap, fbad = fexact + (v == "exact"), fswap + (v == "swap"), fbad + (v == "mismatch")
    out["flat"] = {"value": fdone / fspent, "unit": "queries/s", "sample": f"{fdone} queries, stratified ({fspent:.1f} s)"}
    if gpu_flat_idx is not None:
        out["flat"].update(checked_queries=fdone, sets_exact=int(fexact), set_swaps=int(fswap), mismatches=int(fbad))
        checked["mismatches"] += int(fbad)
    out.update(checked)
    out["check"] = ("GPU block_idx / topk_idx of the sampled queries against the oracle's: equal sets, or sets that differ "
                    "only by ids within the benchmark's tolerance of the oracle's threshold (swaps); anything else is a mismatch")
    return out


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


PEAK_FP32_ALU_TFLOPS = 157.3  # MI355X fp32 vector ALU


def bench_config(name, steps, warmup, flat_steps, torch, hisa, W, with_flat=True):
    """One configuration: the HISA step (pool + Stage 1 + Stage 2; decode: Stage 1 + Stage 2 on the cached
    pooled keys), its stages one by one, the flat DSA indexer at the same shape, and the roofline figure
    of its dominant kernel.  Returns (result dict, context of device tensors for diagnostics)."""
    wl = W.config(name)
    Q, K = hisa.to_device(wl)
    pd = hisa.DTYPE_CODE[wl.pooled_dtype]
    T, M, dev = wl.T, wl.s_max // wl.B, Q.q.device
    decode = wl.q_seq is not None
    pooled = torch.zeros((wl.n_seq, M, wl.d), dtype=torch.bfloat16 if pd == hisa.HISA_BF16 else torch.float32, device=dev)
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
    ms_step, wall_step = time_region(step, steps, warmup)
    ms_pool, _ = time_region(pool, steps, 1)
    ms_s1, _ = time_region(stage1, steps, 1)
    ms_s2, _ = time_region(stage2, steps, 1)     # Stage 2 alone: the dominant kernel

    p1, p2, pf = algorithmic_pairs(wl)
    flop_pair = 2.0 * wl.H * wl.d
    kbytes = {"bf16": 2, "fp8_e4m3": 1, "f32": 4}[wl.k_dtype] * wl.d + (4 if wl.k_dtype == "fp8_e4m3" else 0)
    qbytes = wl.H * wl.d * (2 if wl.q_dtype == "bf16" else 4) + wl.H * 4
    n_keys = int(wl.seq_len.sum())
    # bytes the step has to move through HBM at least: the keys of kept blocks (at most all keys) and the
    # pooled keys once, the queries once per stage, the block ids written and read, the top-k indices written
    hbm_bytes = (min(n_keys, p2) * kbytes + n_keys // wl.B * wl.d * 2 + 2 * T * qbytes + 2 * T * wl.m * 4 + T * wl.k * 4)
    fused = wl.q_dtype == "bf16" and T >= 256 and wl.m * wl.B <= 16384
    fp8 = wl.k_dtype == "fp8_e4m3" and wl.q_dtype == "bf16"
    if wl.q_dtype == "f32":
        # the small fp32 configuration runs on the plain vector ALU; at this size it is bound by launch latency
        roof = {"bound": "alu", "achieved": p2 * flop_pair / (ms_s2 * 1e-3) / 1e12, "peak": PEAK_FP32_ALU_TFLOPS,
                "unit": "TFLOP/s", "kernel": "k_score_ranges_f32 + k_select",
                "note": "launch-latency bound at this size: three launches of a few microseconds each"}
    elif decode:
        # every candidate key is read once: the whole step (both stages, three launches) against the HBM peak
        roof = {"bound": "hbm", "achieved": hbm_bytes / (ms_step * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "kernel": "whole step: k_stage1_query (Stage 1), k_score_ranges + k_select (Stage 2)",
                "stage2_scoring_and_select_GBs": (p2 * kbytes + T * (qbytes + wl.m * 4 + wl.k * 4) + 2 * p2 * 4)
                / (ms_s2 * 1e-3) / 1e9}
    else:
        # fp8 keys are scored on the fp8 MFMA, twice per algorithmic flop (the bf16 query enters as
        # the sum of two e4m3 numbers): `achieved` stays the algorithmic rate, `peak` is that pipe's
        roof = {"bound": "mfma", "achieved": p2 * flop_pair / (ms_s2 * 1e-3) / 1e12,
                "peak": PEAK_FP8_TFLOPS if fp8 else PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "kernel": "k_refine_fused" if fused else "k_score_ranges + k_select",
                "mfma": "fp8 e4m3 x e4m3, 2 executed flop per algorithmic flop" if fp8 else "bf16"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    roof["ms_per_launch"] = ms_step if decode else ms_s2
    roof["traffic"], roof["traffic_source"] = measured_traffic(name, hisa.version())
    # key tiles that reach the compute units (from L2 / Infinity Cache / HBM) for the pairs scored
    roof["tile_delivery_GBs"] = p2 * kbytes / (ms_s2 * 1e-3) / 1e9

    out = {"workload": name,
           "dtype": ("fp8" if wl.k_dtype == "fp8_e4m3" else "bf16") if wl.q_dtype == "bf16" else "f32",
           "value": T / (ms_step * 1e-3), "unit": "queries/s", "ms_per_step": ms_step,
           "config": {"workload": name, "T": T, "L": int(wl.seq_len.max()), "n_seq": wl.n_seq, "H": wl.H,
                      "d": wl.d, "B": wl.B, "m": wl.m, "k": wl.k, "q_dtype": wl.q_dtype, "k_dtype": wl.k_dtype},
           "stage_ms": {"pool": ms_pool, "stage1": ms_s1, "stage2": ms_s2, "wall_ms_per_step": wall_step},
           "algorithmic": {"stage1_pairs": p1, "stage2_pairs": p2, "flat_pairs": pf, "flop_per_pair": flop_pair,
                           "hisa_tflop": (p1 + p2) * flop_pair / 1e12, "flat_tflop": pf * flop_pair / 1e12},
           "roofline": roof,
           "hbm_step": {"algorithmic_bytes": hbm_bytes, "GBs": hbm_bytes / (ms_step * 1e-3) / 1e9,
                        "frac_of_peak": hbm_bytes / (ms_step * 1e-3) / 1e9 / PEAK_HBM_GBS}}
    ctx = dict(wl=wl, Q=Q, K=K, block_idx=block_idx, topk_idx=topk_idx, flat_idx=None)
    if with_flat:
        ws_f = torch.empty(hisa.hisa_workspace_bytes(hisa.OP_FLAT_TOPK, Q, K, 1, 0, wl.k), dtype=torch.uint8, device=dev)
        flat_idx = torch.empty((T, wl.k), dtype=torch.int32, device=dev)
        ms_flat, _ = time_region(lambda: hisa.dsa_flat_indexer_topk(Q, K, wl.k, topk_idx=flat_idx, ws=ws_f), flat_steps, 1)
        peak = roof["peak"] if roof["bound"] in ("mfma", "alu") else PEAK_BF16_TFLOPS
        out["flat"] = {"ms": ms_flat, "queries_per_s": T / (ms_flat * 1e-3),
                       "tflops": pf * flop_pair / (ms_flat * 1e-3) / 1e12,
                       "frac_of_mfma_peak": pf * flop_pair / (ms_flat * 1e-3) / 1e12 / peak,
                       "what": "the flat DSA indexer built here (scoring kernel + separate top-k over logits in HBM)"}
        out["speedup_vs_flat"] = ms_flat / ms_step
        # Eq. 12 over every query, computed by the library's own diagnostic kernel
        out["iou_hisa_vs_flat_mean"] = float(hisa.hisa_index_iou(topk_idx, flat_idx).mean().item())
        if wl.needles:
            out["needles"] = needle_recall(wl, block_idx, topk_idx, flat_idx)
        ctx["flat_idx"] = flat_idx
        del ws_f
    del ws1, ws2, pooled
    return out, ctx


def short_form(r):
    """The fields of a configuration's result that go into `all_configs` of the headline line."""
    roof = {k: r["roofline"][k] for k in ("bound", "achieved", "peak", "unit", "frac", "kernel", "ms_per_launch")}
    out = {"workload": r["workload"], "dtype": r["dtype"], "value": r["value"], "unit": r["unit"],
           "ms_per_step": r["ms_per_step"], "stage_ms": r["stage_ms"], "roofline": roof}
    for key in ("flat", "speedup_vs_flat"):
        if key in r:
            out[key] = r[key] if key != "flat" else {"ms": r["flat"]["ms"]}
    return out


def profile_mode(a, torch, hisa, W):
    """For rocprofv3: the step (or the flat indexer) a few times plus a 256 MiB device copy whose
    FETCH_SIZE / WRITE_SIZE readings calibrate those counters; nothing is timed here."""
    wl = W.config(a.workload)
    Q, K = hisa.to_device(wl)
    pd = hisa.DTYPE_CODE[wl.pooled_dtype]
    T, M, dev = wl.T, wl.s_max // wl.B, Q.q.device
    decode = wl.q_seq is not None
    pooled = torch.zeros((wl.n_seq, M, wl.d), dtype=torch.bfloat16 if pd == hisa.HISA_BF16 else torch.float32, device=dev)
    block_idx = torch.empty((T, wl.m), dtype=torch.int32, device=dev)
    topk_idx = torch.empty((T, wl.k), dtype=torch.int32, device=dev)
    ws1 = torch.empty(max(1, hisa.hisa_workspace_bytes(hisa.OP_BLOCK_SCORE_TOPK, Q, K, wl.B, wl.m, wl.k)),
                      dtype=torch.uint8, device=dev)
    ws2 = torch.empty(max(1, hisa.hisa_workspace_bytes(hisa.OP_TOKEN_REFINE_TOPK, Q, K, wl.B, wl.m, wl.k)),
                      dtype=torch.uint8, device=dev)
    hisa.hisa_pool_blocks(K, wl.B, pooled=pooled, pooled_dtype=pd)
    if a.profile_flat:
        ws_f = torch.empty(hisa.hisa_workspace_bytes(hisa.OP_FLAT_TOPK, Q, K, 1, 0, wl.k), dtype=torch.uint8, device=dev)
        for _ in range(max(1, a.steps)):
            hisa.dsa_flat_indexer_topk(Q, K, wl.k, topk_idx=topk_idx, ws=ws_f)
    else:
        for _ in range(max(1, a.steps)):
            if not decode:
                hisa.hisa_pool_blocks(K, wl.B, pooled=pooled, pooled_dtype=pd)
            hisa.hisa_block_score_topk(Q, K, pooled, pd, wl.B, wl.m, block_idx=block_idx, ws=ws1)
            hisa.hisa_token_refine_topk(Q, K, wl.B, wl.m, block_idx, wl.k, topk_idx=topk_idx, ws=ws2)
    src = torch.ones(64 << 20, dtype=torch.float32, device=dev)     # 256 MiB read + 256 MiB written
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"profile_mode": True, "workload": a.workload, "steps": a.steps,
                      "library_version": hisa.version(), "calibration_copy_bytes": src.numel() * 4}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="prefill64k_bf16")
    ap.add_argument("--flat-steps", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-flat", action="store_true")
    ap.add_argument("--no-all-configs", action="store_true",
                    help="headline workload only: leave out the fp8-keys variant and the other four configurations")
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
    if a.profile_mode:
        profile_mode(a, torch, hisa, W)
        return
    out_cfg, ctx = bench_config(a.workload, a.steps, a.warmup, a.flat_steps, torch, hisa, W, with_flat=not a.no_flat)
    wl, dev = ctx["wl"], ctx["Q"].q.device
    roof = out_cfg["roofline"]
    # what this chip delivers to a kernel that does nothing else: a 1 GiB streaming copy and a loop
    # of MFMAs only (the library's probe kernels), for the fraction of the ATTAINABLE peak
    src = torch.empty(1 << 29, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    ms_copy, _ = time_region(lambda: hisa.hisa_probe_copy(src, dst), 5, 1)
    probe_out = torch.empty(512 * 256, dtype=torch.float32, device=dev)
    flop_box = []
    ms_mfma, _ = time_region(lambda: flop_box.append(hisa.hisa_probe_mfma(probe_out, 20000)), 3, 1)
    ms_mfma8, _ = time_region(lambda: flop_box.append(hisa.hisa_probe_mfma_fp8(probe_out, 10000)), 3, 1)
    # the same two loops on operands that toggle like real data (pseudo-random values): the chip does
    # not hold its full clock under them, so this is the ceiling a scoring kernel on real keys has
    tog_box = []
    ms_tog, _ = time_region(lambda: tog_box.append(hisa.hisa_probe_mfma_toggling(probe_out, 40000, False)), 3, 1)
    ms_tog8, _ = time_region(lambda: tog_box.append(hisa.hisa_probe_mfma_toggling(probe_out, 20000, True)), 3, 1)
    attainable = {"hbm_copy_GBs": 2.0 * src.numel() / (ms_copy * 1e-3) / 1e9,
                  "mfma_bf16_TFLOPs": flop_box[0] / (ms_mfma * 1e-3) / 1e12,
                  "mfma_fp8_TFLOPs": flop_box[-1] / (ms_mfma8 * 1e-3) / 1e12,
                  "mfma_bf16_toggling_operands_TFLOPs": tog_box[0] / (ms_tog * 1e-3) / 1e12,
                  "mfma_fp8_toggling_operands_TFLOPs": tog_box[-1] / (ms_tog8 * 1e-3) / 1e12}
    del src, dst
    if roof["bound"] == "hbm":
        roof["frac_of_attainable"] = roof["achieved"] / attainable["hbm_copy_GBs"]
    elif roof["bound"] == "mfma":
        roof["frac_of_attainable"] = roof["achieved"] / (
            attainable["mfma_fp8_TFLOPs"] if roof["peak"] == PEAK_FP8_TFLOPS else attainable["mfma_bf16_TFLOPs"])
        roof["frac_of_attainable_toggling_operands"] = roof["achieved"] / (
            attainable["mfma_fp8_toggling_operands_TFLOPs"] if roof["peak"] == PEAK_FP8_TFLOPS
            else attainable["mfma_bf16_toggling_operands_TFLOPs"])

    out = {
        "metric": "indexer queries/s at 64K context (HISA: pool + Stage 1 + Stage 2)" if "64k" in a.workload
                  else f"indexer queries/s ({a.workload})",
        "value": out_cfg["value"], "unit": "queries/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": out_cfg["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": out_cfg["dtype"], "data": "synthetic", "library_version": hisa.version(),
    }
    for key in ("config", "stage_ms", "algorithmic", "roofline"):
        out[key] = out_cfg[key]
    out["attainable"] = attainable
    out["hbm_step"] = out_cfg["hbm_step"]
    for key in ("flat", "speedup_vs_flat", "iou_hisa_vs_flat_mean", "needles"):
        if key in out_cfg:
            out[key] = out_cfg[key]

    headline = a.workload == "prefill64k_bf16" and not a.no_flat
    host = None
    if not a.no_cpu_baseline:
        # the rows the oracle is compared with, on the host, before the device tensors are released
        host = [ctx["block_idx"].cpu().numpy(), ctx["topk_idx"].cpu().numpy(),
                None if ctx["flat_idx"] is None else ctx["flat_idx"].cpu().numpy()]
    del ctx
    torch.cuda.empty_cache()
    if headline and not a.no_all_configs:
        # the configuration's second variant (fp8 e4m3 keys with per-token scales) and the four other
        # configurations of the benchmark definition, each timed the same way, in short form
        r, c = bench_config("prefill64k_fp8", a.steps, a.warmup, a.flat_steps, torch, hisa, W)
        out["fp8_keys_variant"] = short_form(r)
        del c
        torch.cuda.empty_cache()
        out["all_configs"] = {}
        for name, st, fst in (("tiny_f32", a.steps, a.flat_steps), ("prefill16k_bf16", a.steps, a.flat_steps),
                              ("decode32x128k_bf16", max(a.steps, 50), 5), ("chunk16k_1m_fp8", min(a.steps, 10), 1)):
            r, c = bench_config(name, st, a.warmup, fst, torch, hisa, W)
            out["all_configs"][name] = short_form(r)
            del c
            torch.cuda.empty_cache()
    if host is not None:
        out["cpu_baseline"] = cpu_baseline(wl, *host)
    print(json.dumps(out), flush=True)
    if host is not None and out["cpu_baseline"]["mismatches"]:
        print(f"bench.py: {out['cpu_baseline']['mismatches']} of the sampled queries differ from the oracle beyond "
              f"the benchmark's tolerance", file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
