"""Parity at the full benchmark sizes, in the launch configuration bench.py times: the library
runs on ALL queries of each configuration and the oracle checks a stratified sample of them
(uniform positions, the regime boundaries of Section 4.1, block edges, needle targets): more than 4096
HISA queries at the 16K and 64K prefills, more than 1024 at the 1M chunk, every query of the decode
batch.  The flat oracle costs the whole causal prefix per query (hours over every query of a 64K
context), so its sample stays small."""
import numpy as np
import pytest

from paper_2603_28458_amd import workloads as W
from tests.parity import run_and_check, sample_queries

pytestmark = pytest.mark.gpu


def _run(name, n_hisa, n_flat):
    wl = W.config(name)
    qs = sample_queries(wl, n_hisa, seed=1)
    fq = qs if n_flat is None else sample_queries(wl, n_flat, seed=2)[:: max(1, len(qs) // max(1, n_flat))][:n_flat]
    print(f"\n[parity-full] {name}: T={wl.T} L={int(wl.seq_len.max())} n_seq={wl.n_seq} B={wl.B} m={wl.m} k={wl.k} "
          f"k_dtype={wl.k_dtype}; oracle on {len(qs)} queries (flat on {len(fq)})", flush=True)
    return run_and_check(wl, queries=qs, flat_queries=fq, verbose=True)


def test_config2_prefill_16k_bf16():
    _run("prefill16k_bf16", 4096, 96)


def test_config3_prefill_64k_bf16():
    _run("prefill64k_bf16", 4096, 24)


def test_config3_prefill_64k_fp8():
    _run("prefill64k_fp8", 4096, 24)


def test_config4_decode_32x128k():
    _run("decode32x128k_bf16", 32, None)


def test_config5_chunk_16k_against_1m_fp8():
    _run("chunk16k_1m_fp8", 1024, 6)


def test_maximum_block_count_budget_and_k():
    # the limits of the boundary: 65536 pooled keys per query (B = 32 over 2M tokens), m = 1024 kept blocks
    # (32768 candidates), k = 8192; four queries at the end of the context.  (The flat call at k = 8192 over
    # 2M keys is outside its own limit -- 32 segments x 8192 -- and is not part of this case.)
    wl = W.make_workload("max_M_m_k", seq_len=2097152, T=4, H=64, d=128, B=32, m=1024, k=8192, q_dtype="bf16",
                         k_dtype="bf16", seed=180)
    print(f"\n[parity-full] {wl.name}: blocks={wl.s_max // wl.B} m={wl.m} k={wl.k}", flush=True)
    run_and_check(wl, check_flat=False, verbose=True)


def test_maximum_candidate_count():
    # m * B = 65536 candidates per query (the limit), k = 8192, through the two-kernel Stage 2
    wl = W.make_workload("max_cand", seq_len=131072, T=4, H=64, d=128, B=64, m=1024, k=8192, q_dtype="bf16",
                         k_dtype="fp8_e4m3", seed=181)
    print(f"\n[parity-full] {wl.name}: candidates={wl.m * wl.B} k={wl.k}", flush=True)
    run_and_check(wl, check_flat=False, verbose=True)
