"""Parity on seeded random shapes: every call of the library against the oracle (tests/parity.py)
on small workloads whose mode (prefill, chunk against a longer prefix, decode batch, padded varlen,
packed stream with straddling blocks), head count, block size, budgets, lengths and key type are
drawn at random.  The fixed-shape tests aim at known branches; this one walks between them."""
import numpy as np
import pytest

from paper_2603_28458_amd import workloads as W
from tests.parity import run_and_check, sample_queries

pytestmark = pytest.mark.gpu


def _draw(rng, name, seed):
    mfma = rng.random() < 0.7
    if mfma:
        H, d = int(rng.choice([32, 64])), 128
        B = int(rng.choice([32, 64, 128, 256]))
        kd, qd = str(rng.choice(["bf16", "fp8_e4m3"])), "bf16"
    else:
        H, d = int(rng.integers(1, 9)), int(rng.choice([4, 8, 20, 64]))
        B = int(rng.choice([1, 3, 8, 16, 50]))
        kd = qd = "f32"
    mode = str(rng.choice(["prefill", "chunk", "decode", "varlen", "packed"]))
    m = int(rng.integers(2, 12))
    k = min(int(rng.integers(1, m * B + 1)), 700)
    if mode in ("prefill", "chunk"):
        L = min(int(rng.integers(1, 40 * B if B > 8 else 600)), 6000)
        T = L if mode == "prefill" else int(rng.integers(1, L + 1))
        kw = dict(n_seq=1, seq_len=L, T=T, mode="prefill")
    elif mode == "decode":
        n = int(rng.integers(1, 7))
        lens = [int(rng.integers(0 if rng.random() < 0.1 else 1, 3000)) for _ in range(n)]
        if max(lens) == 0:
            lens[0] = 5
        kw = dict(n_seq=n, seq_len=lens, T=n, mode="decode")
    else:
        n = int(rng.integers(1, 6))
        lens = [int(rng.integers(1, 900)) for _ in range(n)]
        kw = dict(n_seq=n, seq_len=lens, T=int(sum(lens)), mode="varlen")
    wl = W.make_workload(name, H=H, d=d, B=B, m=m, k=k, q_dtype=qd, k_dtype=kd, seed=seed, **kw)
    return (W.pack(wl) if mode == "packed" else wl), mode


@pytest.mark.parametrize("stream", [11, 12])
def test_random_shapes(stream):
    rng = np.random.default_rng(stream)
    for case in range(50):
        wl, mode = _draw(rng, f"rand{stream}_{case}", 1000 * stream + case)
        print(f"\n[parity] {wl.name}: mode={mode} T={wl.T} H={wl.H} d={wl.d} B={wl.B} m={wl.m} k={wl.k} "
              f"k={wl.k_dtype} n_seq={wl.n_seq} s_max={wl.s_max} seed={wl.seed}", flush=True)
        run_and_check(wl, queries=sample_queries(wl, 40, seed=case))


def test_random_small_batches_against_long_contexts():
    """Up to 256 queries against up to hundreds of thousands of keys (a chunk at the end of a long
    prefix, or a decode batch of up to 39 ragged sequences): the shapes whose Stage 1 runs in one
    launch per batch, with up to 8000 blocks per sequence, and whose Stage 2 takes the two-kernel path."""
    rng = np.random.default_rng(21)
    for case in range(16):
        H, B = int(rng.choice([32, 64])), int(rng.choice([32, 64, 128]))
        kd = str(rng.choice(["bf16", "fp8_e4m3"]))
        m = int(rng.integers(2, 65))
        k = min(int(rng.integers(1, m * B + 1)), 2048)
        if rng.random() < 0.5:
            L = int(rng.integers(B, 260000 if B == 32 else 400000))
            kw = dict(n_seq=1, seq_len=L, T=int(rng.integers(1, 257)), mode="prefill")
        else:
            n = int(rng.integers(1, 40))
            top = int(rng.integers(2000, 120000))
            kw = dict(n_seq=n, seq_len=[int(rng.integers(1, top)) for _ in range(n)], T=n, mode="decode")
        wl = W.make_workload(f"small{case}", H=H, d=128, B=B, m=m, k=k, q_dtype="bf16", k_dtype=kd,
                             seed=21000 + case, **kw)
        print(f"\n[parity] {wl.name}: T={wl.T} H={H} B={B} m={m} k={k} k={kd} n_seq={wl.n_seq} s_max={wl.s_max} "
              f"blocks={wl.s_max // B}", flush=True)
        run_and_check(wl, queries=sample_queries(wl, 24, seed=case), check_flat=wl.s_max <= 70000)
