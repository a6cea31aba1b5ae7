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
