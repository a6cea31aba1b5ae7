"""Exact top-k over long rows (flat indexer, Eq. 2) on crafted score rows.

One head, d = 4, q = (1, 0, 0, 0), gate w: the score of key s is exactly w * max(0, k_s[0]), so a
test can plant any score pattern.  Expected sets come from the oracle's top_select (score
descending, index ascending) on the same scores.  The patterns aim at the branches of the
streaming select: ties that overflow the candidate list, a threshold outside the sampled key
range on either side, values spread over many magnitudes, negative scores, short rows.
"""
import numpy as np
import pytest
import torch

from oracle import hisa_oracle as O
from paper_2603_28458_amd import hisa

pytestmark = pytest.mark.gpu

S_MAX = 20000          # > 16384: the row goes through the streaming select
K = 2048


def _run(values: np.ndarray, positions, k=K, w=1.0, want_scores=True):
    """values[s] >= 0 is the planted score / w of key s; queries sit at `positions`."""
    dev = "cuda:0"
    n = values.size
    keys = np.zeros((1, n, 4), dtype=np.float32)
    keys[0, :, 0] = values
    kt = torch.from_numpy(keys).to(dev)
    seq_len = torch.tensor([n], dtype=torch.int32, device=dev)
    Kd = hisa.Keys(kt, seq_len, hisa.HISA_F32)
    T = len(positions)
    q = torch.zeros((T, 1, 4), dtype=torch.float32, device=dev)
    q[:, 0, 0] = 1.0
    wt = torch.full((T, 1), float(w), dtype=torch.float32, device=dev)
    qpos = torch.tensor(list(positions), dtype=torch.int32, device=dev)
    Qd = hisa.Queries(q, wt, hisa.HISA_F32, q_pos=qpos)
    idx, sc = hisa.dsa_flat_indexer_topk(Qd, Kd, k, want_topk_scores=want_scores)
    torch.cuda.synchronize()
    idx = idx.cpu().numpy()
    sc = sc.cpu().numpy() if sc is not None else None
    scores_all = np.float32(w) * np.maximum(values.astype(np.float32), np.float32(0))
    for r, p in enumerate(positions):
        vis = scores_all[: p + 1].astype(np.float64)
        want = O.top_select(vis, np.arange(p + 1, dtype=np.int64), k)
        got = idx[r]
        nv = want.size
        assert np.array_equal(got[:nv], want), f"row {r} (pos {p}): selection differs"
        assert np.all(got[nv:] == -1)
        if sc is not None:
            assert np.array_equal(sc[r, :nv], scores_all[want])
            assert np.all(np.isneginf(sc[r, nv:]))


POS = [S_MAX - 1, S_MAX - 2, 12345, 8193, 4096, K, K - 1, 100, 0]


def test_all_scores_equal_takes_the_lowest_indices():
    _run(np.full(S_MAX, 3.0, dtype=np.float32), POS)


def test_all_scores_zero():
    _run(np.zeros(S_MAX, dtype=np.float32), POS)


def test_random_normal_and_wide_magnitudes():
    rng = np.random.default_rng(7)
    _run(np.abs(rng.standard_normal(S_MAX)).astype(np.float32), POS)
    _run(np.exp(rng.uniform(-30, 30, S_MAX)).astype(np.float32), POS)


def test_few_distinct_values_with_ties_at_the_threshold():
    rng = np.random.default_rng(8)
    v = rng.integers(0, 4, S_MAX).astype(np.float32)          # ~5000 copies of each of 4 values
    _run(v, POS)
    v = np.where(rng.random(S_MAX) < 0.05, 2.0, 1.0).astype(np.float32)   # ~1000 above, ties below
    _run(v, POS)


def _sampled_indices(n):
    # the select samples up to 4096 entries: 64 evenly spaced runs of 64 consecutive entries
    run_stride = n >> 6 if n > 4096 else 64
    return {(j >> 6) * run_stride + (j & 63) for j in range(4096) if (j >> 6) * run_stride + (j & 63) < n}


def test_threshold_above_the_sampled_range():
    # every sampled position holds a small value; 3000 unsampled positions hold large distinct ones
    n = S_MAX
    rng = np.random.default_rng(9)
    v = rng.uniform(1.0, 2.0, n).astype(np.float32)
    free = np.array(sorted(set(range(n)) - _sampled_indices(n)))
    big = rng.choice(free, size=3000, replace=False)
    v[big] = rng.uniform(100.0, 1.0e6, 3000).astype(np.float32)
    _run(v, [n - 1])


def test_threshold_below_the_sampled_range():
    # every sampled position holds a large value (1000 of them are unique maxima), the rest small:
    # the k-th best lies below everything the sample saw
    n = S_MAX
    rng = np.random.default_rng(10)
    v = rng.uniform(1.0e-3, 2.0e-3, n).astype(np.float32)
    samp = np.array(sorted(_sampled_indices(n)))
    keep = rng.choice(samp, size=1000, replace=False)
    v[samp] = 5.0
    v[keep] = rng.uniform(10.0, 20.0, 1000).astype(np.float32)
    v[samp[~np.isin(samp, keep)]] = 1.0e-3 * 1.5    # sampled but inside the small range
    v[keep[:5]] = 7.0
    _run(v, [n - 1], k=K)


def test_negative_gate_gives_negative_scores():
    rng = np.random.default_rng(11)
    _run(np.abs(rng.standard_normal(S_MAX)).astype(np.float32), [S_MAX - 1, 9000], w=-1.5)


def test_small_budgets_and_no_score_output():
    rng = np.random.default_rng(12)
    v = np.abs(rng.standard_normal(S_MAX)).astype(np.float32)
    _run(v, [S_MAX - 1, 5000], k=1, want_scores=False)
    _run(v, [S_MAX - 1, 5000], k=37)
