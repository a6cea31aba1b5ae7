"""Exact top-k over rows of up to 16384 scores (the in-LDS select behind Eqs. 2, 6 and 9) on
crafted score rows, through the flat indexer with one head, d = 4, q = (1, 0, 0, 0): the score of
key s is exactly w * max(0, k_s[0]) (see test_select_stream_gpu for the harness).

The threshold search brackets the k-th largest key by key ranges: first [largest per-thread
minimum, row maximum], then 256 equal bins of the range that holds the k-th, a list of the
candidates of the kept bin, and an early end when a bin is taken whole.  The patterns aim at its
branches: an estimate of the low end that lies above the k-th (sorted rows), a maximum far from
the rest (bins too coarse, list overflow), ties at the threshold, zeros from the ReLU, negative
scores, ranges down to one key, budgets next to the row length.
"""
import numpy as np
import pytest

from tests.test_select_stream_gpu import _run

pytestmark = pytest.mark.gpu

N = 16384          # the longest row the in-LDS select takes


def _pos(n):
    return [n - 1, n - 2, n // 2, 4097, 2048, 2047, 300, 0]


def test_sorted_rows_put_the_low_estimate_on_the_wrong_side():
    up = np.arange(1, N + 1, dtype=np.float32)              # ascending: every thread's minimum is large
    _run(up, _pos(N))
    _run(up[::-1].copy(), _pos(N))                          # descending
    _run(up, [N - 1, 9000], k=128)
    _run(up[::-1].copy(), [N - 1, 9000], k=8000)            # the k-th far below the first range


def test_one_far_maximum_and_a_crowd():
    rng = np.random.default_rng(21)
    v = rng.uniform(1.0, 1.001, N).astype(np.float32)       # 16384 keys inside a few thousand ulps
    v[777] = 3.0e38
    _run(v, _pos(N))
    v[5] = 1.0e-30                                          # and a far minimum
    _run(v, [N - 1, 8193], k=8192)                          # the largest budget the library takes


def test_ties_at_the_threshold_and_list_overflow():
    rng = np.random.default_rng(22)
    v = rng.integers(0, 3, N).astype(np.float32)            # ~5400 copies of 0, 1, 2
    _run(v, _pos(N))
    v = np.full(N, 7.0, dtype=np.float32)                   # one key only
    _run(v, _pos(N))
    v[::2] = np.nextafter(np.float32(7.0), np.float32(8.0))  # two adjacent keys, 8192 each
    _run(v, _pos(N))
    _run(v, [N - 1], k=8192)                                # exactly the upper key's copies
    _run(v, [N - 1], k=8191)


def test_relu_zeros_and_negative_scores():
    rng = np.random.default_rng(23)
    v = rng.standard_normal(N).astype(np.float32)           # half of the scores are exactly 0
    _run(v, _pos(N))
    _run(v, [N - 1, 5000], k=8192)                          # the budget reaches the zeros (about half the row)
    _run(np.where(v > 1.0, v, 0).astype(np.float32), [N - 1, 5000])   # ~2600 positive, zeros tie at the threshold
    _run(np.abs(v), [N - 1, 5000], w=-2.0)                  # all scores negative
    _run(v, [N - 1, 5000], w=-2.0, k=8192)                  # zeros on top, negatives below


def test_wide_magnitudes_and_small_rows():
    rng = np.random.default_rng(24)
    v = np.exp(rng.uniform(-60, 60, N)).astype(np.float32)
    _run(v, _pos(N))
    for n in (2049, 2050, 2112, 5000):                      # budgets next to the row length
        _run(v[:n].copy(), [n - 1, n - 2], k=2048)
    _run(v[:300].copy(), [299, 128, 127, 5], k=128)
    _run(v[:300].copy(), [299], k=1, want_scores=False)
