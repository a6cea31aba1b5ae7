"""The regression bounds of tests/util.py must bite where the acceptance tolerance does not.

The fp8-key path scores the stored e4m3 codes against the bf16 query written as a SUM OF TWO e4m3
numbers per element (after a power-of-two scaling per head).  A kernel that lost the second term
would halve its matrix work and still pass the benchmark's 2e-2 acceptance tolerance.  Here that
mistake is planted on the CPU: the one-term and the two-term query are built with the library's
float8 cast and scored by the oracle; the one-term scores must fail the fp8 regression bound, the
two-term scores must pass it."""
import numpy as np
import pytest
import torch

from oracle import hisa_oracle as O
from paper_2603_28458_amd import workloads as W
from tests.util import DESIGN_RTOL, RTOL, check_scores


def _e4m3(x):
    """Round-to-nearest-even cast to OCP e4m3fn and back, by the library routine."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)


def _two_terms(q):
    """q [H, d] float64 (bf16 values) -> (hi, lo) with hi + lo ~ q: each head row is scaled by the power
    of two that puts its largest magnitude into [128, 256), hi = e4m3(q), lo = e4m3(q - hi)."""
    mag = np.abs(q).max(axis=1)
    e = np.floor(np.log2(np.where(mag > 0, mag, 1.0)))
    up = 2.0 ** (7.0 - e)[:, None]
    hi = _e4m3(q * up)
    lo = _e4m3(q * up - hi)
    return hi / up, lo / up


@pytest.mark.parametrize("seed", [7, 11])
def test_a_dropped_second_query_term_fails_the_fp8_bound_but_not_the_acceptance_tolerance(seed):
    wl = W.make_workload("bound_fp8", seq_len=2000, T=2000, H=64, d=128, B=128, m=6, k=384, q_dtype="bf16",
                         k_dtype="fp8_e4m3", n_needles=2, seed=seed)
    rng = np.random.default_rng(seed)
    keys = O.decode(wl.keys[0], wl.k_dtype, wl.k_scale[0])
    worst_one, worst_two = 0.0, 0.0
    for t in rng.choice(wl.T, size=12, replace=False):
        q = O.decode(wl.q[t], wl.q_dtype)
        w = wl.w[t].astype(np.float64)
        vis = keys[: int(wl.positions()[t]) + 1]
        want = O.score(q, w, vis)[None]
        hi, lo = _two_terms(q)
        one = O.score(hi, w, vis)[None]                   # the planted mistake: the lo term never ran
        # two MFMAs accumulate (hi . k) + (lo . k) per head before the ReLU
        two = (w @ np.maximum(hi @ vis.T + lo @ vis.T, 0.0))[None]
        # the acceptance tolerance alone lets the mistake through ...
        worst_one = max(worst_one, check_scores(one, want, RTOL["fp8_e4m3"], "one-term query, acceptance"))
        # ... the regression bound does not
        with pytest.raises(AssertionError, match="regression bound"):
            check_scores(one, want, RTOL["fp8_e4m3"], "one-term query", DESIGN_RTOL["fp8_e4m3"])
        worst_two = max(worst_two, check_scores(two, want, RTOL["fp8_e4m3"], "two-term query", DESIGN_RTOL["fp8_e4m3"]))
    assert worst_one > 10 * DESIGN_RTOL["fp8_e4m3"]
    # the two-term form is the query to 2^-17 of each head's largest element: far inside even the bf16 bound
    assert worst_two < DESIGN_RTOL["bf16"]


def test_a_lost_mantissa_bit_fails_the_bf16_bound_but_not_the_acceptance_tolerance():
    """bf16 keys: an operand path that loses the lowest mantissa bit of the query (a wrong packing, a
    conversion through a narrower type) changes the scores by about 1e-4 of the row maximum: invisible
    to the 2e-2 acceptance tolerance, outside the 1e-5 regression bound."""
    wl = W.make_workload("bound_bf16", seq_len=1500, T=1500, H=64, d=128, B=128, m=6, k=384, q_dtype="bf16",
                         k_dtype="bf16", seed=5)
    keys = O.decode(wl.keys[0], wl.k_dtype)
    for t in (700, 1400):
        q = O.decode(wl.q[t], wl.q_dtype)
        w = wl.w[t].astype(np.float64)
        vis = keys[: t + 1]
        want = O.score(q, w, vis)[None]
        q_cut = O.decode(wl.q[t] & np.uint16(0xFFFE), wl.q_dtype)     # lowest mantissa bit cleared
        got = O.score(q_cut, w, vis)[None]
        worst = check_scores(got, want, RTOL["bf16"], "lost mantissa bit, acceptance")
        assert worst > 2 * DESIGN_RTOL["bf16"]
        with pytest.raises(AssertionError, match="regression bound"):
            check_scores(got, want, RTOL["bf16"], "lost mantissa bit", DESIGN_RTOL["bf16"])
