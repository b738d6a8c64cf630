"""Pins for the oracle's execution of Chen et al.'s two strategies (Section 2) and for the
numerical comparison of Section 4.3.  Every expected value here is a closed form derived from
the strategies' definitions or a claim the paper makes about them; none comes from the library."""
import math

import pytest

from oracle import chen, policy_dp


@pytest.mark.parametrize("t", [1, 2, 3, 4, 9, 10, 16, 17, 50, 100, 1000])
@pytest.mark.parametrize("beta", [1, 3, 7])
def test_sqrt_cost_and_memory_closed_forms(t, beta):
    nseg, L, last = chen.chen_sqrt_segments(t)
    assert (nseg - 1) * L + last == t and 1 <= last <= L
    tr = chen.execute_chen_sqrt(t, beta)
    assert tr.backwards == t and tr.backward_order == list(range(t, 0, -1))
    # the first pass stops at the last cut; every part is then run once with its states kept
    assert tr.forwards == (nseg - 1) * L + t
    assert tr.forwards < 2 * t or t == 1             # "an additional forward pass on average" (Section 2)
    # stack while part j is loaded: h_0 and the cuts before it, plus all but its last internal state
    expect = max(nseg + (last - 1) * beta, (nseg - 1) + (L - 1) * beta) if nseg > 1 else 1 + (t - 1) * beta
    assert tr.peak == expect


@pytest.mark.parametrize("k", [2, 5, 10, 31])
def test_sqrt_memory_is_the_papers_figure_on_perfect_squares(k):
    # Section 4.3: sqrt(t) hidden states and sqrt(t) internal states of beta units each
    for beta in (2, 5, 10):
        tr = chen.execute_chen_sqrt(k * k, beta)
        assert tr.peak == k + (k - 1) * beta
        assert tr.peak <= chen.chen_sqrt_memory(k * k, beta)
        assert tr.forwards == 2 * k * k - k


@pytest.mark.parametrize("p", [1, 2, 3, 6, 10])
def test_recursive_bisection_closed_forms(p):
    # k = 1 on t = 2^p: F(n) = n/2 + 2 F(n/2), F(1) = 1; one memorised state per level
    t = 1 << p
    tr = chen.execute_chen_recursive(t, 1)
    assert tr.forwards == t + p * (t // 2)
    assert tr.peak == 1 + p                            # "minimum possible memory usage of log2(t)"
    assert tr.backward_order == list(range(t, 0, -1))


@pytest.mark.parametrize("t", [1, 2, 7, 30, 100, 257, 1000])
@pytest.mark.parametrize("k", [1, 2, 3, 9])
def test_recursive_bounds(t, k):
    tr = chen.execute_chen_recursive(t, k)
    levels = 0
    n = t
    while n > 1:
        n = -(-n // min(k + 1, n))
        levels += 1
    assert tr.peak <= 1 + k * levels                   # O(k log_{k+1} t) memory
    assert tr.forwards <= t * (1 + levels)             # O(t log_k t) cost
    assert tr.backwards == t


def test_capacity_is_enforced():
    tr = chen.execute_chen_sqrt(50, 3)
    chen.execute_chen_sqrt(50, 3, capacity=tr.peak)
    with pytest.raises(AssertionError):
        chen.execute_chen_sqrt(50, 3, capacity=tr.peak - 1)


@pytest.mark.parametrize("t", [5, 16, 37, 100, 150])
def test_msm_is_at_least_as_good_at_the_same_memory(t):
    # Section 4.2: both strategies are policies of BPTT-MSM, so the optimum cannot cost more
    alpha, beta = 4, 3
    tr = chen.execute_chen_sqrt(t, beta)
    C = policy_dp.msm_tables(t, tr.peak, alpha, beta)[0]
    assert C[t, tr.peak] <= tr.forwards
    for k in (1, 2, 4):
        tr = chen.execute_chen_recursive(t, k)
        C_h = policy_dp.hsm_tables(t, tr.peak)[0]
        assert C_h[t, tr.peak] <= tr.forwards
        assert policy_dp.msm_tables(t, tr.peak, alpha, beta)[0][t, tr.peak] <= C_h[t, tr.peak]


@pytest.mark.parametrize("beta", [2, 5])
def test_section_4_3_comparison(beta):
    for t in (100, 400):
        # right panel: at the sqrt(t) strategy's memory BPTT-MSM does not do worse than cost 2 ...
        cost = chen.msm_cost_at_chen_memory(t, beta)
        assert cost <= 2.0
        assert cost > 1.5                              # ... and "does not perform significantly faster"
        # left panel: at cost 2 it needs less memory (ratio below 1)
        m, ratio = chen.msm_memory_for_cost(t, beta, 2.0)
        assert ratio < 1.0
        C = policy_dp.msm_tables(t, m, beta + 1, beta)[0]
        assert C[t, m] <= 2 * t and (m == 1 or C[t, m - 1] > 2 * t)
