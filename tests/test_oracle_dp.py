"""Pins for the oracle's policy dynamic programs and its symbolic executor.

Nothing here compares the oracle with itself: every check is a closed form, bound or claim that
the paper prints, a brute-force enumeration that consults no cost table, or an invariant of the
execution procedure checked by an abstract machine.
"""
import math
import os

import numpy as np
import pytest

from oracle import executor_sim as ex
from oracle import policy_dp as dp

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _paper_values():
    out = {}
    for line in open(os.path.join(GOLDEN, "paper_values.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = line.split("=")
            out[k.strip()] = float(v)
    return out


@pytest.fixture(scope="module")
def hsm():
    return dp.hsm_tables(600, 60)


@pytest.fixture(scope="module")
def ism():
    return dp.ism_tables(600, 60)


@pytest.fixture(scope="module")
def msm43():
    return dp.msm_tables(300, 120, 4, 3)


# ---- P1: closed forms (Sections 3, 3.1, 3.2, 3.3) -------------------------------------------
def test_closed_forms_hsm(hsm):
    C, D = hsm
    t = np.arange(1, 601)
    assert np.array_equal(C[1:, 1], t * (t + 1) // 2)
    for tt in range(1, 61):
        assert np.all(C[tt, tt:] == 2 * tt - 1)
        assert np.all(D[tt, tt:] == 1)
    assert np.all(C[1, 1:] == 1)


def test_closed_forms_ism(ism):
    C, D = ism
    t = np.arange(1, 601)
    assert np.array_equal(C[1:, 1], t * (t + 1) // 2)   # falls out of the recurrence
    assert np.all(C[0, :] == 0)
    assert np.all(C[1:, 0] >= dp.INF)
    for tt in range(1, 61):
        assert np.all(C[tt, tt:] == tt)
        if tt > 1:
            assert C[tt, tt - 1] > tt


@pytest.mark.parametrize("alpha,beta", [(2, 2), (3, 2), (4, 3), (5, 4), (5, 5)])
def test_closed_forms_msm(alpha, beta):
    C = dp.msm_tables(40, 5 * 40, alpha, beta)[0]
    t = np.arange(1, 41)
    assert np.array_equal(C[1:, 1], t * (t + 1) // 2)
    assert np.all(C[1, 1:] == 1)
    for tt in range(1, 41):
        assert np.all(C[tt, alpha * tt:] == tt)         # plentiful memory: standard BPTT
    assert np.all(C[1:, 1:] >= t[:, None])              # never cheaper than one forward per step


# ---- P2: brute force over every policy of the family, t <= 8 --------------------------------
def test_brute_force_hsm_ism():
    C, D = dp.hsm_tables(8, 8)
    Ci, Di = dp.ism_tables(8, 8)
    for t in range(1, 9):
        for m in range(1, 9):
            assert ex.brute_force_hsm(t, m) == C[t, m], (t, m)
            assert ex.brute_force_ism(t, m) == Ci[t, m], (t, m)


@pytest.mark.parametrize("alpha,beta", [(2, 2), (3, 2), (4, 3), (5, 4)])
def test_brute_force_msm(alpha, beta):
    C = dp.msm_tables(8, 10, alpha, beta)[0]
    for t in range(1, 8):
        for m in range(1, 11):
            assert ex.brute_force_msm(t, m, alpha, beta) == C[t, m], (alpha, beta, t, m)
    for m in (1, 2, alpha, alpha + 1, 2 * alpha):       # t = 8 on a few budgets (the trees grow fast)
        if m <= 10:
            assert ex.brute_force_msm(8, m, alpha, beta) == C[8, m], (alpha, beta, 8, m)


# ---- P3: the paper's upper bounds (Section 3.5, appendix) ------------------------------------
def test_upper_bounds(hsm, ism):
    pv = _paper_values()
    C, _ = hsm
    Ci, _ = ism
    for t in range(1, 601):
        for m in range(1, 61):
            p = float(t) ** (1.0 + 1.0 / m)
            assert C[t, m] <= m * p * (1 + 1e-12), (t, m)
            assert C[t, m] < pv["bound_general_factor"] * p, (t, m)
            assert C[t, m] - t < pv["bound_without_first_pass_factor"] * p, (t, m)
            assert Ci[t, m] <= m * p * (1 + 1e-12), (t, m)          # appendix C.3
    for m in range(1, 61):
        for a in range(1, 8):
            lim = m ** a / math.factorial(a)
            tt = np.arange(1, 601)
            sel = tt[tt <= lim]
            assert np.all(C[sel, m] <= (a + 1) * sel), (m, a)
            assert np.all(Ci[sel, m] <= a * sel), (m, a)


# ---- P4: monotonicity and ordering of the three strategies ------------------------------------
def test_monotone_and_ordering(hsm, ism, msm43):
    C, _ = hsm
    Ci, _ = ism
    Cm = msm43[0]
    assert np.all(np.diff(C[1:, 1:], axis=0) > 0)       # increasing in t (appendix C.2)
    assert np.all(np.diff(C[1:, 1:], axis=1) <= 0)      # more memory never costs more
    assert np.all(np.diff(Ci[1:, 1:], axis=0) > 0)
    assert np.all(np.diff(Ci[1:, 1:], axis=1) <= 0)
    assert np.all(np.diff(Cm[1:, 1:], axis=0) > 0)
    assert np.all(np.diff(Cm[1:, 1:], axis=1) <= 0)
    # MSM searches a superset of both strategy spaces (Section 3.6)
    assert np.all(Cm[1:301, 1:61] <= C[1:301, 1:61])
    for k in range(1, 31):
        assert np.all(Cm[1:301, 4 * k] <= Ci[1:301, k]), k
    # same memory (alpha = 4 units per internal state): hidden wins for long sequences,
    # internal for short ones (Section 3.6)
    assert C[600, 40] < Ci[600, 10]
    assert Ci[12, 10] < C[12, 40]


# ---- P5: the headline claim ---------------------------------------------------------------------
def test_headline_claim():
    pv = _paper_values()
    t = int(pv["headline_t"])
    m = round(t * (1 - pv["headline_memory_saved"]))
    C, _ = dp.ism_tables(t, m)
    bw = pv["headline_backward_over_forward"]
    ratio = (C[t, m] + bw * t) / (t + bw * t)
    assert abs((ratio - 1.0) - pv["headline_time_overhead"]) < 0.02
    assert ratio == dp.theoretical_cost_ratio(int(C[t, m]), t)


# ---- P6: execution of the optimal policy on the abstract machine ------------------------------
def test_executor_counts_hsm(hsm):
    C, D = hsm
    for t, ms in [(20, range(1, 21)), (10, range(1, 11)), (4, [4]), (200, [1, 2, 3, 5, 8, 13, 21, 34, 55, 60]),
                  (600, [2, 7, 50])]:
        for m in ms:
            tr = ex.execute_hsm(D, t, m)
            assert tr.forwards == C[t, m] and tr.backwards == t, (t, m)
            assert tr.backward_order == list(range(t, 0, -1))
            assert tr.peak <= m
            if m <= t:
                assert tr.peak == m or C[t, m] == C[t, tr.peak]


def test_executor_counts_ism(ism):
    C, D = ism
    for t, ms in [(20, range(1, 21)), (200, [1, 2, 3, 5, 8, 13, 21, 34, 55, 60]), (600, [2, 7, 50])]:
        for m in ms:
            tr = ex.execute_ism(D, t, m)
            assert tr.forwards == C[t, m] and tr.backwards == t, (t, m)
            assert tr.backward_order == list(range(t, 0, -1))
            assert tr.peak <= m


@pytest.mark.parametrize("alpha,beta", [(4, 3), (4, 4), (5, 4), (2, 1)])
def test_executor_counts_msm(alpha, beta):
    C, C1, C2, D1, D2, H = dp.msm_tables(120, 90, alpha, beta)
    for t in (1, 2, 3, 7, 20, 57, 120):
        for m in range(1, 91):
            tr = ex.execute_msm(D1, D2, H, t, m, alpha, beta)
            assert tr.forwards == C[t, m] and tr.backwards == t, (t, m)
            assert tr.backward_order == list(range(t, 0, -1))
            assert tr.peak <= m, (t, m, tr.peak)


def test_machine_rejects_illegal_programs():
    """The abstract machine must actually be able to fail (otherwise P6 proves nothing)."""
    mc = ex.Machine(3, capacity=1, start_units=1)
    mc.forward('top')
    with pytest.raises(ex.MachineError):
        mc.push_hidden()                                 # over budget
    mc = ex.Machine(3, capacity=3, start_units=1)
    mc.forward('top')
    with pytest.raises(ex.MachineError):
        mc.backward('core')                              # step 1 before step 3
    mc = ex.Machine(2, capacity=3, start_units=1)
    mc.forward('top'); mc.forward('core')
    mc.backward('core')
    with pytest.raises(ex.MachineError):
        mc.backward('core')                              # internal state already consumed
    with pytest.raises(ex.MachineError):
        mc.finish()
    # a deliberately bad policy costs more than the optimum but still runs
    C, D = dp.hsm_tables(12, 3)
    bad = D.copy(); bad[12, 3] = 11
    assert ex.execute_hsm(bad, 12, 3).forwards > C[12, 3]


# ---- tie-break: smallest y (Algorithm 1 scans upward with a strict comparison) ---------------
def test_leftmost_tie_break():
    C, D = dp.hsm_tables(60, 12)
    for m in range(2, 13):
        for t in range(m + 1, 61):
            q = [y + C[y, m] + C[t - y, m - 1] for y in range(1, t)]
            first = 1 + min(range(len(q)), key=lambda k: (q[k], k))
            assert D[t, m] == first
    Ci, Di = dp.ism_tables(60, 12)
    for m in range(1, 13):
        for t in range(1, 61):
            q = [y + Ci[y - 1, m] + Ci[t - y, m - 1] for y in range(1, t + 1)]
            assert Di[t, m] == 1 + min(range(len(q)), key=lambda k: (q[k], k))


@pytest.mark.parametrize("alpha,beta", [(4, 3), (4, 4), (2, 1), (6, 2)])
def test_msm_splits_and_choice_rederived_by_scanning(alpha, beta):
    """D1, D2, C1, C2 and H of BPTT-MSM re-derived cell by cell in plain Python from the finished
    cost table (eq. 6-10): smallest minimising y for each kind of push, the hidden push on a tie."""
    T, M = 40, 24
    C, C1, C2, D1, D2, H = dp.msm_tables(T, M, alpha, beta)
    INF = dp.INF

    def c(t, m):
        return INF if m < 0 else int(C[t, m])

    for m in range(2, M + 1):
        for t in range(2, T + 1):
            q1 = [y + c(y, m) + c(t - y, m - 1) for y in range(1, t)]
            q2 = [y + c(y - 1, m) + c(t - y, m - (beta if y == 1 else alpha)) for y in range(1, t + 1)]
            b1, b2 = min(q1), min(q2)
            if b1 < INF:
                assert C1[t, m] == b1 and D1[t, m] == 1 + q1.index(b1)
            else:
                assert C1[t, m] >= INF
            if b2 < INF:
                assert C2[t, m] == b2 and D2[t, m] == 1 + q2.index(b2)
            else:
                assert C2[t, m] >= INF
            if min(b1, b2) < INF:
                assert C[t, m] == min(b1, b2)
                assert H[t, m] == (1 if b1 <= b2 else 2)
            else:
                assert H[t, m] == 0


def test_small_cases_quoted_in_the_paper():
    """Fig. 3 shows (t=4, m=4) and (t=10, m=4); the appendix checks (t=3, m=2) and (t=3, m=3)
    against the bound numerically."""
    C, D = dp.hsm_tables(10, 4)
    assert C[4, 4] == 7 and D[4, 4] == 1                 # 2t - 1
    assert C[3, 3] == 5 and C[3, 2] == 5                 # D = 1: 1 + C(1,2) + C(2,1) = 1 + 1 + 3
    assert C[3, 2] <= 2 * 3 ** 1.5 and C[3, 3] <= 3 * 3 ** (4 / 3)
    assert C[10, 4] <= 4 * 10                            # 10 <= 4^3/3!, so a = 3 and C <= (a+1) t
