"""Caller-supplied policies and Chen et al.'s two strategies as plans: the schedule is replayed
symbolically and its cost, memory and backward order are compared with the oracle's direct
execution of the same strategy (Section 2, Section 4.2)."""
import pytest

from oracle import chen
from oracle import executor_sim as ex
from oracle import policy_dp as dp
from paper_1606_03401_amd import binding as mb
from test_planner import check_schedule


@pytest.mark.parametrize("t", [1, 2, 3, 4, 10, 16, 17, 99, 100, 1000, 3000])
@pytest.mark.parametrize("beta,alpha", [(3, 4), (4, 5)])
def test_chen_sqrt_plan_matches_the_direct_execution(t, beta, alpha):
    plan = mb.mebptt_plan_chen_sqrt(t, alpha, beta)
    tr = chen.execute_chen_sqrt(t, beta)
    assert plan.kind == mb.MSM and plan.t == t
    assert plan.forward_ops == tr.forwards
    assert plan.m == plan.peak == tr.peak
    assert check_schedule(plan, t, plan.m, mb.MSM, exact_peak=(alpha == 4)) == tr.forwards
    assert plan.cost() is None and plan.split(1) is None and plan.choice() is None


@pytest.mark.parametrize("t", [1, 2, 3, 7, 64, 100, 257, 1000])
@pytest.mark.parametrize("k", [1, 2, 3, 9, 2000])
def test_chen_recursive_plan_matches_the_direct_execution(t, k):
    plan = mb.mebptt_plan_chen_recursive(t, k)
    tr = chen.execute_chen_recursive(t, k)
    assert plan.forward_ops == tr.forwards
    assert plan.m == plan.peak == tr.peak
    assert check_schedule(plan, t, plan.m, mb.MSM) == tr.forwards


def test_chen_long_sequence_is_depth_safe():
    plan = mb.mebptt_plan_chen_recursive(10000, 10000)     # one part per step: t - 1 memorised states
    assert plan.m == 10000 and plan.forward_ops == 2 * 10000 - 1
    plan = mb.mebptt_plan_chen_sqrt(10000)
    assert plan.forward_ops == 2 * 10000 - 100 and plan.m == 100 + 99 * 3


def _decisions_from_tables(D1, D2, H, t, m, alpha, beta):
    """The optimal MSM policy as a decision list, in the order the execution procedure asks."""
    out = []

    def node(tt, mm):
        if tt <= 1 or mm == 1:
            return
        if H[tt, mm] == 1:
            y = int(D1[tt, mm])
            out.append((mb.STORE_HIDDEN, y))
            node(tt - y, mm - 1)
            node(y, mm)
        else:
            y = int(D2[tt, mm])
            out.append((mb.STORE_INTERNAL, y))
            node(tt - y, mm - (beta if y == 1 else alpha))
            node(y - 1, mm)
    node(t, m)
    return out


@pytest.mark.parametrize("t,m", [(2, 2), (9, 4), (20, 13), (40, 7), (100, 30)])
def test_the_optimal_policy_as_a_decision_list_reproduces_the_table_plan(t, m):
    alpha, beta = 4, 3
    C, C1, C2, D1, D2, H = dp.msm_tables(t, m, alpha, beta)
    dec = _decisions_from_tables(D1, D2, H, t, m, alpha, beta)
    a = mb.mebptt_plan_from_policy(t, m, dec, alpha, beta)
    b = mb.mebptt_plan(t, m, mb.MSM, alpha, beta)
    assert a.forward_ops == b.forward_ops == C[t, m]
    assert (a.schedule() == b.schedule()).all()
    check_schedule(a, t, m, mb.MSM, exact_peak=False)


def test_a_hand_written_policy():
    # t = 4, m = 3: memorise the hidden state after 2 steps; each half then has 2 steps and one
    # spare unit for the right half, none for the left
    plan = mb.mebptt_plan_from_policy(4, 3, [(mb.STORE_HIDDEN, 2), (mb.STORE_HIDDEN, 1), (mb.STORE_HIDDEN, 1)])
    # 2 (to the cut) + right half (1 + 1 + 1) + left half (1 + 1 + 1)
    assert plan.forward_ops == 8
    tr_best = ex.brute_force_hsm(4, 3)
    assert tr_best <= plan.forward_ops
    check_schedule(plan, 4, 3, mb.MSM, exact_peak=False)


def test_policy_errors():
    H, I = mb.STORE_HIDDEN, mb.STORE_INTERNAL
    cases = [
        ((4, 3, [(H, 2)]), mb.EINVAL),                           # too few decisions
        ((4, 3, [(H, 2), (H, 1), (H, 1), (H, 1)]), mb.EINVAL),   # too many
        ((4, 3, [(H, 4), (H, 1), (H, 1)]), mb.EINVAL),           # hidden y must be < t'
        ((4, 3, [(I, 5)]), mb.EINVAL),                           # internal y must be <= t'
        ((4, 3, [(7, 1)]), mb.EINVAL),                           # unknown store
        ((4, 3, [(I, 2)]), mb.EINFEASIBLE),                      # alpha = 4 units do not fit into 3
        ((4, 0, []), mb.EINVAL),
        ((0, 3, []), mb.EINVAL),
    ]
    for (t, m, dec), code in cases:
        with pytest.raises(mb.MebpttError) as e:
            mb.mebptt_plan_from_policy(t, m, dec)
        assert e.value.code == code, (t, m, dec, str(e.value))
    with pytest.raises(mb.MebpttError):
        mb.mebptt_plan_from_policy(4, 3, [(H, 2), (H, 1), (H, 1)], alpha=3, beta=2)   # no LSTM schedule
    with pytest.raises(mb.MebpttError):
        mb.mebptt_plan_chen_recursive(10, 0)
    with pytest.raises(mb.MebpttError):
        mb.mebptt_plan_chen_sqrt(0)


@pytest.mark.parametrize("t", [50, 100, 400])
def test_msm_optimum_is_not_worse_than_chen_at_the_same_memory(t):
    # Section 4.2, checked on the library's own tables
    s = mb.mebptt_plan_chen_sqrt(t)
    opt = mb.mebptt_plan(t, s.m, mb.MSM)
    assert opt.forward_ops <= s.forward_ops
    r = mb.mebptt_plan_chen_recursive(t, 2)
    assert mb.mebptt_plan(t, r.m, mb.MSM).forward_ops <= r.forward_ops
