"""Pins for the oracle of the non-homogeneous chain program (appendix "Generalizing to deep
feed-forward networks"): reduction to BPTT-HSM, brute force over every policy of tiny chains,
closed forms at the two memory extremes, and execution of the optimal policy on the machine."""
import itertools
import random

import pytest

from oracle import chain_dp as cd
from oracle import policy_dp as dp


def test_homogeneous_chain_is_hsm_with_the_start_state_outside_the_budget():
    n, M = 24, 12
    chain = cd.Chain([1] * n, [1] * n, [0] * n)
    C, D = cd.chain_tables(chain, M)
    Ch, Dh = dp.hsm_tables(n, M + 1)
    for t in range(1, n + 1):
        for m in range(0, M + 1):
            for x in (0, 3, n - t):
                if x + t <= n:
                    assert C(t, m, x) == Ch[t, m + 1], (t, m, x)
    # the policy too, wherever HSM's recursion takes a decision (t > 1 and at least one spare unit)
    for t in range(2, n + 1):
        for m in range(1, M + 1):
            assert D(t, m, 0) == Dh[t, m + 1], (t, m)
    assert D(5, 0, 0) == 0                      # nothing can be memorised: re-run from the input


def test_memory_extremes():
    u = [3, 1, 4, 1, 5, 9, 2, 6]
    s = [2, 1, 3, 1, 2, 2, 1, 4]
    p = [1, 2, 1, 3, 1, 2, 1, 1]
    chain = cd.Chain(u, s, p)
    n = len(u)
    C, D = cd.chain_tables(chain, 64)
    # working memory only (every layer needs all of it, so nothing can be memorised): every
    # backward step re-runs the chain from the input
    tight = cd.Chain(u, s, [3] * n)
    Ct, Dt = cd.chain_tables(tight, 3)
    assert Ct(n, 3, 0) == sum((n - i) * u[i] for i in range(n)) and Dt(n, 3, 0) == 0
    m0 = max(p)
    assert C(n, m0 - 1, 0) >= cd.INF            # a layer cannot run at all
    assert C(n, m0, 0) <= sum((n - i) * u[i] for i in range(n))
    # plentiful memory: one pass memorising everything, then every layer but the last once more
    big = sum(s) + max(p)
    assert C(n, big, 0) == 2 * sum(u) - u[-1]
    # monotone in memory, and never below one forward pass plus the re-runs that cannot be avoided
    prev = cd.INF
    for m in range(m0, big + 1):
        c = C(n, m, 0)
        assert c <= prev
        assert c >= 2 * sum(u) - u[-1]
        prev = c


@pytest.mark.parametrize("seed", range(6))
def test_brute_force_over_every_policy(seed):
    rng = random.Random(seed)
    n = rng.choice([3, 4, 5, 6])
    chain = cd.Chain([rng.randint(1, 5) for _ in range(n)], [rng.randint(1, 3) for _ in range(n)],
                     [rng.randint(0, 3) for _ in range(n)])
    for m in range(0, sum(chain.s) + max(chain.p) + 1):
        C, D = cd.chain_tables(chain, m)
        best = cd.brute_force_chain(chain, m)
        if best is None:
            assert C(n, m, 0) >= cd.INF, (chain.u, chain.s, chain.p, m)
        else:
            assert C(n, m, 0) == best, (chain.u, chain.s, chain.p, m)


@pytest.mark.parametrize("seed", range(4))
def test_optimal_policy_runs_within_budget_at_the_tabulated_cost(seed):
    rng = random.Random(100 + seed)
    n = 30
    chain = cd.Chain([rng.randint(1, 9) for _ in range(n)], [rng.randint(1, 4) for _ in range(n)],
                     [rng.randint(0, 5) for _ in range(n)])
    for m in (max(chain.p), max(chain.p) + 3, 12, 25, 200):
        C, D = cd.chain_tables(chain, m)
        if C(n, m, 0) >= cd.INF:
            continue
        mc = cd.execute_chain(chain, m, D)
        assert mc.cost == C(n, m, 0)
        assert mc.peak <= m
        assert mc.backward_order == list(range(n, 0, -1))


def test_machine_rejects_illegal_programs():
    chain = cd.Chain([1, 1, 1], [2, 2, 2], [1, 1, 1])
    mc = cd.ChainMachine(chain, 2)
    mc.forward_run(0, 2)
    mc.push(2)                                   # fills the budget ...
    with pytest.raises(AssertionError):
        mc.forward_run(2, 1)                     # ... so the next layer has no working memory left
    mc = cd.ChainMachine(chain, 1)
    with pytest.raises(AssertionError):
        mc.push(1)                               # a 2-unit state into 1 unit
    mc = cd.ChainMachine(chain, 5)
    mc.forward_run(0, 3)
    with pytest.raises(AssertionError):
        mc.backward(2)                           # out of order
    with pytest.raises(AssertionError):
        mc.forward_run(1, 1)                     # the state at position 1 was never memorised
