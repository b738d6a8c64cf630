"""The non-homogeneous chain planner (appendix): tables cell for cell against the oracle, and the
flattened schedule replayed on a symbolic memory (every operand where the entry says it is,
backward order n..1, memorised outputs plus working memory within the budget)."""
import random
import time

import numpy as np
import pytest

from oracle import chain_dp as cd
from oracle import policy_dp as dp
from paper_1606_03401_amd import binding as mb


def replay(plan, layers, m):
    u = [l[0] for l in layers]
    s = [l[1] for l in layers]
    p = [l[2] for l in layers]
    n = len(layers)
    mem = {}                 # unit offset -> (position, size)
    working = None           # position of the output held in working memory (the last layer run)
    working_in = None        # position of that layer's input, when the run covered it (count > 1)
    used = 0
    peak = 0
    cost = 0
    next_bwd = n

    def state_at(loc):
        if loc == mb.CHAIN_INPUT:
            return 0
        if loc == mb.CHAIN_WORKING:
            assert working is not None
            return working
        assert loc in mem, f"nothing memorised at unit {loc}"
        return mem[loc][0]

    for op in plan.schedule():
        layer, count = int(op["layer"]), int(op["count"])
        # memorised outputs above the one being read have been dropped (LIFO): drop them here
        if op["op"] == mb.CHAIN_FORWARD:
            src = int(op["src"])
            assert state_at(src) == layer - 1, (op, state_at(src))
            if src != mb.CHAIN_WORKING:
                limit = -1 if src == mb.CHAIN_INPUT else src
                for off in [o for o in mem if o > limit]:
                    used -= mem.pop(off)[1]
            for i in range(layer, layer + count):
                peak = max(peak, used + p[i - 1])
                cost += u[i - 1]
            assert used + max(p[layer - 1:layer - 1 + count]) <= m
            pos = layer + count - 1
            working_in = pos - 1 if count > 1 else None
            if op["dst"] == mb.CHAIN_WORKING:
                working = pos
            else:
                dst = int(op["dst"])
                assert dst == used, (op, used)
                mem[dst] = (pos, s[pos - 1])
                used += s[pos - 1]
                assert used <= m
                peak = max(peak, used)
                working = pos
        else:
            assert op["op"] == mb.CHAIN_BACKWARD and layer == next_bwd
            assert working == layer, "the layer's internal state is not in working memory"
            if op["src"] == mb.CHAIN_WORKING:
                assert working_in == layer - 1
            else:
                assert state_at(int(op["src"])) == layer - 1
            assert used + p[layer - 1] <= m
            peak = max(peak, used + p[layer - 1])
            next_bwd -= 1
            working = working_in = None
    assert next_bwd == 0
    return cost, peak


def random_chain(rng, n):
    return [(rng.randint(1, 9), rng.randint(1, 4), rng.randint(0, 5)) for _ in range(n)]


@pytest.mark.parametrize("seed", range(8))
def test_tables_and_schedule_against_the_oracle(seed):
    rng = random.Random(seed)
    n = rng.choice([1, 2, 3, 7, 12, 20])
    layers = random_chain(rng, n)
    chain = cd.Chain(*zip(*layers))
    for m in sorted({max(chain.p), max(chain.p) + 1, 6, 11, 30, sum(chain.s) + max(chain.p)}):
        C, D = cd.chain_tables(chain, m)
        if C(n, m, 0) >= cd.INF:
            with pytest.raises(mb.MebpttError) as e:
                mb.mebptt_chain_plan(layers, m)
            assert e.value.code == mb.EINFEASIBLE
            continue
        plan = mb.mebptt_chain_plan(layers, m)
        for x in range(n + 1):
            for t in range(n - x + 1):
                for mm in range(m + 1):
                    want = C(t, mm, x)
                    got = plan.cost(t, mm, x)
                    assert got == (want if want < cd.INF else mb.COST_INF), (t, mm, x)
                    if want < cd.INF:
                        assert plan.split(t, mm, x) == D(t, mm, x), (t, mm, x)
        assert plan.forward_cost == C(n, m, 0)
        cost, peak = replay(plan, layers, m)
        assert cost == plan.forward_cost and peak == plan.peak and peak <= m
        assert cd.execute_chain(chain, m, D).peak == peak


def test_homogeneous_chain_reproduces_the_hsm_tables_of_the_library():
    n, m = 200, 20
    plan = mb.mebptt_chain_plan([(1, 1, 0)] * n, m)
    hsm = mb.mebptt_plan(n, m + 1, mb.HSM)
    C = hsm.cost()
    for t in (1, 2, 3, 17, 100, 200):
        for mm in (0, 1, 2, 7, 20):
            assert plan.cost(t, mm, n - t) == C[t, mm + 1]
    assert plan.forward_cost == hsm.forward_ops


def test_a_layered_network_shape():
    """A convolutional-network-like profile: early layers have large outputs and cheap
    operations, late layers small outputs and expensive ones.  The plan must fit, cost no more than
    with less memory, and reach the lower bound 2 sum(u) - u_n when everything can be memorised."""
    layers = [(1 + i // 4, max(1, 64 >> (i // 6)), max(1, 32 >> (i // 6))) for i in range(36)]
    total_u = sum(l[0] for l in layers)
    costs = []
    for m in (64, 96, 128, 256, 512, 1024):
        t0 = time.perf_counter()
        plan = mb.mebptt_chain_plan(layers, m)
        assert time.perf_counter() - t0 < 20.0
        cost, peak = replay(plan, layers, m)
        assert cost == plan.forward_cost and peak <= m
        costs.append(cost)
    assert costs == sorted(costs, reverse=True)
    assert costs[-1] == 2 * total_u - layers[-1][0]


def test_chain_errors():
    for args in (([], 4), ([(0, 1, 0)], 4), ([(1, 0, 0)], 4), ([(1, 1, -1)], 4), ([(1, 1, 0)], -1)):
        with pytest.raises(mb.MebpttError) as e:
            mb.mebptt_chain_plan(*args)
        assert e.value.code == mb.EINVAL
    with pytest.raises(mb.MebpttError) as e:
        mb.mebptt_chain_plan([(1, 1, 5)], 4)
    assert e.value.code == mb.EINFEASIBLE
    plan = mb.mebptt_chain_plan([(2, 1, 1), (3, 1, 1)], 4)
    assert plan.cost(3, 4, 0) == mb.COST_INF and plan.cost(1, 9, 0) == mb.COST_INF and plan.cost(1, -1, 0) == mb.COST_INF
