"""CPU ORACLE (test infrastructure, not product code) -- the two strategies of Chen et al. that the
paper compares against (Section 2, "Chen's sqrt(t) algorithm" and "Chen's recursive algorithm"),
executed step by step on the abstract machine of `executor_sim`, plus the two quantities of the
numerical comparison in Section 4.3.

Both strategies are written here directly from their prose definitions -- which states are
memorised and when -- and not as decisions of the divide-and-conquer protocol, so that the
planner's way of expressing them as a policy (Section 4.2: every such strategy is a, possibly
sub-optimal, policy of BPTT-MSM) can be checked against an independent execution: the forward
count, the peak memory and the order of the backward steps must agree.

Readings (the paper gives the strategies in two sentences each):
  * sqrt(t): the sequence is cut into k = ceil(sqrt(t)) parts of length L = ceil(t / k) (the last
    one shorter).  The first pass memorises the hidden state at every cut; each part is then
    (re)run from its cut with every internal state memorised.  An internal state is stored
    without its input hidden state (beta units): that state is the entry below it on the stack.
    The last step of a part is back-propagated straight from the working core.
  * recursive, parameter k >= 1: a sub-sequence of length n is cut into min(k + 1, n) parts of
    length ceil(n / parts) by memorising k hidden states (k = 1: one state in the middle, which
    gives the log2(t) memory the paper quotes); each part is treated the same way until its
    length is 1.  Only hidden states are memorised.
  * Memory is counted as in BPTT-MSM: in units of one hidden state, the start state h_0 included.
"""
from __future__ import annotations

import math

from .executor_sim import Machine, Trace, _trace
from .policy_dp import msm_tables


def _ceil_div(a: int, b: int) -> int:
    return -(-a // b)


def chen_sqrt_segments(t: int):
    """(number of parts, length of every part but the last, length of the last part)."""
    k = math.isqrt(t - 1) + 1 if t > 1 else 1          # ceil(sqrt(t))
    L = _ceil_div(t, k)
    nseg = _ceil_div(t, L)
    return nseg, L, t - L * (nseg - 1)


def execute_chen_sqrt(t: int, beta: int, capacity: int = 1 << 60) -> Trace:
    nseg, L, last = chen_sqrt_segments(t)
    mc = Machine(t, capacity=capacity, start_units=1)
    for _ in range(nseg - 1):                           # first pass: one hidden state per cut
        for i in range(L):
            mc.forward('top' if i == 0 else 'core')
        mc.push_hidden()
    for seg in range(nseg - 1, -1, -1):
        n = last if seg == nseg - 1 else L
        for i in range(n):                              # run the part, keeping its internal states
            mc.forward('top')
            if i < n - 1:
                mc.push_internal(beta, with_input_state=False)
        mc.backward('core')
        for _ in range(n - 1):
            mc.backward('top')
            mc.pop()
        if seg > 0:
            mc.pop()                                    # the cut this part started from
    return _trace(mc)


def _recursive(mc: Machine, n: int, k: int) -> None:
    if n == 0:
        return
    if n == 1:
        mc.forward('top')
        mc.backward('core')
        return
    parts = min(k + 1, n)
    L = _ceil_div(n, parts)
    ncut = _ceil_div(n, L) - 1
    for _ in range(ncut):
        for i in range(L):
            mc.forward('top' if i == 0 else 'core')
        mc.push_hidden()
    for seg in range(ncut, -1, -1):
        _recursive(mc, n - L * ncut if seg == ncut else L, k)
        if seg > 0:
            mc.pop()


def execute_chen_recursive(t: int, k: int, capacity: int = 1 << 60) -> Trace:
    if k < 1:
        raise ValueError("k must be >= 1")
    mc = Machine(t, capacity=capacity, start_units=1)
    _recursive(mc, t, k)
    return _trace(mc)


# ---- Section 4.3: BPTT-MSM against the sqrt(t) strategy ---------------------------------------
def chen_sqrt_memory(t: int, beta: int) -> float:
    """Memory the paper assigns to the sqrt(t) strategy: sqrt(t) hidden states plus sqrt(t)
    internal states without their input states, sqrt(t) * (1 + beta) units."""
    return math.sqrt(t) * (1 + beta)


def msm_memory_for_cost(t: int, beta: int, cost_per_step: float = 2.0):
    """Smallest budget m (units) with C(t, m) <= cost_per_step * t for alpha = beta + 1, and the
    ratio of that m to sqrt(t) * (1 + beta)  (left panel of the comparison figure)."""
    ref = chen_sqrt_memory(t, beta)
    m_max = max(int(math.ceil(ref)) + 1, 2)
    while True:
        C = msm_tables(t, m_max, beta + 1, beta)[0]
        ok = [m for m in range(1, m_max + 1) if C[t, m] <= cost_per_step * t]
        if ok:
            return ok[0], ok[0] / ref
        m_max *= 2


def msm_cost_at_chen_memory(t: int, beta: int) -> float:
    """C(t, m) / t of BPTT-MSM at m = floor(sqrt(t) * (1 + beta)) units, alpha = beta + 1
    (right panel of the comparison figure)."""
    m = int(math.floor(chen_sqrt_memory(t, beta)))
    C = msm_tables(t, m, beta + 1, beta)[0]
    return C[t, m] / t
