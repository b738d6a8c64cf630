"""CPU ORACLE (test infrastructure, not product code) -- the checkpoint policy for a linear chain
of non-homogeneous layers (appendix "Generalizing to deep feed-forward networks").

Layers i = 1..n have a forward cost u_i, an output ("hidden state") of s_i memory units and need
p_i units of working memory while their forward or backward operation runs.  C(t, m, x) is the
cost, in forward cost units, of back-propagating through the t layers x+1 .. x+t when the input
of layer x+1 is available and m units are free.  The appendix's equations, in its notation:

    U(x, y) = u_{x+1} + ... + u_{x+y}                 forward over y layers above the cut x
    P(x, y) = max(p_{x+1}, ..., p_{x+y})              working memory that takes; infeasible if > m
    Q(t, m, y, x) = U(x, y) + K(x, y, m) + C(t - y, m - s_{x+y}, x + y) + C(y, m, x),  1 <= y < t
    C(t, m, x) = min_y Q(t, m, y, x),   D(t, m, x) = the smallest minimising y

Readings (the appendix's boundary conditions are printed inconsistently):
  * C(0, m, x) = 0.  C(1, m, x) = u_{x+1} if p_{x+1} <= m, else infinite: the layer is run forward
    and back-propagated on the working memory.
  * "When no extra memory is left" the sub-chain is processed without memorising anything:
    before each backward step the layers are re-run from the sub-chain's input, which costs
    U(x, t) + U(x, t-1) + ... + U(x, 1) (the appendix's sum of (t - i + 1) u_i) and needs
    P(x, t) <= m.  That procedure is admitted at every node, not only at m = 0 (a state may simply
    be too large to memorise although some memory is left); D = 0 records it.  A tie between it and
    a memorisation goes to the memorisation.
  * A memorisation must fit: m - s_{x+y} >= 0; K makes the forward run to y infeasible when its
    working memory does not fit.  The right part then runs with m - s_{x+y} units.
  * The network's input is always available and not counted (as the appendix assumes).
  * With u = 1, s = 1, p = 0 everywhere this is BPTT-HSM with the start state outside the budget:
    C(t, m, 0) = C_HSM(t, m + 1).

`chain_tables` fills the recursion by memoised recursion, cell by cell.  `ChainMachine` executes a
policy symbolically (stack of memorised states, working memory, cost, backward order) and
`brute_force_chain` enumerates every policy tree of a tiny chain on it.
"""
from __future__ import annotations

import functools
from typing import List, Optional, Sequence, Tuple

INF = 1 << 60


class Chain:
    def __init__(self, u: Sequence[int], s: Sequence[int], p: Sequence[int]):
        assert len(u) == len(s) == len(p) and len(u) >= 1
        assert all(c >= 1 for c in u) and all(v >= 1 for v in s) and all(v >= 0 for v in p)
        self.n = len(u)
        self.u, self.s, self.p = list(u), list(s), list(p)

    def U(self, x: int, y: int) -> int:
        return sum(self.u[x:x + y])

    def P(self, x: int, y: int) -> int:
        return max(self.p[x:x + y])


def chain_tables(chain: Chain, m_max: int):
    """Returns (C, D): functions of (t, m, x) for 0 <= t, x + t <= n, 0 <= m <= m_max."""

    @functools.lru_cache(maxsize=None)
    def solve(t: int, m: int, x: int) -> Tuple[int, int]:
        if m < 0:
            return INF, 0
        if t == 0:
            return 0, 0
        if t == 1:
            return (chain.u[x], 0) if chain.p[x] <= m else (INF, 0)
        best, arg = INF, 0
        if chain.P(x, t) <= m:                       # no memorisation: re-run from the input each time
            best = sum(chain.U(x, k) for k in range(1, t + 1))
        for y in range(1, t):
            if chain.P(x, y) > m or m - chain.s[x + y - 1] < 0:
                continue
            right = solve(t - y, m - chain.s[x + y - 1], x + y)[0]
            left = solve(y, m, x)[0]
            if right >= INF or left >= INF:
                continue
            q = chain.U(x, y) + right + left
            if q < best or (q == best and arg == 0):
                best, arg = q, y
        return best, arg

    def C(t, m, x):
        return solve(t, m, x)[0]

    def D(t, m, x):
        return solve(t, m, x)[1]

    assert m_max >= 0
    return C, D


class ChainMachineError(AssertionError):
    pass


class ChainMachine:
    """Abstract machine for a chain: memorised outputs on a stack with a unit budget, the working
    memory of the layer being run counted against the same budget."""

    def __init__(self, chain: Chain, m: int):
        self.chain, self.m = chain, m
        self.stack: List[int] = []        # positions (number of layers below) of memorised outputs
        self.used = 0
        self.peak = 0
        self.cost = 0
        self.next_backward = chain.n
        self.backward_order: List[int] = []

    def _work(self, layer: int) -> None:   # layer is 1-based
        need = self.used + self.chain.p[layer - 1]
        if need > self.m:
            raise ChainMachineError(f"layer {layer} needs {need} units, {self.m} available")
        self.peak = max(self.peak, need)

    def forward_run(self, x: int, y: int) -> None:
        """Forward over layers x+1 .. x+y from the state at position x (the stack top or the input)."""
        top = self.stack[-1] if self.stack else 0
        if x != top:
            raise ChainMachineError(f"state at position {x} is not available (top is {top})")
        for layer in range(x + 1, x + y + 1):
            self._work(layer)
            self.cost += self.chain.u[layer - 1]

    def push(self, position: int) -> None:
        size = self.chain.s[position - 1]
        if self.used + size > self.m:
            raise ChainMachineError("memorised state does not fit")
        self.stack.append(position)
        self.used += size
        self.peak = max(self.peak, self.used)

    def pop(self) -> None:
        self.used -= self.chain.s[self.stack.pop() - 1]

    def backward(self, layer: int) -> None:
        if layer != self.next_backward:
            raise ChainMachineError(f"backward of layer {layer}, expected {self.next_backward}")
        self._work(layer)
        self.backward_order.append(layer)
        self.next_backward -= 1


def _execute(mc: ChainMachine, policy, t: int, m: int, x: int) -> None:
    """policy(t, m, x) -> y (0 = no memorisation).  Mirrors the appendix's last paragraph."""
    if t == 0:
        return
    if t == 1:
        mc.forward_run(x, 1)
        mc.backward(x + 1)
        return
    y = policy(t, m, x)
    if y == 0:
        for k in range(t, 0, -1):
            mc.forward_run(x, k)
            mc.backward(x + k)
        return
    if not 1 <= y < t:
        raise ChainMachineError("split out of range")
    mc.forward_run(x, y)
    mc.push(x + y)
    _execute(mc, policy, t - y, m - mc.chain.s[x + y - 1], x + y)
    mc.pop()
    _execute(mc, policy, y, m, x)


def execute_chain(chain: Chain, m: int, D) -> ChainMachine:
    mc = ChainMachine(chain, m)
    _execute(mc, D, chain.n, m, 0)
    if mc.next_backward != 0 or mc.stack:
        raise ChainMachineError("incomplete run")
    return mc


def brute_force_chain(chain: Chain, m: int) -> Optional[int]:
    """Cheapest cost over every policy tree (every y, or no memorisation, at every node), each run
    on the machine; None if no policy fits."""

    def trees(t, x):
        if t <= 1:
            yield None
            return
        yield (0, None, None)
        for y in range(1, t):
            for r in trees(t - y, x + y):
                for l in trees(y, x):
                    yield (y, r, l)

    best = None
    for tree in trees(chain.n, 0):
        pending = [tree]

        def policy(t, mm, x):
            node = pending.pop()
            y, r, l = node
            for sub in (l, r):
                if sub is not None:
                    pending.append(sub)
            return y
        mc = ChainMachine(chain, m)
        try:
            _execute(mc, policy, chain.n, m, 0)
        except ChainMachineError:
            continue
        best = mc.cost if best is None else min(best, mc.cost)
    return best
