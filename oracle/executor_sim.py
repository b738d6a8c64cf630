"""CPU ORACLE (test infrastructure, not product code) -- symbolic execution of checkpoint policies.

A tiny abstract machine models what the paper's execution procedures may do: one working RNN
core that can evaluate and hold a single internal state (Section 3.1), and a LIFO stack of
memorised states whose total size may never exceed the budget (Section 3.1: states are read in
the reverse order in which they were written).  It performs no arithmetic; it counts forward
and backward operations, checks that every operation's operands really are available, that the
backward operations come in the order t, t-1, ..., 1, and tracks the peak stack occupancy.

On top of the machine:
  * `execute_hsm / execute_ism / execute_msm` run a given policy table the way Algorithm 2
    (HSM), Section 3.2's four steps (ISM) and Section 3.3's last paragraph (MSM) describe;
  * `brute_force_*` enumerate every policy of the divide-and-conquer family explicitly (every
    admissible y -- and, for MSM, both kinds of push -- at every node), run each one on the
    machine, and return the cheapest cost found.  No cost table is consulted.

Readings:
  * HSM/MSM: the start state of the sequence (h_0) sits on the stack and uses one unit of the
    budget -- only then do C(t,1) = t(t+1)/2 and "C(t,m) = 2t-1 iff m >= t" hold.
  * ISM: h_0 is a given input outside the budget; all m slots hold internal states -- only then
    does "C(t,m) = t iff m >= t" hold.
  * A budget of one unit (HSM/MSM) cannot push: the sub-sequence is processed by re-forwarding
    from the stack top before every backward step (the constant-memory procedure of Section 3).
    Algorithm 2 has no line for it; Algorithm 1 prices it as t(t+1)/2.
  * Algorithm 2's forward loop is printed as t iterations; step 1 of Section 3.1 and the leading
    term y of eq. 1 make it y iterations.
  * An internal state whose right-hand remainder is empty (y = t) is consumed by the very next
    backward operation, so it stays in the working core and takes no stack space.  (This is what
    keeps MSM's peak occupancy within m for the y = t push that C(0, 0) = 0 admits.)
  * Outputs are produced, and loss gradients fetched, when the step's internal state is
    (re)evaluated for its backward operation.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional, Tuple


class MachineError(AssertionError):
    pass


@dataclasses.dataclass
class _Entry:
    kind: str        # 'h' hidden state of `step`; 'i' internal state of `step`
    step: int
    units: int
    has_input_state: bool = True   # internal entries: is the input hidden state stored inside?


class Machine:
    """Abstract machine: a stack with a unit budget plus one working core."""

    def __init__(self, t: int, capacity: int, start_units: int):
        self.t = t
        self.capacity = capacity
        self.stack: List[_Entry] = [_Entry('h', 0, start_units)]
        self.used = start_units
        self.peak = start_units
        self.core_hidden: Optional[int] = None     # step whose hidden state the core just produced
        self.core_internal: Optional[int] = None   # step whose internal state the core holds
        self.forwards = 0
        self.backwards = 0
        self.next_backward = t
        self.backward_order: List[int] = []
        if self.used > capacity:
            raise MachineError("start state does not fit")

    # -- operand lookup ---------------------------------------------------------------------
    def _top_hidden_step(self) -> int:
        return self.stack[-1].step                 # 'h': that state; 'i': its output hidden state

    def forward(self, source: str) -> int:
        """One forward operation from the hidden state at the stack top ('top') or from the one
        the core produced last ('core').  Leaves the new step's internal state in the core."""
        if source == 'top':
            k = self._top_hidden_step()
        elif source == 'core':
            if self.core_hidden is None:
                raise MachineError("core holds no hidden state")
            k = self.core_hidden
        else:
            raise MachineError(source)
        if k + 1 > self.t:
            raise MachineError("forward past the end of the sequence")
        self.core_hidden = k + 1
        self.core_internal = k + 1
        self.forwards += 1
        return k + 1

    def push_hidden(self) -> None:
        if self.core_hidden is None:
            raise MachineError("nothing to push")
        self._push(_Entry('h', self.core_hidden, 1))

    def push_internal(self, units: int, with_input_state: bool) -> None:
        if self.core_internal is None:
            raise MachineError("no internal state to push")
        if not with_input_state and self._top_hidden_step() != self.core_internal - 1:
            raise MachineError("input hidden state is not on the stack: cannot omit it")
        self._push(_Entry('i', self.core_internal, units, with_input_state))

    def _push(self, e: _Entry) -> None:
        if self.used + e.units > self.capacity:
            raise MachineError(f"budget exceeded: {self.used}+{e.units} > {self.capacity}")
        self.stack.append(e)
        self.used += e.units
        self.peak = max(self.peak, self.used)

    def pop(self) -> None:
        if len(self.stack) <= 1:
            raise MachineError("cannot pop the start state")
        self.used -= self.stack.pop().units

    def backward(self, source: str) -> None:
        """One backward operation through the internal state in the core ('core') or in the
        stack-top entry ('top')."""
        if source == 'core':
            k = self.core_internal
        elif source == 'top':
            e = self.stack[-1]
            if e.kind != 'i':
                raise MachineError("stack top is not an internal state")
            if not e.has_input_state and self.stack[-2].step != e.step - 1:
                raise MachineError("omitted input hidden state is not below on the stack")
            k = e.step
        else:
            raise MachineError(source)
        if k is None or k != self.next_backward:
            raise MachineError(f"backward of step {k}, expected {self.next_backward}")
        self.backward_order.append(k)
        self.backwards += 1
        self.next_backward -= 1
        self.core_internal = None
        self.core_hidden = None

    def finish(self) -> None:
        if self.next_backward != 0:
            raise MachineError(f"backward sweep stopped at step {self.next_backward}")
        if len(self.stack) != 1:
            raise MachineError("stack not unwound")


# ---------------------------------------------------------------------------------------------
# shared pieces of the three procedures
def _forward_run(mc: Machine, n: int) -> None:
    """n consecutive forward operations starting from the stack top."""
    for i in range(n):
        mc.forward('top' if i == 0 else 'core')


def _constant_memory(mc: Machine, t: int) -> None:
    """Section 3, first example: before every backward step re-forward from the stored start."""
    for k in range(t, 0, -1):
        _forward_run(mc, k)
        mc.backward('core')


class Policy:
    """What to do at node (t, m): returns ('hidden', y) or ('internal', y)."""

    def __call__(self, t: int, m: int) -> Tuple[str, int]:
        raise NotImplementedError


def _exec_hsm_like(mc: Machine, policy, t: int, m: int, alpha: int, beta: int) -> None:
    """Algorithm 2 generalised to MSM (Section 3.3): the stack top is the sub-sequence's start
    state and is counted inside m."""
    if t == 0:
        return
    if t == 1:
        mc.forward('top')
        mc.backward('core')
        return
    if m == 1:
        _constant_memory(mc, t)
        return
    what, y = policy(t, m)
    if what == 'hidden':
        if not (1 <= y < t):
            raise MachineError("hidden push position out of range")
        _forward_run(mc, y)
        mc.push_hidden()
        _exec_hsm_like(mc, policy, t - y, m - 1, alpha, beta)
        mc.pop()
        _exec_hsm_like(mc, policy, y, m, alpha, beta)
    else:
        if not (1 <= y <= t):
            raise MachineError("internal push position out of range")
        units = beta if y == 1 else alpha
        if m - units < 0 or (t - y > 0 and m - units < 1):
            raise MachineError("internal push does not fit")
        _forward_run(mc, y)
        if y == t:                         # consumed at once: stays in the working core
            mc.backward('core')
        else:
            mc.push_internal(units, with_input_state=(y > 1))
            _exec_hsm_like(mc, policy, t - y, m - units, alpha, beta)
            mc.backward('top')
            mc.pop()
        _exec_hsm_like(mc, policy, y - 1, m, alpha, beta)


def _exec_ism(mc: Machine, policy, t: int, m: int) -> None:
    """Section 3.2, steps 1-4.  The start state is the stack top but is not counted in m."""
    if t == 0:
        return
    if m < 1:
        raise MachineError("no slot left")
    _what, y = policy(t, m)
    if not (1 <= y <= t):
        raise MachineError("push position out of range")
    _forward_run(mc, y)
    if y == t:
        mc.backward('core')
    else:
        mc.push_internal(1, with_input_state=True)
        _exec_ism(mc, policy, t - y, m - 1)
        mc.backward('top')
        mc.pop()
    _exec_ism(mc, policy, y - 1, m)


@dataclasses.dataclass
class Trace:
    forwards: int
    backwards: int
    peak: int
    backward_order: List[int]


def _trace(mc: Machine) -> Trace:
    mc.finish()
    return Trace(mc.forwards, mc.backwards, mc.peak, mc.backward_order)


def execute_hsm(D, t: int, m: int) -> Trace:
    mc = Machine(t, capacity=m, start_units=1)
    _exec_hsm_like(mc, lambda tt, mm: ('hidden', int(D[tt, mm])), t, m, 0, 0)
    return _trace(mc)


def execute_ism(D, t: int, m: int) -> Trace:
    mc = Machine(t, capacity=m, start_units=0)
    _exec_ism(mc, lambda tt, mm: ('internal', int(D[tt, mm])), t, m)
    return _trace(mc)


def execute_msm(D1, D2, H, t: int, m: int, alpha: int, beta: int) -> Trace:
    def policy(tt, mm):
        if H[tt, mm] == 1:
            return 'hidden', int(D1[tt, mm])
        if H[tt, mm] == 2:
            return 'internal', int(D2[tt, mm])
        raise MachineError(f"no policy at ({tt},{mm})")
    mc = Machine(t, capacity=m, start_units=1)
    _exec_hsm_like(mc, policy, t, m, alpha, beta)
    return _trace(mc)


# ---------------------------------------------------------------------------------------------
# brute force: enumerate whole policies as explicit trees, run each on the machine.
#
# A policy tree for node (t, m) is None for the nodes that need no decision (t <= 1, or m == 1 in
# the HSM/MSM protocol) and otherwise a tuple (what, y, right_subtree, left_subtree).

def _trees_hsm_like(t: int, m: int, alpha: int, beta: int, allow_internal: bool):
    if t <= 1 or m == 1:
        yield None
        return
    for y in range(1, t):
        for r in _trees_hsm_like(t - y, m - 1, alpha, beta, allow_internal):
            for l in _trees_hsm_like(y, m, alpha, beta, allow_internal):
                yield ('hidden', y, r, l)
    if allow_internal:
        for y in range(1, t + 1):
            units = beta if y == 1 else alpha
            rest = m - units
            if rest < 0 or (t - y > 0 and rest < 1):
                continue
            for r in _trees_hsm_like(t - y, rest, alpha, beta, True):
                for l in _trees_hsm_like(y - 1, m, alpha, beta, True):
                    yield ('internal', y, r, l)


def _trees_ism(t: int, m: int):
    if t == 0:
        yield None
        return
    if m < 1:
        return
    for y in range(1, t + 1):
        if t - y > 0 and m - 1 < 1:
            continue
        for r in _trees_ism(t - y, m - 1):
            for l in _trees_ism(y - 1, m):
                yield ('internal', y, r, l)


class _TreePolicy:
    """Feeds a tree to the executors: the executor asks for decisions in the same pre-order
    (node, right subtree, left subtree) in which the tree was built."""

    def __init__(self, tree):
        self.pending = [tree]

    def __call__(self, t: int, m: int):
        node = self.pending.pop()
        what, y, r, l = node
        # the executor descends right first, then left; subtrees that need no decision are None
        for sub in (l, r):
            if sub is not None:
                self.pending.append(sub)
        return what, y


def brute_force_hsm(t: int, m: int) -> int:
    best = None
    for tree in _trees_hsm_like(t, m, 0, 0, allow_internal=False):
        mc = Machine(t, capacity=m, start_units=1)
        _exec_hsm_like(mc, _TreePolicy(tree) if tree is not None else None, t, m, 0, 0)
        mc.finish()
        best = mc.forwards if best is None else min(best, mc.forwards)
    return best


def brute_force_ism(t: int, m: int) -> Optional[int]:
    best = None
    for tree in _trees_ism(t, m):
        mc = Machine(t, capacity=m, start_units=0)
        _exec_ism(mc, _TreePolicy(tree) if tree is not None else None, t, m)
        mc.finish()
        best = mc.forwards if best is None else min(best, mc.forwards)
    return best


def brute_force_msm(t: int, m: int, alpha: int, beta: int) -> int:
    best = None
    for tree in _trees_hsm_like(t, m, alpha, beta, allow_internal=True):
        mc = Machine(t, capacity=m, start_units=1)
        _exec_hsm_like(mc, _TreePolicy(tree) if tree is not None else None, t, m, alpha, beta)
        mc.finish()
        best = mc.forwards if best is None else min(best, mc.forwards)
    return best
