"""CPU ORACLE (test infrastructure, not product code) -- the checkpoint-policy dynamic programs.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package.  It
shares no code with the HIP library and never imports it.

Each function writes the recurrences of the paper out directly, cell by cell, in the paper's
notation:  C(t, m) = optimal number of forward operations for back-propagating through a
sequence of length t with m memory slots; D(t, m) = position of the first state to memorise.

  * BPTT-HSM  (Section 3.1, eq. 1-3)
        Q(t,m,y) = y + C(t-y, m-1) + C(y, m),           D = argmin over 1 <= y <  t
        base cases C(t,1) = t(t+1)/2 and C(1,m) = 1; the boundary C(t,m) = 2t-1, D = 1 for
        m >= t that the section quotes follows from the recurrence.
  * BPTT-ISM  (Section 3.2, eq. 4-5)
        Q(t,m,y) = y + C(y-1, m) + C(t-y, m-1),         D = argmin over 1 <= y <= t
        single base case C(0,m) = 0 (m >= 0); C(t,0) = infinity for t > 0.  The boundaries the
        section quotes (C(t,1) = t(t+1)/2, C(t,m) = t for m >= t) follow from the recurrence.
  * BPTT-MSM  (Sections 3.3-3.4, eq. 6-10), m in hidden-state units, integers alpha >= 2,
        1 <= beta <= alpha:
        Q1(t,m,y) = y + C(y, m)   + C(t-y, m-1),                     1 <= y <  t
        Q2(t,m,y) = y + C(y-1, m) + C(t-y, m - (beta if y == 1 else alpha)),  1 <= y <= t
        C = min(C1, C2),  H = 1 (hidden) if C1 <= C2 else 2 (internal).

Readings where the text is silent or inconsistent:
  * argmin ties go to the smallest y, which is what Algorithm 1's upward scan with a strict
    "<" comparison produces; H prefers the hidden branch on a tie (argmin over i = 1, 2 in order).
  * the appendix prints C(t,1) = t(t+2)/2 once; the body and Algorithm 1 say t(t+1)/2, which is
    also what the constant-memory procedure of Section 3 costs.  t(t+1)/2 is used.
  * MSM: Section 3.3 gives "C = infinity for m <= 0" and "C(0, m) = 0" which collide at
    (0, m <= 0), and states no t = 1 base case.  Used here: C(0,m) = 0 for m >= 0, infinity
    for m < 0; C(t,0) = infinity for t > 0; C(1,m) = 1 for m >= 1 (the HSM base case);
    C(t,1) = t(t+1)/2.  The boundary "C(t,m) = t for m >= alpha*t" is not imposed: it follows.
  * D(t,1) for t > 1 (HSM, MSM) is not defined by the paper (no push is possible with a single
    slot); it is stored as 0.  Undefined D1/D2/H cells are 0 as well.

`numpy.argmin` returns the first minimum, i.e. the smallest y; it is the only library step.
Tables are (t_max+1) x (m_max+1), row = t, column = m, int64 cost / int32 split / uint8 choice.
INF marks an infeasible cell.
"""
from __future__ import annotations

import numpy as np

INF = np.int64(1) << np.int64(60)     # "infinity": three of them still fit in int64


def _clip(c):
    return INF if c >= INF else c


def hsm_tables(t_max: int, m_max: int):
    """BPTT-HSM cost and policy tables: eq. 1-3 applied to every cell the boundary conditions of
    Section 3.1 do not fix.

    Boundaries (Section 3.1): C(t, 1) = t(t+1)/2 -- with one slot every backward step re-forwards
    from the start state -- and C(1, m) = 1, the single forward operation of a one-step sequence
    (the m >= t boundary C = 2t - 1 at t = 1).  Every other cell is the recurrence
        C(t, m) = min over 1 <= y < t of  y + C(y, m) + C(t - y, m - 1)
    with D(t, m) the smallest minimiser.  The section's second boundary, C(t, m) = 2t - 1 with
    D = 1 for all m >= t, is not imposed: it follows (y = 1 gives 1 + 1 + 2(t-1) - 1), and the tests
    pin it.  D(1, m) = 1 is the value the section's boundary assigns where no split exists."""
    assert t_max >= 1 and m_max >= 1
    C = np.full((t_max + 1, m_max + 1), INF, dtype=np.int64)
    D = np.zeros((t_max + 1, m_max + 1), dtype=np.int32)
    C[0, :] = 0                                       # empty sequence: nothing to do
    tt = np.arange(1, t_max + 1, dtype=np.int64)
    C[1:, 1] = tt * (tt + 1) // 2
    C[1, 1:] = 1
    D[1, 1:] = 1
    for m in range(2, m_max + 1):
        for t in range(2, t_max + 1):
            y = np.arange(1, t, dtype=np.int64)       # 1 <= y < t
            Q = y + C[y, m] + C[t - y, m - 1]         # eq. 1
            k = int(np.argmin(Q))                     # first minimum = smallest y
            C[t, m] = _clip(Q[k])                     # eq. 2
            D[t, m] = y[k]                            # eq. 3
    return C, D


def ism_tables(t_max: int, m_max: int):
    """BPTT-ISM cost and policy tables (Section 3.2, eq. 4-5)."""
    assert t_max >= 0 and m_max >= 0
    C = np.full((t_max + 1, m_max + 1), INF, dtype=np.int64)
    D = np.zeros((t_max + 1, m_max + 1), dtype=np.int32)
    C[0, :] = 0                                   # the single base case
    for m in range(1, m_max + 1):
        for t in range(1, t_max + 1):
            y = np.arange(1, t + 1, dtype=np.int64)   # 1 <= y <= t
            Q = y + C[y - 1, m] + C[t - y, m - 1]
            k = int(np.argmin(Q))
            if Q[k] < INF:
                C[t, m] = Q[k]
                D[t, m] = y[k]
    return C, D


def msm_tables(t_max: int, m_max: int, alpha: int, beta: int):
    """BPTT-MSM tables (Sections 3.3-3.4, eq. 6-10).  Returns C, C1, C2, D1, D2, H."""
    assert alpha >= 2 and 1 <= beta <= alpha and t_max >= 1 and m_max >= 1
    shape = (t_max + 1, m_max + 1)
    C = np.full(shape, INF, dtype=np.int64)
    C1 = np.full(shape, INF, dtype=np.int64)
    C2 = np.full(shape, INF, dtype=np.int64)
    D1 = np.zeros(shape, dtype=np.int32)
    D2 = np.zeros(shape, dtype=np.int32)
    H = np.zeros(shape, dtype=np.uint8)
    C[0, :] = 0

    def cost(tt, mm):
        """C(tt, mm) with C = infinity for mm < 0 (tt may be an index array)."""
        if mm < 0:
            return INF
        return C[tt, mm]

    for t in range(1, t_max + 1):
        C[t, 1] = t * (t + 1) // 2
    for m in range(1, m_max + 1):
        C[1, m] = 1
    for m in range(2, m_max + 1):
        for t in range(2, t_max + 1):
            # hidden-state push, eq. 6
            y = np.arange(1, t, dtype=np.int64)
            Q1 = y + C[y, m] + C[t - y, m - 1]
            k1 = int(np.argmin(Q1))
            if Q1[k1] < INF:
                C1[t, m] = Q1[k1]
                D1[t, m] = y[k1]
            # internal-state push, eq. 10 (eq. 7 when beta == alpha)
            y = np.arange(1, t + 1, dtype=np.int64)
            right = np.empty(t, dtype=np.int64)
            right[0] = cost(np.int64(t - 1), m - beta)            # y = 1 costs beta units
            if t > 1:
                right[1:] = cost(t - y[1:], m - alpha)            # y > 1 costs alpha units
            Q2 = y + C[y - 1, m] + right
            k2 = int(np.argmin(Q2))
            if Q2[k2] < INF:
                C2[t, m] = Q2[k2]
                D2[t, m] = y[k2]
            if C1[t, m] >= INF and C2[t, m] >= INF:
                continue
            if C1[t, m] <= C2[t, m]:
                C[t, m] = C1[t, m]
                H[t, m] = 1
            else:
                C[t, m] = C2[t, m]
                H[t, m] = 2
    return C, C1, C2, D1, D2, H


def theoretical_cost_ratio(C_tm: int, t: int) -> float:
    """Cost relative to store-everything BPTT when one backward costs two forwards
    (Section 3.2, last paragraph): (C + 2t) / (t + 2t)."""
    return (C_tm + 2 * t) / (3 * t)
