"""CPU ORACLE (test infrastructure, not product code) -- store-everything back-propagation through
a chain of dense tanh layers of differing widths, in float64.

The appendix "Generalizing to deep feed-forward networks" applies the checkpointing policy to a
chain whose layers differ in cost and size; what such a chain *computes* is ordinary
back-propagation, which recomputation does not change.  This is that plain definition, for
    y_i = tanh(y_{i-1} W_i^T + b_i),   i = 1 .. n,   y_0 = x0,
with the loss gradient dy = dL/dy_n handed in:
    dz_i = g_i * (1 - y_i^2),  dW_i = dz_i^T y_{i-1},  db_i = sum over the batch of dz_i,
    g_{i-1} = dz_i W_i,  g_n = dy,  dx0 = g_0.
numpy matmul is the only library step.  Only tests and the benchmark's CPU leg may import this.
"""
from __future__ import annotations

import dataclasses
from typing import List, Sequence

import numpy as np


@dataclasses.dataclass
class ChainGrads:
    dW: List[np.ndarray]
    db: List[np.ndarray]
    dx0: np.ndarray
    y: np.ndarray           # output of the last layer


def chain_forward(W: Sequence[np.ndarray], b: Sequence[np.ndarray], x0: np.ndarray) -> List[np.ndarray]:
    """All activations y_0 .. y_n."""
    ys = [np.asarray(x0, np.float64)]
    for Wi, bi in zip(W, b):
        ys.append(np.tanh(ys[-1] @ np.asarray(Wi, np.float64).T + np.asarray(bi, np.float64)))
    return ys


def chain_backprop(W: Sequence[np.ndarray], b: Sequence[np.ndarray], x0: np.ndarray, dy: np.ndarray) -> ChainGrads:
    ys = chain_forward(W, b, x0)
    n = len(W)
    g = np.asarray(dy, np.float64)
    dW, db = [None] * n, [None] * n
    for i in range(n, 0, -1):
        dz = g * (1.0 - ys[i] * ys[i])
        dW[i - 1] = dz.T @ ys[i - 1]
        db[i - 1] = dz.sum(axis=0)
        g = dz @ np.asarray(W[i - 1], np.float64)
    return ChainGrads(dW, db, g, ys[n])
