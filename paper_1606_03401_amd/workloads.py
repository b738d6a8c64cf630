"""Seeded synthetic LSTM workloads.

This module holds the named workload shapes and the seeded random input generators that both
the CPU oracle's tests and the HIP path's tests/benchmarks consume.  It contains none of the
method's arithmetic (no LSTM step, no cost recursion): only shapes and random draws.

The workloads stand in for the paper's single timing experiment (Discussion section: an LSTM
with a fixed batch, timed for one combined forward+backward gradient step as a function of the
sequence length under several slot budgets); the paper uses no public dataset.

Draw order for every workload (numpy ``default_rng(seed)``): ``W_ih, W_hh, x, dy``.
Weights are U(-1/sqrt(H), 1/sqrt(H)); the bias, h0 and c0 are zero; x ~ N(0, 1); the upstream
gradient dy ~ N(0, variance 0.01) (standard deviation 0.1) on the steps that carry a loss.
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np

KIND_HSM, KIND_ISM, KIND_MSM = 0, 1, 2
GEMM_FP32, GEMM_BF16 = 0, 1
LOSS_EXTERNAL_DY, LOSS_HALF_SUM_H2 = 0, 1
CELL_LSTM, CELL_GRU = 0, 1


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    B: int
    I: int
    H: int
    t: int
    kind: int
    m: int                       # budget: slots (HSM/ISM) or hidden-state units (MSM)
    gemm_dtype: int              # GEMM_FP32 or GEMM_BF16 operands; accumulation is always fp32
    loss: int                    # LOSS_EXTERNAL_DY: dy array; LOSS_HALF_SUM_H2: dy_t = h_t
    dy_first_step: int = 1       # dy covers steps dy_first_step..t (1-based); zero before
    alpha: int = 4               # MSM: units of an internal state with unknown input state
    beta: int = 3                # MSM: units of an internal state whose input state is known
    seed: int = 0
    cell: int = 0                # CELL_LSTM or CELL_GRU

    def scaled(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The five named configurations (seed = configuration number).
CONFIGS = {
    "cfg1": Workload("cfg1", B=4, I=16, H=32, t=20, kind=KIND_HSM, m=4,
                     gemm_dtype=GEMM_FP32, loss=LOSS_HALF_SUM_H2, seed=1),
    "cfg2": Workload("cfg2", B=64, I=256, H=1024, t=1000, kind=KIND_HSM, m=50,
                     gemm_dtype=GEMM_BF16, loss=LOSS_EXTERNAL_DY, seed=2),
    "cfg3": Workload("cfg3", B=128, I=512, H=2048, t=1000, kind=KIND_ISM, m=100,
                     gemm_dtype=GEMM_BF16, loss=LOSS_EXTERNAL_DY, seed=3),
    "cfg4": Workload("cfg4", B=256, I=128, H=512, t=10000, kind=KIND_HSM, m=100,
                     gemm_dtype=GEMM_BF16, loss=LOSS_EXTERNAL_DY, dy_first_step=9901, seed=4),
    "cfg5": Workload("cfg5", B=32, I=1024, H=4096, t=1000, kind=KIND_MSM, m=50,
                     gemm_dtype=GEMM_BF16, loss=LOSS_EXTERNAL_DY, seed=5),
}
CFG5_BUDGET_SWEEP = (1000, 250, 50, 31, 2)      # t, t/4, t/20, floor(sqrt(t)), 2 units
CFG5_BYTE_CAP = 4_000_000_000                   # "4 GB of HBM for checkpoints"


@dataclasses.dataclass
class Inputs:
    W_ih: np.ndarray            # [4H, I]  float32, gate order i, f, g, o along the 4H axis (GRU: [3H, I], r, z, n)
    W_hh: np.ndarray            # [4H, H]  float32
    b: np.ndarray               # [4H]     float32
    x: np.ndarray               # [t, B, I] float32
    dy: Optional[np.ndarray]    # [t - dy_first_step + 1, B, H] float32, or None (built-in loss)
    h0: np.ndarray              # [B, H]   float32
    c0: np.ndarray              # [B, H]   float32


def make_inputs(w: Workload, *, nonzero_state: bool = False, nonzero_bias: bool = False) -> Inputs:
    """Draw the inputs of workload ``w``.  The two flags give non-zero h0/c0 or bias for tests
    that must exercise those paths; the named configurations keep them zero."""
    rng = np.random.default_rng(w.seed)
    k = 1.0 / np.sqrt(w.H)
    G = 3 if w.cell == CELL_GRU else 4          # gate blocks of the weight matrices
    NB = 6 if w.cell == CELL_GRU else 4         # bias blocks: the GRU carries b_ih and b_hh
    W_ih = rng.uniform(-k, k, size=(G * w.H, w.I)).astype(np.float32)
    W_hh = rng.uniform(-k, k, size=(G * w.H, w.H)).astype(np.float32)
    x = rng.standard_normal(size=(w.t, w.B, w.I), dtype=np.float32)
    dy = None
    if w.loss == LOSS_EXTERNAL_DY:
        n = w.t - w.dy_first_step + 1
        dy = (0.1 * rng.standard_normal(size=(n, w.B, w.H), dtype=np.float32)).astype(np.float32)
    if nonzero_state:
        h0 = (0.5 * rng.standard_normal(size=(w.B, w.H), dtype=np.float32)).astype(np.float32)
        c0 = (0.5 * rng.standard_normal(size=(w.B, w.H), dtype=np.float32)).astype(np.float32)
    else:
        h0 = np.zeros((w.B, w.H), np.float32)
        c0 = np.zeros((w.B, w.H), np.float32)
    if nonzero_bias:
        b = rng.uniform(-k, k, size=(NB * w.H,)).astype(np.float32)
    else:
        b = np.zeros((NB * w.H,), np.float32)
    return Inputs(W_ih, W_hh, b, x, dy, h0, c0)
