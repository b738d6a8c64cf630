"""CPU ORACLE (test infrastructure, not product code) -- store-everything GRU BPTT in float64.

A second RNN core behind the same checkpointing executor (the paper's method "is largely
architecture agnostic", Section 1): as for the LSTM, checkpointing changes what is recomputed,
never the result, so the oracle is ordinary back-propagation through time written out.

The core is the gated recurrent unit in the form most libraries implement (gate order r, z, n
along the 3H axis; two bias vectors, because the recurrent bias of the candidate sits inside the
reset gate's product):

    r   = sigmoid(x_t W_ir^T + b_ir + h_{t-1} W_hr^T + b_hr)
    z   = sigmoid(x_t W_iz^T + b_iz + h_{t-1} W_hz^T + b_hz)
    n   = tanh   (x_t W_in^T + b_in + r * (h_{t-1} W_hn^T + b_hn))
    h_t = (1 - z) * n + z * h_{t-1}

Hidden state = h_t alone.  Loss as for the LSTM oracle: L = sum_t <dy_t, h_t> for a given
upstream gradient (steps dy_first_step..t), or the built-in 0.5 * sum_t sum(h_t^2).
The bias is passed as one vector [b_ih (3H) | b_hh (3H)]; its gradient has the same layout.

All arithmetic is float64 regardless of the input dtype.  numpy's matmul is the only library step.
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np


def _sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


@dataclasses.dataclass
class Gradients:
    dW_ih: np.ndarray   # [3H, I]
    dW_hh: np.ndarray   # [3H, H]
    db: np.ndarray      # [6H]  = [db_ih | db_hh]
    dh0: np.ndarray     # [B, H]
    dx: np.ndarray      # [t, B, I]
    y: np.ndarray       # [t, B, H]
    loss: float


def gru_forward_all(W_ih, W_hh, b, x, h0):
    """Forward over all steps keeping every internal state: dict of [t, B, H] arrays r, z, n,
    q (= h_{t-1} W_hn^T + b_hn) and h (index s-1 holds step s)."""
    f64 = np.float64
    W_ih, W_hh, b, x = (np.asarray(a, f64) for a in (W_ih, W_hh, b, x))
    t, B, _ = x.shape
    H = W_hh.shape[1]
    b_ih, b_hh = b[:3 * H], b[3 * H:]
    st = {k: np.empty((t, B, H), f64) for k in "rznqh"}
    h_prev = np.asarray(h0, f64)
    for s in range(t):
        Gx = x[s] @ W_ih.T + b_ih
        Gh = h_prev @ W_hh.T + b_hh
        r = _sigmoid(Gx[:, 0:H] + Gh[:, 0:H])
        z = _sigmoid(Gx[:, H:2 * H] + Gh[:, H:2 * H])
        q = Gh[:, 2 * H:3 * H]
        n = np.tanh(Gx[:, 2 * H:3 * H] + r * q)
        h = (1.0 - z) * n + z * h_prev
        st["r"][s], st["z"][s], st["n"][s], st["q"][s], st["h"][s] = r, z, n, q, h
        h_prev = h
    return st


def gru_loss(W_ih, W_hh, b, x, h0, dy: Optional[np.ndarray], dy_first_step: int = 1) -> float:
    h = gru_forward_all(W_ih, W_hh, b, x, h0)["h"]
    if dy is None:
        return 0.5 * float(np.sum(h * h))
    return float(np.sum(np.asarray(dy, np.float64) * h[dy_first_step - 1:]))


def gru_bptt(W_ih, W_hh, b, x, h0, dy: Optional[np.ndarray], dy_first_step: int = 1) -> Gradients:
    f64 = np.float64
    W_ih, W_hh, b, x = (np.asarray(a, f64) for a in (W_ih, W_hh, b, x))
    h0 = np.asarray(h0, f64)
    t, B, I = x.shape
    H = W_hh.shape[1]
    st = gru_forward_all(W_ih, W_hh, b, x, h0)
    if dy is not None:
        dy = np.asarray(dy, f64)
        assert dy.shape == (t - dy_first_step + 1, B, H)
        loss = float(np.sum(dy * st["h"][dy_first_step - 1:]))
    else:
        loss = 0.5 * float(np.sum(st["h"] ** 2))
    dW_ih = np.zeros((3 * H, I), f64)
    dW_hh = np.zeros((3 * H, H), f64)
    db_ih = np.zeros((3 * H,), f64)
    db_hh = np.zeros((3 * H,), f64)
    dx = np.zeros((t, B, I), f64)
    dh = np.zeros((B, H), f64)           # gradient arriving from step s+1 through h_s
    for s in range(t, 0, -1):
        r, z, n, q = (st[k][s - 1] for k in "rznq")
        h_prev = st["h"][s - 2] if s > 1 else h0
        if dy is None:
            dh = dh + st["h"][s - 1]
        elif s >= dy_first_step:
            dh = dh + dy[s - dy_first_step]
        dn = dh * (1.0 - z)
        dz = dh * (h_prev - n)
        da_n = dn * (1.0 - n * n)        # pre-activation of the candidate
        da_z = dz * z * (1.0 - z)
        dq = da_n * r
        da_r = da_n * q * r * (1.0 - r)
        dGx = np.concatenate([da_r, da_z, da_n], axis=1)   # through x_t W_ih^T + b_ih
        dGh = np.concatenate([da_r, da_z, dq], axis=1)     # through h_{t-1} W_hh^T + b_hh
        dW_ih += dGx.T @ x[s - 1]
        dW_hh += dGh.T @ h_prev
        db_ih += dGx.sum(axis=0)
        db_hh += dGh.sum(axis=0)
        dx[s - 1] = dGx @ W_ih
        dh = dGh @ W_hh + dh * z
    return Gradients(dW_ih, dW_hh, np.concatenate([db_ih, db_hh]), dh, dx, st["h"], loss)
