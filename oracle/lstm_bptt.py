"""CPU ORACLE (test infrastructure, not product code) -- store-everything LSTM BPTT in float64.

The checkpointed procedures of the paper change how much is recomputed, never what is
computed: their result is exactly the gradient of ordinary back-propagation through time, which
keeps the internal state of every time step (Section 2.1).  So the oracle for the numerical
path is that plain definition written out: forward over all t steps storing every internal
state, then backward over steps t, t-1, ..., 1.

The paper cites the LSTM but never writes it down; the core used here is the standard LSTM
without peepholes, all four gates from one affine map of [x_t, h_{t-1}]:

    G   = x_t W_ih^T + h_{t-1} W_hh^T + b            (gate order i, f, g, o along the 4H axis)
    i,f,o = sigmoid(G_i, G_f, G_o),  g = tanh(G_g)
    c_t = f * c_{t-1} + i * g,       h_t = o * tanh(c_t)

Hidden state (what one core hands to the next) = the pair (h_t, c_t).
Loss: either L = sum_t <dy_t, h_t> for a given upstream gradient dy (so dL/dh_t gets dy_t added
at every step that carries one), or the built-in L = 0.5 * sum_t sum(h_t^2) (dy_t = h_t).

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
    dW_ih: np.ndarray   # [4H, I]
    dW_hh: np.ndarray   # [4H, H]
    db: np.ndarray      # [4H]
    dh0: np.ndarray     # [B, H]
    dc0: np.ndarray     # [B, H]
    dx: np.ndarray      # [t, B, I]
    y: np.ndarray       # [t, B, H]  the outputs h_1..h_t
    loss: float


def lstm_forward_all(W_ih, W_hh, b, x, h0, c0):
    """Forward over all steps keeping every internal state.  Returns dict of [t, B, H] arrays
    i, f, g, o, c, h (index s-1 holds step s)."""
    f64 = np.float64
    W_ih, W_hh, b, x = (np.asarray(a, f64) for a in (W_ih, W_hh, b, x))
    t, B, _ = x.shape
    H = W_hh.shape[1]
    st = {k: np.empty((t, B, H), f64) for k in "ifgoch"}
    h_prev = np.asarray(h0, f64)
    c_prev = np.asarray(c0, f64)
    for s in range(t):
        G = x[s] @ W_ih.T + h_prev @ W_hh.T + b
        i = _sigmoid(G[:, 0 * H:1 * H])
        f = _sigmoid(G[:, 1 * H:2 * H])
        g = np.tanh(G[:, 2 * H:3 * H])
        o = _sigmoid(G[:, 3 * H:4 * H])
        c = f * c_prev + i * g
        h = o * np.tanh(c)
        st["i"][s], st["f"][s], st["g"][s], st["o"][s], st["c"][s], st["h"][s] = i, f, g, o, c, h
        h_prev, c_prev = h, c
    return st


def lstm_loss(W_ih, W_hh, b, x, h0, c0, dy: Optional[np.ndarray], dy_first_step: int = 1) -> float:
    """The scalar loss whose gradient `lstm_bptt` returns."""
    st = lstm_forward_all(W_ih, W_hh, b, x, h0, c0)
    h = st["h"]
    if dy is None:
        return 0.5 * float(np.sum(h * h))
    dy = np.asarray(dy, np.float64)
    return float(np.sum(dy * h[dy_first_step - 1:]))


def lstm_bptt(W_ih, W_hh, b, x, h0, c0, dy: Optional[np.ndarray], dy_first_step: int = 1) -> Gradients:
    """Store-everything back-propagation through time.

    dy: [t - dy_first_step + 1, B, H] upstream gradients for steps dy_first_step..t (1-based),
    zero before; None selects the built-in loss 0.5 * sum h^2."""
    f64 = np.float64
    W_ih, W_hh, b, x = (np.asarray(a, f64) for a in (W_ih, W_hh, b, x))
    h0 = np.asarray(h0, f64)
    c0 = np.asarray(c0, f64)
    t, B, I = x.shape
    H = W_hh.shape[1]
    st = lstm_forward_all(W_ih, W_hh, b, x, h0, c0)
    if dy is not None:
        dy = np.asarray(dy, f64)
        assert dy.shape == (t - dy_first_step + 1, B, H)
        loss = float(np.sum(dy * st["h"][dy_first_step - 1:]))
    else:
        loss = 0.5 * float(np.sum(st["h"] ** 2))

    dW_ih = np.zeros((4 * H, I), f64)
    dW_hh = np.zeros((4 * H, H), f64)
    db = np.zeros((4 * H,), f64)
    dx = np.zeros((t, B, I), f64)
    dh = np.zeros((B, H), f64)       # gradient arriving from step s+1 through h_s
    dc = np.zeros((B, H), f64)       # gradient arriving from step s+1 through c_s
    for s in range(t, 0, -1):        # 1-based step s, arrays hold it at index s-1
        i, f, g, o, c = (st[k][s - 1] for k in "ifgoc")
        h_prev = st["h"][s - 2] if s > 1 else h0
        c_prev = st["c"][s - 2] if s > 1 else c0
        if dy is None:
            dh = dh + st["h"][s - 1]
        elif s >= dy_first_step:
            dh = dh + dy[s - dy_first_step]
        tc = np.tanh(c)
        do = dh * tc
        dc_tot = dc + dh * o * (1.0 - tc * tc)
        di = dc_tot * g
        dg = dc_tot * i
        df = dc_tot * c_prev
        dG = np.concatenate([di * i * (1.0 - i),          # through the sigmoid of the input gate
                             df * f * (1.0 - f),          # forget gate
                             dg * (1.0 - g * g),          # tanh of the candidate
                             do * o * (1.0 - o)], axis=1)  # output gate
        dW_ih += dG.T @ x[s - 1]
        dW_hh += dG.T @ h_prev
        db += dG.sum(axis=0)
        dx[s - 1] = dG @ W_ih
        dh = dG @ W_hh
        dc = dc_tot * f
    return Gradients(dW_ih, dW_hh, db, dh, dc, dx, st["h"], loss)
