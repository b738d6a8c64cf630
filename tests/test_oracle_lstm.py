"""Pins for the oracle's store-everything LSTM BPTT (float64).

P7: every gradient element against central finite differences of the scalar loss.
P8: against a library LSTM's autograd on the host (same gate order i, f, g, o).
Plus hand-checkable special cases.
"""
import numpy as np
import pytest
import torch

from oracle import lstm_bptt as ob
from paper_1606_03401_amd import workloads as wl


def _tiny(loss, dy_first_step=1, t=5, B=2, I=3, H=4, seed=11):
    w = wl.Workload("tiny", B=B, I=I, H=H, t=t, kind=wl.KIND_HSM, m=2, gemm_dtype=wl.GEMM_FP32,
                    loss=loss, dy_first_step=dy_first_step, seed=seed)
    inp = wl.make_inputs(w, nonzero_state=True, nonzero_bias=True)
    return w, [np.asarray(a, np.float64) if a is not None else None
               for a in (inp.W_ih, inp.W_hh, inp.b, inp.x, inp.h0, inp.c0, inp.dy)]


def _fd_check(params, dy, dy_first_step, rtol=2e-6):
    W_ih, W_hh, b, x, h0, c0 = params
    g = ob.lstm_bptt(W_ih, W_hh, b, x, h0, c0, dy, dy_first_step)
    analytic = dict(W_ih=g.dW_ih, W_hh=g.dW_hh, b=g.db, x=g.dx, h0=g.dh0, c0=g.dc0)
    names = ["W_ih", "W_hh", "b", "x", "h0", "c0"]
    eps = 1e-6
    for idx, name in enumerate(names):
        base = params[idx]
        num = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            k = it.multi_index
            p = [a.copy() for a in params]
            p[idx][k] += eps
            lp = ob.lstm_loss(*p, dy, dy_first_step)
            p[idx][k] -= 2 * eps
            lm = ob.lstm_loss(*p, dy, dy_first_step)
            num[k] = (lp - lm) / (2 * eps)
        scale = max(np.abs(num).max(), 1e-12)
        assert np.abs(num - analytic[name]).max() <= rtol * scale + 1e-9, name


def test_finite_differences_builtin_loss():
    _, (W_ih, W_hh, b, x, h0, c0, dy) = _tiny(wl.LOSS_HALF_SUM_H2)
    _fd_check([W_ih, W_hh, b, x, h0, c0], None, 1)


def test_finite_differences_external_dy():
    _, (W_ih, W_hh, b, x, h0, c0, dy) = _tiny(wl.LOSS_EXTERNAL_DY)
    _fd_check([W_ih, W_hh, b, x, h0, c0], dy, 1)


def test_finite_differences_late_loss():
    _, (W_ih, W_hh, b, x, h0, c0, dy) = _tiny(wl.LOSS_EXTERNAL_DY, dy_first_step=4)
    assert dy.shape[0] == 2
    _fd_check([W_ih, W_hh, b, x, h0, c0], dy, 4)


def test_finite_differences_cfg1_shape():
    """Configuration 1's shape (I=16, H=32, B=4) on a shortened sequence; every element of
    dW_ih, dW_hh, db, dh0, dc0 and dx."""
    w = wl.CONFIGS["cfg1"].scaled(t=3)
    inp = wl.make_inputs(w)
    p = [np.asarray(a, np.float64) for a in (inp.W_ih, inp.W_hh, inp.b, inp.x, inp.h0, inp.c0)]
    _fd_check(p, None, 1, rtol=5e-6)


@pytest.mark.parametrize("loss", [wl.LOSS_HALF_SUM_H2, wl.LOSS_EXTERNAL_DY])
def test_against_library_lstm_autograd(loss):
    w = wl.CONFIGS["cfg1"].scaled(loss=loss)
    inp = wl.make_inputs(w, nonzero_state=True, nonzero_bias=True)
    g = ob.lstm_bptt(inp.W_ih, inp.W_hh, inp.b, inp.x, inp.h0, inp.c0, inp.dy, 1)
    lstm = torch.nn.LSTM(w.I, w.H, num_layers=1, bias=True).double()
    with torch.no_grad():
        lstm.weight_ih_l0.copy_(torch.from_numpy(inp.W_ih).double())
        lstm.weight_hh_l0.copy_(torch.from_numpy(inp.W_hh).double())
        lstm.bias_ih_l0.copy_(torch.from_numpy(inp.b).double())
        lstm.bias_hh_l0.zero_()
    x = torch.from_numpy(inp.x).double().requires_grad_(True)
    h0 = torch.from_numpy(inp.h0).double()[None].requires_grad_(True)
    c0 = torch.from_numpy(inp.c0).double()[None].requires_grad_(True)
    y, _ = lstm(x, (h0, c0))
    if loss == wl.LOSS_HALF_SUM_H2:
        L = 0.5 * (y * y).sum()
    else:
        L = (y * torch.from_numpy(inp.dy).double()).sum()
    L.backward()
    assert abs(L.item() - g.loss) <= 1e-10 * max(1.0, abs(g.loss))
    np.testing.assert_allclose(g.y, y.detach().numpy(), rtol=0, atol=1e-12)
    for ours, ref in [(g.dW_ih, lstm.weight_ih_l0.grad), (g.dW_hh, lstm.weight_hh_l0.grad),
                      (g.db, lstm.bias_ih_l0.grad), (g.dx, x.grad), (g.dh0, h0.grad[0]), (g.dc0, c0.grad[0])]:
        ref = ref.numpy()
        assert np.abs(ours - ref).max() <= 1e-11 * max(1.0, np.abs(ref).max())


def test_single_step_by_hand():
    """t = 1, B = 1, I = 1, H = 1: every quantity written out by hand."""
    W_ih = np.array([[0.3], [-0.2], [0.5], [0.1]])
    W_hh = np.array([[0.4], [0.6], [-0.7], [0.2]])
    b = np.array([0.05, -0.1, 0.2, 0.0])
    x = np.array([[[1.5]]]); h0 = np.array([[0.25]]); c0 = np.array([[-0.5]]); dy = np.array([[[2.0]]])
    z = W_ih[:, 0] * 1.5 + W_hh[:, 0] * 0.25 + b
    sg = lambda v: 1 / (1 + np.exp(-v))
    i, f, g_, o = sg(z[0]), sg(z[1]), np.tanh(z[2]), sg(z[3])
    c = f * -0.5 + i * g_
    h = o * np.tanh(c)
    dc = 2.0 * o * (1 - np.tanh(c) ** 2)
    dz = np.array([dc * g_ * i * (1 - i), dc * -0.5 * f * (1 - f), dc * i * (1 - g_ ** 2),
                   2.0 * np.tanh(c) * o * (1 - o)])
    g = ob.lstm_bptt(W_ih, W_hh, b, x, h0, c0, dy)
    assert np.allclose(g.y[0, 0, 0], h, atol=1e-15)
    assert np.allclose(g.db, dz, atol=1e-15)
    assert np.allclose(g.dW_ih[:, 0], dz * 1.5, atol=1e-15)
    assert np.allclose(g.dW_hh[:, 0], dz * 0.25, atol=1e-15)
    assert np.allclose(g.dh0[0, 0], dz @ W_hh[:, 0], atol=1e-15)
    assert np.allclose(g.dc0[0, 0], dc * f, atol=1e-15)
    assert np.allclose(g.dx[0, 0, 0], dz @ W_ih[:, 0], atol=1e-15)


def test_zero_upstream_gradient_gives_zero():
    w, (W_ih, W_hh, b, x, h0, c0, dy) = _tiny(wl.LOSS_EXTERNAL_DY)
    g = ob.lstm_bptt(W_ih, W_hh, b, x, h0, c0, np.zeros_like(dy))
    for a in (g.dW_ih, g.dW_hh, g.db, g.dh0, g.dc0, g.dx):
        assert not a.any()
