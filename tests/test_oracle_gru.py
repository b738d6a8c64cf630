"""Pins for the GRU oracle: central finite differences of its own scalar loss, the library GRU's
autograd on the CPU, and a single step worked out by hand."""
import numpy as np
import pytest

from oracle import gru_bptt as og


def _inputs(B, I, H, t, seed, nonzero=True):
    rng = np.random.default_rng(seed)
    k = 1.0 / np.sqrt(H)
    W_ih = rng.uniform(-k, k, (3 * H, I))
    W_hh = rng.uniform(-k, k, (3 * H, H))
    b = rng.uniform(-k, k, (6 * H,)) if nonzero else np.zeros(6 * H)
    x = rng.standard_normal((t, B, I))
    h0 = rng.standard_normal((B, H)) * 0.5 if nonzero else np.zeros((B, H))
    return W_ih, W_hh, b, x, h0, rng


def _fd(fun, arr, idx, eps=1e-6):
    old = arr[idx]
    arr[idx] = old + eps
    up = fun()
    arr[idx] = old - eps
    dn = fun()
    arr[idx] = old
    return (up - dn) / (2 * eps)


@pytest.mark.parametrize("loss,first", [("builtin", 1), ("dy", 1), ("dy", 4)])
def test_finite_differences(loss, first):
    B, I, H, t = 2, 3, 4, 5
    W_ih, W_hh, b, x, h0, rng = _inputs(B, I, H, t, 7)
    dy = None if loss == "builtin" else rng.standard_normal((t - first + 1, B, H))
    g = og.gru_bptt(W_ih, W_hh, b, x, h0, dy, first)
    f = lambda: og.gru_loss(W_ih, W_hh, b, x, h0, dy, first)
    assert abs(g.loss - f()) < 1e-12
    for arr, grad in ((W_ih, g.dW_ih), (W_hh, g.dW_hh), (b, g.db), (x, g.dx), (h0, g.dh0)):
        for _ in range(12):
            idx = tuple(rng.integers(0, s) for s in arr.shape)
            assert abs(_fd(f, arr, idx) - grad[idx]) < 1e-6 * max(1.0, abs(grad[idx])), (arr.shape, idx)


@pytest.mark.parametrize("loss", ["builtin", "dy"])
def test_against_library_gru_autograd(loss):
    torch = pytest.importorskip("torch")
    B, I, H, t = 3, 5, 6, 7
    W_ih, W_hh, b, x, h0, rng = _inputs(B, I, H, t, 11)
    dy = None if loss == "builtin" else rng.standard_normal((t, B, H))
    g = og.gru_bptt(W_ih, W_hh, b, x, h0, dy)
    gru = torch.nn.GRU(I, H, num_layers=1, bias=True, dtype=torch.float64)
    with torch.no_grad():
        gru.weight_ih_l0.copy_(torch.from_numpy(W_ih))
        gru.weight_hh_l0.copy_(torch.from_numpy(W_hh))
        gru.bias_ih_l0.copy_(torch.from_numpy(b[:3 * H]))
        gru.bias_hh_l0.copy_(torch.from_numpy(b[3 * H:]))
    xt = torch.from_numpy(x).requires_grad_(True)
    ht = torch.from_numpy(h0)[None].clone().requires_grad_(True)
    out, _ = gru(xt, ht)
    L = 0.5 * (out * out).sum() if dy is None else (out * torch.from_numpy(dy)).sum()
    L.backward()
    np.testing.assert_allclose(g.y, out.detach().numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(g.dW_ih, gru.weight_ih_l0.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g.dW_hh, gru.weight_hh_l0.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g.db[:3 * H], gru.bias_ih_l0.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g.db[3 * H:], gru.bias_hh_l0.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g.dx, xt.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(g.dh0, ht.grad.numpy()[0], rtol=1e-10, atol=1e-12)


def test_single_step_by_hand():
    # B = I = H = 1, t = 1: scalars
    W_ih = np.array([[0.5], [-0.25], [0.75]])
    W_hh = np.array([[0.1], [0.2], [-0.3]])
    b = np.array([0.01, 0.02, 0.03, 0.04, 0.05, 0.06])
    x = np.array([[[2.0]]])
    h0 = np.array([[0.4]])
    sig = lambda v: 1 / (1 + np.exp(-v))
    r = sig(0.5 * 2 + 0.01 + 0.1 * 0.4 + 0.04)
    z = sig(-0.25 * 2 + 0.02 + 0.2 * 0.4 + 0.05)
    q = -0.3 * 0.4 + 0.06
    n = np.tanh(0.75 * 2 + 0.03 + r * q)
    h = (1 - z) * n + z * 0.4
    g = og.gru_bptt(W_ih, W_hh, b, x, h0, np.array([[[1.0]]]))
    assert abs(g.y[0, 0, 0] - h) < 1e-15
    # dL/dh = 1: d/dh0 = z + dz * W_hz + da_r * W_hr + dq * W_hn
    da_n = (1 - z) * (1 - n * n)
    da_z = (0.4 - n) * z * (1 - z)
    da_r = da_n * q * r * (1 - r)
    assert abs(g.dh0[0, 0] - (z + da_z * 0.2 + da_r * 0.1 + da_n * r * -0.3)) < 1e-15
    assert abs(g.db[5] - da_n * r) < 1e-15 and abs(g.db[2] - da_n) < 1e-15
    assert abs(g.dx[0, 0, 0] - (da_r * 0.5 + da_z * -0.25 + da_n * 0.75)) < 1e-15


def test_zero_upstream_gradient_gives_zero():
    W_ih, W_hh, b, x, h0, _ = _inputs(2, 3, 4, 3, 5)
    g = og.gru_bptt(W_ih, W_hh, b, x, h0, np.zeros((3, 2, 4)))
    for a in (g.dW_ih, g.dW_hh, g.db, g.dx, g.dh0):
        assert not a.any()
