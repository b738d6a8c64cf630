"""Pins for the dense-chain back-propagation oracle: central finite differences of a scalar loss on
every parameter and input element, a library's autograd, and a hand-worked one-layer case."""
import numpy as np
import torch

from oracle import chain_bptt as cb


def _chain(widths, B, seed):
    rng = np.random.default_rng(seed)
    W = [rng.uniform(-1, 1, size=(widths[i + 1], widths[i])) / np.sqrt(widths[i]) for i in range(len(widths) - 1)]
    b = [rng.uniform(-0.5, 0.5, size=(widths[i + 1],)) for i in range(len(widths) - 1)]
    x0 = rng.standard_normal((B, widths[0]))
    R = rng.standard_normal((B, widths[-1]))     # loss = sum(R * y_n): dL/dy_n = R
    return W, b, x0, R


def test_finite_differences_every_element():
    W, b, x0, R = _chain([3, 5, 2, 4], 3, 1)
    ref = cb.chain_backprop(W, b, x0, R)
    loss = lambda W_, b_, x_: float((R * cb.chain_forward(W_, b_, x_)[-1]).sum())
    eps = 1e-6
    for i in range(len(W)):
        for idx in np.ndindex(W[i].shape):
            Wp = [w.copy() for w in W]; Wm = [w.copy() for w in W]
            Wp[i][idx] += eps; Wm[i][idx] -= eps
            fd = (loss(Wp, b, x0) - loss(Wm, b, x0)) / (2 * eps)
            assert abs(fd - ref.dW[i][idx]) <= 1e-7 * max(1.0, abs(fd)), (i, idx)
        for j in range(b[i].shape[0]):
            bp = [v.copy() for v in b]; bm = [v.copy() for v in b]
            bp[i][j] += eps; bm[i][j] -= eps
            fd = (loss(W, bp, x0) - loss(W, bm, x0)) / (2 * eps)
            assert abs(fd - ref.db[i][j]) <= 1e-7 * max(1.0, abs(fd)), (i, j)
    for idx in np.ndindex(x0.shape):
        xp = x0.copy(); xm = x0.copy()
        xp[idx] += eps; xm[idx] -= eps
        fd = (loss(W, b, xp) - loss(W, b, xm)) / (2 * eps)
        assert abs(fd - ref.dx0[idx]) <= 1e-7 * max(1.0, abs(fd)), idx


def test_against_library_autograd():
    W, b, x0, R = _chain([7, 12, 5, 9, 3], 6, 2)
    ref = cb.chain_backprop(W, b, x0, R)
    tW = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in W]
    tb = [torch.tensor(v, dtype=torch.float64, requires_grad=True) for v in b]
    tx = torch.tensor(x0, dtype=torch.float64, requires_grad=True)
    y = tx
    for w, v in zip(tW, tb):
        y = torch.tanh(torch.nn.functional.linear(y, w, v))
    (torch.tensor(R) * y).sum().backward()
    assert np.allclose(ref.y, y.detach().numpy(), rtol=0, atol=1e-13)
    for i in range(len(W)):
        assert np.allclose(ref.dW[i], tW[i].grad.numpy(), rtol=1e-11, atol=1e-13)
        assert np.allclose(ref.db[i], tb[i].grad.numpy(), rtol=1e-11, atol=1e-13)
    assert np.allclose(ref.dx0, tx.grad.numpy(), rtol=1e-11, atol=1e-13)


def test_hand_worked_single_layer():
    # one layer, one sequence: y = tanh(w x + b) with w = [[0.5, -1.0]], x = [2, 1], b = [0.25]
    W, b = [np.array([[0.5, -1.0]])], [np.array([0.25])]
    x0, dy = np.array([[2.0, 1.0]]), np.array([[3.0]])
    z = 0.5 * 2.0 - 1.0 * 1.0 + 0.25
    y = np.tanh(z)
    dz = 3.0 * (1.0 - y * y)
    ref = cb.chain_backprop(W, b, x0, dy)
    assert np.allclose(ref.y, [[y]])
    assert np.allclose(ref.dW[0], [[dz * 2.0, dz * 1.0]])
    assert np.allclose(ref.db[0], [dz])
    assert np.allclose(ref.dx0, [[dz * 0.5, dz * -1.0]])
