"""Pins for the oracle's least-squares gradient (CPU only): automatic
differentiation, finite differences, hand cases, a library GEMV."""
import numpy as np
import pytest
import torch


def problem(seed, n, b, d):
    r = np.random.default_rng(seed)
    A = r.standard_normal((n, b, d)).astype(np.float32)
    y = r.standard_normal((n, b)).astype(np.float32)
    x = r.standard_normal((n, d))
    return A, y, x


@pytest.mark.parametrize("n,b,d,scale", [(3, 7, 5, 1.0), (2, 1, 9, 0.25), (4, 33, 1, 1.0 / 33), (1, 64, 48, 1.0 / 64)])
def test_gradient_is_autograd_of_the_loss(oracle, n, b, d, scale):
    """g_i must be the derivative of f_i(x) = (scale/2)||A_i x - y_i||^2 and loss_i its value."""
    A, y, x = problem(1, n, b, d)
    g, loss = oracle.lsq_grad(A, y, x, scale)
    xt = torch.tensor(x, requires_grad=True)
    At, yt = torch.tensor(A, dtype=torch.float64), torch.tensor(y, dtype=torch.float64)
    f = 0.5 * scale * ((torch.einsum("nbd,nd->nb", At, xt) - yt) ** 2).sum(dim=1)
    f.sum().backward()
    np.testing.assert_allclose(g, xt.grad.numpy(), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(loss, f.detach().numpy(), rtol=1e-13)


def test_finite_difference_of_loss(oracle):
    A, y, x = problem(2, 2, 6, 4)
    g, _ = oracle.lsq_grad(A, y, x, 0.5)
    h = 1e-6
    for i in range(2):
        for c in range(4):
            xp, xm = x.copy(), x.copy()
            xp[i, c] += h
            xm[i, c] -= h
            fd = (oracle.lsq_grad(A, y, xp, 0.5)[1][i] - oracle.lsq_grad(A, y, xm, 0.5)[1][i]) / (2 * h)
            assert abs(fd - g[i, c]) < 1e-7 * (1 + abs(g[i, c]))


def test_identity_data_matrix(oracle):
    """A_i = I: g_i = scale (x_i - y_i)."""
    n, d = 3, 6
    r = np.random.default_rng(3)
    A = np.tile(np.eye(d, dtype=np.float32), (n, 1, 1))
    y = r.standard_normal((n, d)).astype(np.float32)
    x = r.standard_normal((n, d))
    g, loss = oracle.lsq_grad(A, y, x, 2.0)
    np.testing.assert_allclose(g, 2.0 * (x - y), rtol=0, atol=1e-15)
    np.testing.assert_allclose(loss, ((x - y) ** 2).sum(axis=1), rtol=1e-15)


def test_scalar_case_by_hand(oracle):
    """b = d = 1: f = (s/2)(a x - y)^2, f' = s a (a x - y).  a=3, x=2, y=1.5, s=0.5 -> 6.75, loss 5.0625."""
    g, loss = oracle.lsq_grad(np.array([[[3.0]]], np.float32), np.array([[1.5]], np.float32),
                              np.array([[2.0]]), 0.5)
    assert g[0, 0] == 6.75 and loss[0] == 5.0625


def test_nodes_use_their_own_data(oracle):
    """Node i's gradient depends on (A_i, y_i, x_i) only; a per-node library GEMV gives it."""
    A, y, x = problem(4, 5, 8, 6)
    g, _ = oracle.lsq_grad(A, y, x, 1.0)
    for i in range(5):
        Ai = A[i].astype(np.float64)
        np.testing.assert_allclose(g[i], Ai.T @ (Ai @ x[i] - y[i]), rtol=1e-13, atol=1e-13)
    A2 = A.copy()
    A2[3] *= 2
    g2, _ = oracle.lsq_grad(A2, y, x, 1.0)
    changed = [i for i in range(5) if not np.array_equal(g[i], g2[i])]
    assert changed == [3]
