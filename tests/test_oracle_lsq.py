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


def test_sampled_rows_gradient(oracle):
    """The mini-batch gradient is the full-batch gradient of the gathered sub-problem (checked through
    automatic differentiation of the sampled loss), repeated rows count as often as they are drawn,
    and its mean over uniform samples is the full gradient scaled by bs/b (unbiasedness, Assumption A.2)."""
    n, b, d, bs = 3, 9, 5, 4
    A, y, x = problem(7, n, b, d)
    rows = np.array([[0, 3, 3, 8], [1, 2, 4, 6], [8, 8, 8, 0]], dtype=np.int32)
    g, loss = oracle.lsq_grad_rows(A, y, x, rows, 0.5)
    xt = torch.tensor(x, requires_grad=True)
    total = 0.0
    for i in range(n):
        Ai = torch.tensor(A[i][rows[i]], dtype=torch.float64)
        yi = torch.tensor(y[i][rows[i]], dtype=torch.float64)
        fi = 0.25 * ((Ai @ xt[i] - yi) ** 2).sum()
        np.testing.assert_allclose(loss[i], fi.item(), rtol=1e-13)
        total = total + fi
    total.backward()
    np.testing.assert_allclose(g, xt.grad.numpy(), rtol=1e-13, atol=1e-13)
    # all rows once = the full-batch gradient
    full, full_loss = oracle.lsq_grad(A, y, x, 0.5)
    g_all, loss_all = oracle.lsq_grad_rows(A, y, x, np.tile(np.arange(b, dtype=np.int32), (n, 1)), 0.5)
    np.testing.assert_allclose(g_all, full, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(loss_all, full_loss, rtol=1e-13)
    # unbiased: average over every single-row sample equals full / b
    acc = np.zeros_like(full)
    for r in range(b):
        acc += oracle.lsq_grad_rows(A, y, x, np.full((n, 1), r, dtype=np.int32), 0.5)[0]
    np.testing.assert_allclose(acc / b, full / b, rtol=1e-12, atol=1e-13)
    with pytest.raises(ValueError):
        oracle.lsq_grad_rows(A, y, x, np.full((n, 1), b, dtype=np.int32), 1.0)
