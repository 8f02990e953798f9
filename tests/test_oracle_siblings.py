"""Pins for the oracle's AWC-DmSGD and DA-DmSGD steps (CPU only).

The paper names the two methods in a sentence each and prints no recursion, so the oracle follows
this build's reading (stated in the oracle source).  The pins below fix the ARITHMETIC of that reading
against independent evaluations -- a library optimizer, dense matrix products, momentum-free
second-order recursions, directly solved fixed points, invariants; they cannot fix the reading itself
("parity weakly pinned").
"""
import numpy as np
import pytest
import torch

from test_oracle_steps import (_quadratic_problem, identity_topology, metropolis_ring, random_state, rng,
                               topo_from_dense)

ALGOS = ["awc_dmsgd", "da_dmsgd"]


@pytest.mark.parametrize("algo", ALGOS)
def test_identity_weights_is_library_momentum_sgd(oracle, algo):
    n, d, steps, gamma, beta = 3, 17, 6, 0.05, 0.9
    x0, _, _ = random_state(1, n, d)
    grads = [rng(10 + k).standard_normal((n, d)) for k in range(steps)]
    x, m = oracle.run(algo, x0, lambda k, x: grads[k], identity_topology(oracle, n), gamma, beta, steps,
                      storage="fp64")
    p = torch.tensor(x0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=gamma, momentum=beta)
    for k in range(steps):
        p.grad = torch.tensor(grads[k], dtype=torch.float64)
        opt.step()
    np.testing.assert_allclose(x, p.detach().numpy(), rtol=0, atol=1e-15)
    np.testing.assert_allclose(m, opt.state[p]["momentum_buffer"].numpy(), rtol=0, atol=1e-15)


@pytest.mark.parametrize("kind,n", [(0, 5), (1, 8), (2, 8), (4, 6)])
def test_beta_zero_reduces_to_the_two_forms_of_dsgd(oracle, kind, n):
    """beta = 0: AWC-DmSGD is the adaptation-with-combination recursion x <- W x - gamma g printed in
    the paper; DA-DmSGD is the adapt-then-combine compact form x <- W (x - gamma g)."""
    d, gamma = 7, 0.07
    topo = oracle.topology(kind, n)
    x, m, g = random_state(3, n, d)
    for k in range(topo.period):
        W = topo.dense(k)
        xa, ma = oracle.awc_dmsgd_step(x, m, g, topo, gamma, 0.0, k)
        xd, md = oracle.da_dmsgd_step(x, m, g, topo, gamma, 0.0, k)
        np.testing.assert_allclose(xa, W @ x - gamma * g, rtol=0, atol=1e-14)
        np.testing.assert_allclose(ma, g, rtol=0, atol=0)
        np.testing.assert_allclose(xd, W @ (x - gamma * g), rtol=0, atol=1e-14)
        np.testing.assert_allclose(xd, oracle.dsgd_step(x, g, topo, gamma, k), rtol=0, atol=1e-15)
        np.testing.assert_allclose(md, W @ g, rtol=0, atol=1e-14)


@pytest.mark.parametrize("kind,n", [(0, 6), (2, 8), (4, 12), (5, 8)])
def test_momentum_free_second_order_recursions(oracle, kind, n):
    """Eliminating m (gamma m^k = W x^{k-1} - x^k in both methods) gives recursions in x alone:
    AWC:  x^{k+1} = W x^k - gamma g^k + beta (x^k - W x^{k-1})
    DA:   x^{k+1} = W [ x^k - gamma g^k + beta (x^k - W x^{k-1}) ]
    (W of the iteration that produced x^k inside the bracket when W varies in time)."""
    d, gamma, beta, steps = 4, 0.05, 0.8, 9
    topo = oracle.topology(kind, n, seed=5, phases=4)
    x0, _, _ = random_state(11, n, d)
    grads = [rng(50 + k).standard_normal((n, d)) for k in range(steps)]
    for algo in ALGOS:
        xs = [x0]
        oracle.run(algo, x0, lambda k, x: grads[k], topo, gamma, beta, steps, storage="fp64",
                   record=lambda k, x, m: xs.append(x.copy()))
        for k in range(1, steps):
            Wk, Wp = topo.dense(k % topo.period), topo.dense((k - 1) % topo.period)
            inner = xs[k] - gamma * grads[k] + beta * (xs[k] - Wp @ xs[k - 1])
            if algo == "awc_dmsgd":
                want = Wk @ xs[k] - gamma * grads[k] + beta * (xs[k] - Wp @ xs[k - 1])
            else:
                want = Wk @ inner
            np.testing.assert_allclose(xs[k + 1], want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("algo", ALGOS)
def test_dense_matrix_form_with_momentum(oracle, algo):
    n, d, gamma, beta = 8, 6, 0.03, 0.9
    topo = oracle.topology(3, n)
    W = topo.dense()
    x, m, g = random_state(4, n, d)
    xo, mo = oracle.STEP[algo](x, m, g, topo, gamma, beta, 0)
    mh = beta * m + g
    if algo == "awc_dmsgd":
        np.testing.assert_allclose(mo, mh, rtol=0, atol=1e-15)
        np.testing.assert_allclose(xo, W @ x - gamma * mh, rtol=0, atol=1e-14)
    else:
        np.testing.assert_allclose(mo, W @ mh, rtol=0, atol=1e-14)
        np.testing.assert_allclose(xo, W @ x - gamma * (W @ mh), rtol=0, atol=1e-14)   # = W (x - gamma mh)


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("kind", [1, 2])
def test_node_average_follows_centralized_momentum_sgd(oracle, algo, kind):
    n, d, gamma, beta, steps = 8, 5, 0.05, 0.9, 10      # weights 1/2, 1/4: exact
    topo = oracle.topology(kind, n)
    x0, _, _ = random_state(8, n, d)
    grads = [rng(80 + k).standard_normal((n, d)) for k in range(steps)]
    xbar, mbar = x0.mean(axis=0), np.zeros(d)
    track = []
    oracle.run(algo, x0, lambda k, x: grads[k], topo, gamma, beta, steps, storage="fp64",
               record=lambda k, x, m: track.append((x.mean(axis=0), m.mean(axis=0))))
    for k in range(steps):
        mbar = beta * mbar + grads[k].mean(axis=0)
        xbar = xbar - gamma * mbar
        np.testing.assert_allclose(track[k][0], xbar, rtol=0, atol=1e-12)
        np.testing.assert_allclose(track[k][1], mbar, rtol=0, atol=1e-11)


def test_da_dmsgd_with_global_averaging_is_parallel_momentum_sgd(oracle):
    """W = 11^T/n: after one iteration all nodes hold the same x and m, and from then on they follow
    momentum SGD on the averaged gradient."""
    n, d, gamma, beta, steps = 4, 6, 0.05, 0.9, 6
    topo = topo_from_dense(oracle, np.full((n, n), 1.0 / n))
    x0, _, _ = random_state(2, n, d)
    grads = [rng(30 + k).standard_normal((n, d)) for k in range(steps)]
    xbar, mbar = x0.mean(axis=0), np.zeros(d)
    x, m = x0, np.zeros_like(x0)
    for k in range(steps):
        x, m = oracle.da_dmsgd_step(x, m, grads[k], topo, gamma, beta, k)
        mbar = beta * mbar + grads[k].mean(axis=0)
        xbar = xbar - gamma * mbar
        np.testing.assert_allclose(x, np.tile(xbar, (n, 1)), rtol=0, atol=1e-13)
        np.testing.assert_allclose(m, np.tile(mbar, (n, 1)), rtol=0, atol=1e-13)


def test_long_run_limits_match_directly_solved_fixed_points(oracle):
    """Full-batch least squares (grad f_i = H_i x - c_i) on a symmetric ring.
    AWC fixed point: m = g/(1-beta), (I - W) x = -gamma/(1-beta) grad f(x).
    DA fixed point:  m = (I - beta W)^-1 W g, (I - W) x = -gamma m."""
    n, b, d, gamma, beta = 8, 12, 5, 0.002, 0.8
    A, y = _quadratic_problem(21, n, b, d)
    topo = topo_from_dense(oracle, metropolis_ring(n))
    W = topo.dense()
    A64, y64 = A.astype(np.float64), y.astype(np.float64)
    H, c = np.zeros((n * d, n * d)), np.zeros(n * d)
    for i in range(n):
        H[i * d:(i + 1) * d, i * d:(i + 1) * d] = A64[i].T @ A64[i]
        c[i * d:(i + 1) * d] = A64[i].T @ y64[i]
    Wk, I = np.kron(W, np.eye(d)), np.eye(n * d)
    grad = lambda k, x: oracle.lsq_grad(A, y, x, 1.0)[0]
    x0 = np.zeros((n, d))
    steps = 12000
    xa, ma = oracle.run("awc_dmsgd", x0, grad, topo, gamma, beta, steps, storage="fp64")
    xd, md = oracle.run("da_dmsgd", x0, grad, topo, gamma, beta, steps, storage="fp64")
    fa = np.linalg.solve((I - Wk) + gamma / (1 - beta) * H, gamma / (1 - beta) * c).reshape(n, d)
    np.testing.assert_allclose(xa, fa, rtol=0, atol=1e-10)
    np.testing.assert_allclose(ma, (H @ fa.reshape(-1) - c).reshape(n, d) / (1 - beta), rtol=0, atol=1e-7)
    K = np.linalg.solve(I - beta * Wk, Wk)                  # (I - beta W)^-1 W
    fd = np.linalg.solve((I - Wk) + gamma * K @ H, gamma * K @ c).reshape(n, d)
    np.testing.assert_allclose(xd, fd, rtol=0, atol=1e-10)
    np.testing.assert_allclose(md, (K @ (H @ fd.reshape(-1) - c)).reshape(n, d), rtol=0, atol=1e-7)


@pytest.mark.parametrize("algo", ALGOS)
def test_columns_are_independent_and_relabelling_permutes(oracle, algo):
    n, d, gamma, beta = 6, 9, 0.05, 0.9
    topo = oracle.topology(0, n)
    x, m, g = random_state(6, n, d)
    xo, mo = oracle.STEP[algo](x, m, g, topo, gamma, beta, 0)
    sub = [1, 4, 7]
    xs, ms = oracle.STEP[algo](x[:, sub], m[:, sub], g[:, sub], topo, gamma, beta, 0)
    np.testing.assert_array_equal(xs, xo[:, sub])
    np.testing.assert_array_equal(ms, mo[:, sub])
    shift = np.roll(np.arange(n), 2)                        # the ring is invariant under rotation
    xr, mr = oracle.STEP[algo](x[shift], m[shift], g[shift], topo, gamma, beta, 0)
    np.testing.assert_allclose(xr, xo[shift], rtol=0, atol=1e-15)
    np.testing.assert_allclose(mr, mo[shift], rtol=0, atol=1e-15)
