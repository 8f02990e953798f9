"""Pins for the oracle's DmSGD / DecentLaM / DSGD steps (CPU only).

None of these re-types the oracle's formulas.  Each test compares the oracle
with something the paper or the mathematics fixes independently: a library
optimizer, a dense matrix product, the momentum-free second-order recursions,
the s-domain derivation, exact rational arithmetic, invariants, fixed points.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch


def rng(seed):
    return np.random.default_rng(seed)


def random_state(seed, n, d):
    r = rng(seed)
    return r.standard_normal((n, d)), r.standard_normal((n, d)), r.standard_normal((n, d))


def identity_topology(oracle, n):
    return oracle.custom_topology(n, [[[(i, 1.0)] for i in range(n)]])


def topo_from_dense(oracle, W):
    n = W.shape[0]
    return oracle.custom_topology(n, [[[(j, float(W[i, j])) for j in range(n) if W[i, j] != 0]
                                       for i in range(n)]])


def metropolis_ring(n, self_weight=None):
    """Symmetric doubly stochastic ring; optional larger self weight (positive definite)."""
    W = np.zeros((n, n))
    for i in range(n):
        W[i, (i + 1) % n] += 1 / 3
        W[i, (i - 1) % n] += 1 / 3
        W[i, i] += 1 / 3
    if self_weight is not None:
        W = self_weight * np.eye(n) + (1 - self_weight) * W
    return W


# ---------------------------------------------------------------- W = I
@pytest.mark.parametrize("algo", ["dmsgd", "decentlam"])
def test_identity_weights_is_library_momentum_sgd(oracle, algo):
    """With W = I every node runs plain heavy-ball SGD; torch.optim.SGD is the library form
    (buf = beta*buf + g, p = p - lr*buf), the optimizer the paper says the update maps to."""
    n, d, steps, gamma, beta = 3, 17, 6, 0.05, 0.9
    x0, _, _ = random_state(1, n, d)
    grads = [rng(10 + k).standard_normal((n, d)) for k in range(steps)]
    topo = identity_topology(oracle, n)
    x, _ = oracle.run(algo, x0, lambda k, x: grads[k], topo, gamma, beta, steps, storage="fp64")

    p = torch.tensor(x0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=gamma, momentum=beta)
    for k in range(steps):
        p.grad = torch.tensor(grads[k], dtype=torch.float64)
        opt.step()
    # DecentLaM forms (x - z)/gamma with z = x - gamma g: a few ulp of |x|/gamma per step
    tol = 1e-15 if algo == "dmsgd" else 5e-13
    np.testing.assert_allclose(x, p.detach().numpy(), rtol=0, atol=tol)


# ---------------------------------------------------------------- beta = 0
@pytest.mark.parametrize("kind,n", [(0, 5), (1, 8), (2, 8)])
def test_beta_zero_is_dsgd_compact_form(oracle, kind, n):
    """beta = 0: both algorithms collapse to x+ = W (x - gamma g) (DSGD compact form)."""
    d, gamma = 11, 0.07
    topo = oracle.topology(kind, n)
    x, m, g = random_state(2, n, d)
    for k in range(topo.period):
        W = topo.dense(k)
        expect = W @ (x - gamma * g)
        for algo in (oracle.dmsgd_step, oracle.decentlam_step):
            xn, _ = algo(x, m, g, topo, gamma, 0.0, k)
            np.testing.assert_allclose(xn, expect, rtol=0, atol=2e-14)
        np.testing.assert_allclose(oracle.dsgd_step(x, g, topo, gamma, k), expect, rtol=0, atol=1e-15)


def test_first_step_from_zero_momentum_coincides(oracle):
    """k = 0, m = 0: x^1 = W(x^0 - gamma g^0) for both; they part ways from k = 1 on."""
    n, d, gamma, beta = 8, 9, 0.1, 0.9
    topo = oracle.topology(0, n)
    x, _, g = random_state(3, n, d)
    m0 = np.zeros_like(x)
    xa, ma = oracle.dmsgd_step(x, m0, g, topo, gamma, beta)
    xb, mb = oracle.decentlam_step(x, m0, g, topo, gamma, beta)
    np.testing.assert_allclose(xa, xb, rtol=0, atol=1e-14)
    g1 = rng(4).standard_normal((n, d))
    xa2, _ = oracle.dmsgd_step(xa, ma, g1, topo, gamma, beta, 1)
    xb2, _ = oracle.decentlam_step(xb, mb, g1, topo, gamma, beta, 1)
    assert np.abs(xa2 - xb2).max() > 1e-3


# ---------------------------------------------------------------- second-order recursions
def test_dmsgd_second_order_recursion(oracle):
    """x^{k+1} = W(x^k - gamma g^k) + beta (x^k - W x^{k-1})   (static W)."""
    n, d, gamma, beta, steps = 8, 7, 0.05, 0.8, 12
    topo = oracle.topology(1, n)
    W = topo.dense()
    x0, _, _ = random_state(5, n, d)
    grads = [rng(50 + k).standard_normal((n, d)) for k in range(steps)]
    hist = [x0]
    oracle.run("dmsgd", x0, lambda k, x: grads[k], topo, gamma, beta, steps, storage="fp64",
               record=lambda k, x, m: hist.append(x.copy()))
    for k in range(1, steps):
        expect = W @ (hist[k] - gamma * grads[k]) + beta * (hist[k] - W @ hist[k - 1])
        np.testing.assert_allclose(hist[k + 1], expect, rtol=0, atol=1e-12)


@pytest.mark.parametrize("kind", [0, 2])
def test_decentlam_second_order_recursion(oracle, kind):
    """x^{k+1} = W^k (x^k - gamma g^k) + beta (x^k - x^{k-1}), W^k may vary with k."""
    n, d, gamma, beta, steps = 8, 7, 0.05, 0.8, 12
    topo = oracle.topology(kind, n)
    x0, _, _ = random_state(6, n, d)
    grads = [rng(60 + k).standard_normal((n, d)) for k in range(steps)]
    hist = [x0]
    oracle.run("decentlam", x0, lambda k, x: grads[k], topo, gamma, beta, steps, storage="fp64",
               record=lambda k, x, m: hist.append(x.copy()))
    for k in range(1, steps):
        Wk = topo.dense(k % topo.period)
        expect = Wk @ (hist[k] - gamma * grads[k]) + beta * (hist[k] - hist[k - 1])
        np.testing.assert_allclose(hist[k + 1], expect, rtol=0, atol=1e-11)


# ---------------------------------------------------------------- forms of the corrected gradient
def test_corrected_gradient_forms_and_zero_sum(oracle):
    """gt = m+ - beta m must equal W g + (1/gamma)(I - W) x, and the correction
    (1/gamma)(I - W) x sums to zero over nodes for a column-stochastic W."""
    n, d, gamma, beta = 8, 13, 0.01, 0.9       # n = 8: weights 1/4 are exact in fp32
    topo = oracle.topology(1, n)
    W = topo.dense()
    x, m, g = random_state(7, n, d)
    _, mn = oracle.decentlam_step(x, m, g, topo, gamma, beta)
    gt = mn - beta * m
    np.testing.assert_allclose(gt, W @ g + (np.eye(n) - W) @ x / gamma, rtol=0, atol=1e-11)
    corr = gt - W @ g
    np.testing.assert_allclose(corr.sum(axis=0), 0.0, atol=1e-11)


# ---------------------------------------------------------------- node average
@pytest.mark.parametrize("algo", ["dmsgd", "decentlam"])
@pytest.mark.parametrize("kind", [0, 1, 2])
def test_node_average_follows_centralized_momentum_sgd(oracle, algo, kind):
    """Doubly stochastic W: mean_i x_i obeys mbar+ = beta mbar + gbar, xbar+ = xbar - gamma mbar+."""
    n, d, gamma, beta, steps = 8, 5, 0.05, 0.9, 10   # n = 8: weights 1/2, 1/4 exact; ring 1/3 not
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
        np.testing.assert_allclose(track[k][0], xbar, rtol=0, atol=2e-6 if kind == 0 else 1e-12)
        if algo == "dmsgd" or kind != 0:
            np.testing.assert_allclose(track[k][1], mbar, rtol=0, atol=2e-5 if kind == 0 else 1e-11)


# ---------------------------------------------------------------- scaled momentum
def test_scaled_momentum_gives_same_iterates(oracle):
    """mhat+ = beta mhat + (1-beta) gt ; x+ = x - gamma/(1-beta) mhat+ gives the same x (mhat^0 = 0)."""
    n, d, gamma, beta, steps = 8, 6, 0.02, 0.8, 15
    topo = oracle.topology(0, n)
    W = topo.dense()
    x0, _, _ = random_state(9, n, d)
    grads = [rng(90 + k).standard_normal((n, d)) for k in range(steps)]
    xs = []
    oracle.run("decentlam", x0, lambda k, x: grads[k], topo, gamma, beta, steps, storage="fp64",
               record=lambda k, x, m: xs.append(x.copy()))
    x, mh = x0.copy(), np.zeros_like(x0)
    for k in range(steps):
        gt = W @ grads[k] + (x - W @ x) / gamma
        mh = beta * mh + (1 - beta) * gt
        x = x - gamma / (1 - beta) * mh
        np.testing.assert_allclose(xs[k], x, rtol=0, atol=1e-11)


# ---------------------------------------------------------------- s-domain derivation
def test_decentlam_is_momentum_sgd_in_the_s_domain(oracle):
    """Positive-definite symmetric W: momentum SGD on f(W^{1/2} s) + (1/2 gamma)||s||^2_{I-W}
    mapped back by x = W^{1/2} s is DecentLaM (Sec. "Improving Inconsistency Bias")."""
    n, d, b, gamma, beta, steps = 6, 4, 7, 0.01, 0.8, 25
    W = metropolis_ring(n, self_weight=0.5)
    lam, U = np.linalg.eigh(W)
    assert lam.min() > 0
    Wh = U @ np.diag(np.sqrt(lam)) @ U.T
    r = rng(11)
    A = r.standard_normal((n, b, d))
    y = r.standard_normal((n, b))

    def grad_f(X):  # stacked gradients of f_i(x) = 0.5 ||A_i x - y_i||^2
        return np.stack([A[i].T @ (A[i] @ X[i] - y[i]) for i in range(n)])

    s = r.standard_normal((n, d))
    ms = np.zeros_like(s)
    topo = topo_from_dense(oracle, W)
    Wf = topo.dense()   # fp32-rounded weights, used on both sides
    lam, U = np.linalg.eigh(Wf)
    Wh = U @ np.diag(np.sqrt(lam)) @ U.T
    x = Wh @ s
    m = np.zeros_like(x)
    for k in range(steps):
        g = grad_f(x)
        x, m = oracle.decentlam_step(x, m, g, topo, gamma, beta, k)
        gs = Wh @ grad_f(Wh @ s) + (s - Wf @ s) / gamma
        ms = beta * ms + gs
        s = s - gamma * ms
        np.testing.assert_allclose(x, Wh @ s, rtol=0, atol=1e-10)
        np.testing.assert_allclose(m, Wh @ ms, rtol=0, atol=1e-8)


# ---------------------------------------------------------------- exact rational brute force
@pytest.mark.parametrize("algo", ["dmsgd", "decentlam"])
def test_exact_rational_brute_force(oracle, algo):
    """Three nodes, two coordinates, every quantity a small dyadic rational (exact in binary):
    the per-node statements of Algorithms 1 and 2 evaluated with Fractions."""
    n, d = 3, 2
    nbrs = [[(0, Fraction(1, 2)), (1, Fraction(1, 4)), (2, Fraction(1, 4))],
            [(1, Fraction(1, 2)), (0, Fraction(1, 4)), (2, Fraction(1, 4))],
            [(2, Fraction(1, 2)), (0, Fraction(1, 4)), (1, Fraction(1, 4))]]
    gamma, beta = Fraction(1, 8), Fraction(3, 4)
    X = [[Fraction(3, 2), Fraction(-1, 4)], [Fraction(5, 8), Fraction(2)], [Fraction(-3), Fraction(1, 2)]]
    M = [[Fraction(1, 2), Fraction(1)], [Fraction(-1, 8), Fraction(0)], [Fraction(2), Fraction(-3, 4)]]
    G = [[Fraction(1), Fraction(-2)], [Fraction(1, 4), Fraction(3)], [Fraction(-1, 2), Fraction(7, 8)]]
    Xn = [[None] * d for _ in range(n)]
    Mn = [[None] * d for _ in range(n)]
    for c in range(d):
        if algo == "dmsgd":
            for i in range(n):
                Mn[i][c] = beta * M[i][c] + G[i][c]
            half = [X[i][c] - gamma * Mn[i][c] for i in range(n)]
            for i in range(n):
                Xn[i][c] = sum(wij * half[j] for j, wij in nbrs[i])
        else:
            for i in range(n):
                gt = X[i][c] / gamma - sum(wij * (X[j][c] - gamma * G[j][c]) for j, wij in nbrs[i]) / gamma
                Mn[i][c] = beta * M[i][c] + gt
                Xn[i][c] = X[i][c] - gamma * Mn[i][c]
    topo = oracle.custom_topology(n, [[[(j, float(wij)) for j, wij in row] for row in nbrs]])
    to_np = lambda T: np.array([[float(v) for v in row] for row in T])
    xo, mo = oracle.STEP[algo](to_np(X), to_np(M), to_np(G), topo, float(gamma), float(beta))
    np.testing.assert_array_equal(xo, to_np(Xn))   # all values dyadic: fp64 is exact here
    np.testing.assert_array_equal(mo, to_np(Mn))


# ---------------------------------------------------------------- structure
@pytest.mark.parametrize("algo", ["dmsgd", "decentlam"])
def test_identical_nodes_follow_single_node_momentum_sgd(oracle, algo):
    n, d, gamma, beta, steps = 8, 5, 0.1, 0.9, 8
    topo = oracle.topology(2, n)   # weights 1/2: rows sum to 1 exactly
    row = rng(12).standard_normal(d)
    grads = [rng(120 + k).standard_normal(d) for k in range(steps)]
    x, m = oracle.run(algo, np.tile(row, (n, 1)), lambda k, x: np.tile(grads[k], (n, 1)), topo,
                      gamma, beta, steps, storage="fp64")
    xs, ms = row.copy(), np.zeros(d)
    for k in range(steps):
        ms = beta * ms + grads[k]
        xs = xs - gamma * ms
    np.testing.assert_allclose(x, np.tile(xs, (n, 1)), rtol=0, atol=1e-12)
    np.testing.assert_allclose(m, np.tile(ms, (n, 1)), rtol=0, atol=1e-11)


def test_global_averaging_weights_give_parallel_sgd(oracle):
    """W = 11^T/n: after one DSGD/DmSGD step every node holds the same model (Parallel SGD)."""
    n, d, gamma = 4, 6, 0.1
    topo = topo_from_dense(oracle, np.full((n, n), 0.25))
    x, m, g = random_state(13, n, d)
    xn, _ = oracle.dmsgd_step(x, np.zeros_like(x), g, topo, gamma, 0.9)
    expect = (x - gamma * g).mean(axis=0)
    np.testing.assert_allclose(xn, np.tile(expect, (n, 1)), rtol=0, atol=1e-15)


@pytest.mark.parametrize("algo", ["dmsgd", "decentlam"])
def test_relabelling_nodes_permutes_the_result(oracle, algo):
    n, d, gamma, beta = 8, 4, 0.05, 0.9
    topo = oracle.topology(1, n)
    W = topo.dense()
    x, m, g = random_state(14, n, d)
    perm = rng(15).permutation(n)
    P = np.eye(n)[perm]
    topo_p = topo_from_dense(oracle, P @ W @ P.T)
    xa, ma = oracle.STEP[algo](x, m, g, topo, gamma, beta)
    xb, mb = oracle.STEP[algo](P @ x, P @ m, P @ g, topo_p, gamma, beta)
    np.testing.assert_allclose(xb, P @ xa, rtol=0, atol=1e-13)
    np.testing.assert_allclose(mb, P @ ma, rtol=0, atol=1e-12)


def test_columns_are_independent(oracle):
    """Mixing acts along the node axis only: a step on a column subset equals the subset of a step."""
    n, d = 8, 40
    topo = oracle.topology(1, n)
    x, m, g = random_state(16, n, d)
    cols = np.array([3, 17, 18, 39])
    for fn in (oracle.dmsgd_step, oracle.decentlam_step):
        xa, ma = fn(x, m, g, topo, 0.1, 0.9)
        xb, mb = fn(x[:, cols], m[:, cols], g[:, cols], topo, 0.1, 0.9)
        np.testing.assert_array_equal(xa[:, cols], xb)
        np.testing.assert_array_equal(ma[:, cols], mb)


def test_time_varying_phase_selection(oracle):
    """Iteration k uses phase k mod period."""
    n, d = 8, 3
    topo = oracle.topology(2, n)
    x, m, g = random_state(17, n, d)
    for k in (0, 1, 2, 3, 7, 300):
        W = topo.dense(k % 3)
        xn, _ = oracle.dmsgd_step(x, m, g, topo, 0.1, 0.9, k)
        np.testing.assert_allclose(xn, W @ (x - 0.1 * (0.9 * m + g)), rtol=0, atol=1e-14)


# ---------------------------------------------------------------- fixed points (quadratic f_i)
def _quadratic_problem(seed, n, b, d):
    r = rng(seed)
    A = r.standard_normal((n, b, d)).astype(np.float32)
    xo = r.standard_normal(d)
    y = (np.einsum("nbd,d->nb", A.astype(np.float64), xo) + 0.01 * r.standard_normal((n, b))).astype(np.float32)
    return A, y


def _fixed_point(W, A, y, gamma, momentum_factor):
    """Solve momentum_factor (I - W) X = -gamma W grad f(X) for stacked X, grad f_i = H_i x - c_i."""
    n, b, d = A.shape
    A64, y64 = A.astype(np.float64), y.astype(np.float64)
    H = np.zeros((n * d, n * d))
    c = np.zeros(n * d)
    for i in range(n):
        H[i * d:(i + 1) * d, i * d:(i + 1) * d] = A64[i].T @ A64[i]
        c[i * d:(i + 1) * d] = A64[i].T @ y64[i]
    Wk = np.kron(W, np.eye(d))
    lhs = momentum_factor * (np.eye(n * d) - Wk) + gamma * Wk @ H
    return np.linalg.solve(lhs, gamma * Wk @ c).reshape(n, d)


def test_long_run_limits_match_fixed_point_equations(oracle):
    """Full-batch least squares on a symmetric ring: the iterates reach the solutions of
    (I-W)x = -gamma W grad f(x) (DecentLaM, same as DSGD, beta-independent) and
    (1-beta)(I-W)x = -gamma W grad f(x) (DmSGD); DecentLaM's momentum dies out; and DecentLaM's
    distance to the global minimiser equals DSGD's and is below DmSGD's."""
    n, b, d, gamma, beta = 8, 12, 5, 0.004, 0.8
    A, y = _quadratic_problem(21, n, b, d)
    topo = oracle.topology(0, n)
    W = topo.dense()
    grad = lambda k, x: oracle.lsq_grad(A, y, x, 1.0)[0]
    x0 = np.zeros((n, d))
    steps = 6000
    x_lam, m_lam = oracle.run("decentlam", x0, grad, topo, gamma, beta, steps, storage="fp64")
    x_dm, _ = oracle.run("dmsgd", x0, grad, topo, gamma, beta, steps, storage="fp64")
    x_ds = x0
    for k in range(4 * steps):
        x_ds = oracle.dsgd_step(x_ds, grad(k, x_ds), topo, gamma, k)

    fp_lam = _fixed_point(W, A, y, gamma, 1.0)
    fp_dm = _fixed_point(W, A, y, gamma, 1.0 - beta)
    np.testing.assert_allclose(x_lam, fp_lam, rtol=0, atol=1e-10)
    np.testing.assert_allclose(x_ds, fp_lam, rtol=0, atol=1e-10)
    np.testing.assert_allclose(x_dm, fp_dm, rtol=0, atol=1e-10)
    assert np.abs(m_lam).max() < 1e-9

    A64 = A.astype(np.float64).reshape(n * b, d)
    xstar = np.linalg.lstsq(A64, y.astype(np.float64).reshape(-1), rcond=None)[0]
    err = lambda X: np.mean(np.sum((X - xstar) ** 2, axis=1)) / np.sum(xstar ** 2)
    assert abs(err(x_lam) - err(x_ds)) < 1e-12
    assert err(x_dm) > 3 * err(x_lam)          # bias amplified by up to 1/(1-beta)^2


# ---------------------------------------------------------------- diagnostics
def test_stats_against_library_moments(oracle):
    """Consensus distance is n times the population variance over nodes summed over columns;
    the other entries are plain squared norms (numpy)."""
    n, d = 7, 23
    r = rng(30)
    x = r.standard_normal((n, d)) * 3 + 100.0      # large common offset: a one-pass formula would cancel
    m = r.standard_normal((n, d))
    ref = r.standard_normal(d)
    out = oracle.stats(x, m, ref)
    np.testing.assert_allclose(out[0], n * np.var(x, axis=0).sum(), rtol=1e-12)
    np.testing.assert_allclose(out[1], (x.mean(axis=0) ** 2).sum(), rtol=1e-13)
    np.testing.assert_allclose(out[2], ((x - ref) ** 2).sum(), rtol=1e-13)
    np.testing.assert_allclose(out[3], (ref ** 2).sum(), rtol=1e-13)
    np.testing.assert_allclose(out[4], np.linalg.norm(m, "fro") ** 2, rtol=1e-13)
    # Pythagoras over nodes: sum_i ||x_i||^2 = consensus + n ||xbar||^2
    np.testing.assert_allclose((x ** 2).sum(), out[0] + n * out[1], rtol=1e-13)
    # identical rows: zero consensus distance exactly
    same = np.tile(r.standard_normal(d), (n, 1))
    assert oracle.stats(same)[0] < 1e-25          # identical rows: no consensus distance beyond rounding of the mean
    assert np.all(oracle.stats(x)[2:] == 0.0)


def test_oracle_reproduces_its_frozen_trajectory():
    """tests/golden/oracle_traj_c1.txt was written by make_golden.py from the oracle alone; the oracle
    must still produce it bit for bit (guards against silent changes of its arithmetic)."""
    import importlib.util
    import os

    here = os.path.join(os.path.dirname(__file__), "golden")
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.trajectories()
    seen = 0
    with open(os.path.join(here, "oracle_traj_c1.txt")) as f:
        for line in f:
            if line.startswith("#"):
                continue
            head, tail = line.split(":")
            algo, name, i = head.split()
            want = np.array([float.fromhex(t) for t in tail.split()], dtype=np.float32)
            got = now[algo][0 if name == "x" else 1][int(i)]
            np.testing.assert_array_equal(got, want)
            seen += 1
    assert seen == 16


# ---------------------------------------------------------------- momentum-free DecentLaM
@pytest.mark.parametrize("kind", [0, 2, 3])
def test_xprev_form_reproduces_algorithm_2(oracle, kind):
    """The (x^k, x^{k-1}) recursion of the appendix "Reformulation of DecentLaM" must generate the
    iterates of Algorithm 2 -- also with a time-varying W and with a learning rate that changes every
    iteration (factor gamma_k / gamma_{k-1}); the momentum Algorithm 2 carries is (x^{k-1} - x^k)/gamma_{k-1}."""
    n, d, beta, steps = 8, 6, 0.9, 14
    topo = oracle.topology(kind, n)
    x0, _, _ = random_state(40, n, d)
    grads = [rng(400 + k).standard_normal((n, d)) for k in range(steps)]
    gammas = [0.05 * (1 + 0.3 * np.sin(k)) for k in range(steps)]       # a schedule
    xa, ma = x0.copy(), np.zeros_like(x0)
    xc, xp = x0.copy(), x0.copy()                                       # x^{-1} = x^0  <=>  m^0 = 0
    for k in range(steps):
        xa, ma = oracle.decentlam_step(xa, ma, grads[k], topo, gammas[k], beta, k)
        xn = oracle.decentlam_xprev_step(xc, xp, grads[k], topo, gammas[k], beta, k,
                                         gamma_prev=gammas[k - 1] if k else gammas[0])
        xc, xp = xn, xc
        np.testing.assert_allclose(xc, xa, rtol=0, atol=1e-10)
        np.testing.assert_allclose((xp - xc) / gammas[k], ma, rtol=0, atol=1e-8)


def test_xprev_form_against_dense_matrices(oracle):
    n, d, gamma, beta = 8, 5, 0.1, 0.8
    topo = oracle.topology(1, n)
    W = topo.dense()
    x, xp, g = random_state(41, n, d)
    out = oracle.decentlam_xprev_step(x, xp, g, topo, gamma, beta)
    np.testing.assert_allclose(out, W @ (x - gamma * g) + beta * (x - xp), rtol=0, atol=1e-14)
