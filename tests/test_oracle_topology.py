"""Pins for the oracle's topology generator (CPU only).

The oracle's neighbour tables are checked against (i) tables written out by
hand from the paper's text (tests/golden), (ii) a dense weight matrix built by
an independent set-based routine from the same textual definitions, and
(iii) properties the paper states: rows sum to one (Assumption A.3), ring is
symmetric, the one-peer phases multiply to exact global averaging when n is a
power of two.
"""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_table(name):
    rows = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, tail = line.split(":")
            p, i = (int(t) for t in head.split())
            rows[(p, i)] = [int(t) for t in tail.split()]
    return rows


def table_of(topo):
    out = {}
    for p in range(topo.period):
        rp = topo.row_ptr[p * (topo.n + 1):(p + 1) * (topo.n + 1)]
        for i in range(topo.n):
            out[(p, i)] = [int(j) for j in topo.col_idx[rp[i]:rp[i + 1]]]
    return out


@pytest.mark.parametrize("kind,n,fname", [
    (0, 4, "topology_ring_n4.txt"),
    (1, 8, "topology_exp_static_n8.txt"),
    (2, 8, "topology_exp_onepeer_n8.txt"),
    (3, 8, "topology_exp_sym_n8.txt"),
])
def test_matches_hand_written_table(oracle, kind, n, fname):
    topo = oracle.topology(kind, n)
    assert table_of(topo) == read_table(fname)
    # uniform weights 1/deg in fp32, bit pattern included
    for (p, i), nb in table_of(topo).items():
        rp = topo.row_ptr[p * (n + 1):(p + 1) * (n + 1)]
        assert np.all(topo.w[rp[i]:rp[i + 1]] == np.float32(1.0) / np.float32(len(nb)))


def neighbour_sets(kind, n, phase):
    """N_i straight from the wording, as sets."""
    hops = [h for h in (2 ** t for t in range(64)) if h <= n - 1]
    out = []
    for i in range(n):
        nb = {i}
        if kind == 0:
            nb |= {(i + 1) % n, (i - 1) % n}
        elif kind == 1:
            nb |= {(i + h) % n for h in hops}
        elif kind == 2 and hops:
            nb |= {(i + hops[phase]) % n}
        elif kind == 3:
            nb |= {(i + h) % n for h in hops} | {(i - h) % n for h in hops}
        elif kind == 4:
            R = max(r for r in range(1, n + 1) if n % r == 0 and r * r <= n)
            C = n // R
            a, b = divmod(i, C)
            nb |= {(a + da) * C + (b + db) for da, db in ((-1, 0), (1, 0), (0, -1), (0, 1))
                   if 0 <= a + da < R and 0 <= b + db < C}
        out.append(nb)
    return out


def dense_from_text(kind, n, phase):
    """W from the sets: uniform 1/|N_i| on the directed graphs, Metropolis-Hastings otherwise."""
    nbs = neighbour_sets(kind, n, phase)
    W = np.zeros((n, n))
    for i, nb in enumerate(nbs):
        if kind in (1, 2):
            for j in nb:
                W[i, j] = 1.0 / len(nb)
        else:
            for j in nb - {i}:
                W[i, j] = 1.0 / (1 + max(len(nb) - 1, len(nbs[j]) - 1))
            W[i, i] = 1.0 - W[i].sum()
    return W


@pytest.mark.parametrize("kind", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 7, 8, 16, 17, 32, 64])
def test_dense_matrix_and_stochasticity(oracle, kind, n):
    topo = oracle.topology(kind, n)
    expected_period = 1
    if kind == 2 and n > 1:
        expected_period = int(np.floor(np.log2(n - 1))) + 1
    assert topo.period == expected_period
    assert topo.row_ptr.dtype == np.int32 and topo.col_idx.dtype == np.int32
    for p in range(topo.period):
        W = topo.dense(p)
        np.testing.assert_allclose(W, dense_from_text(kind, n, p), rtol=0, atol=1e-7)
        np.testing.assert_allclose(W.sum(axis=1), 1.0, atol=2e-7)   # Assumption A.3: W 1 = 1
        np.testing.assert_allclose(W.sum(axis=0), 1.0, atol=2e-7)   # circulant => doubly stochastic
        assert np.all(np.diag(W) > 0)                               # N_i contains i
        rp = topo.row_ptr[p * (n + 1):(p + 1) * (n + 1)]
        for i in range(n):
            nb = topo.col_idx[rp[i]:rp[i + 1]]
            assert nb[0] == i and len(set(nb.tolist())) == len(nb)
        if kind in (0, 3, 4):
            np.testing.assert_array_equal(W, W.T)                   # undirected: Assumption A.3 asks for symmetry


def test_config_sizes(oracle):
    # sizes quoted by the workloads: 32 x 6 entries, period 3 / 6
    t = oracle.topology(1, 32)
    assert len(t.col_idx) == 32 * 6 and np.all(t.w == np.float32(1) / np.float32(6))
    rp = t.row_ptr
    assert [int(j) for j in t.col_idx[rp[5]:rp[6]]] == [5, 6, 7, 9, 13, 21]
    assert oracle.topology(2, 8).period == 3
    t = oracle.topology(2, 64)
    assert t.period == 6 and len(t.col_idx) == 6 * 64 * 2


@pytest.mark.parametrize("n", [2, 4, 8, 64])
def test_onepeer_phases_multiply_to_global_average(oracle, n):
    """With n a power of two, one sweep over the hops averages exactly (weights 1/2 are exact)."""
    topo = oracle.topology(2, n)
    P = np.eye(n)
    for p in range(topo.period):
        P = topo.dense(p) @ P
    np.testing.assert_array_equal(P, np.full((n, n), 1.0 / n))


def test_rejects_bad_arguments(oracle):
    with pytest.raises(ValueError):
        oracle.topology(0, 0)
    with pytest.raises(ValueError):
        oracle.topology(7, 4)


def test_mesh_weights_match_hand_computed_fractions(oracle):
    from fractions import Fraction

    topo = oracle.topology(oracle.MESH, 6)
    rp = topo.row_ptr
    with open(os.path.join(GOLDEN, "topology_mesh_n6_weights.txt")) as f:
        lines = [l.strip() for l in f if l.strip() and not l.startswith("#")]
    assert len(lines) == 6
    for line in lines:
        head, tail = line.split(":")
        _, i = (int(t) for t in head.split())
        want = [(int(e.split("=")[0]), Fraction(e.split("=")[1])) for e in tail.split()]
        got_j = [int(j) for j in topo.col_idx[rp[i]:rp[i + 1]]]
        got_w = topo.w[rp[i]:rp[i + 1]]
        assert got_j == [j for j, _ in want]
        for (j, frac), wij in zip(want, got_w):
            assert abs(float(wij) - float(frac)) <= 6e-8, (i, j)
            if j != i:
                assert wij == np.float32(1.0) / np.float32(frac.denominator)   # 1/(1+max deg) evaluated in fp32


@pytest.mark.parametrize("n", [2, 6, 8, 9, 32, 64])
def test_bipartite_random_match_is_a_seeded_perfect_matching(oracle, n):
    phases = 7
    topo = oracle.topology(oracle.BIPARTITE_MATCH, n, seed=12345, phases=phases)
    again = oracle.topology(oracle.BIPARTITE_MATCH, n, seed=12345, phases=phases)
    other = oracle.topology(oracle.BIPARTITE_MATCH, n, seed=12346, phases=phases)
    assert topo.period == phases
    np.testing.assert_array_equal(topo.col_idx, again.col_idx)     # same seed on all nodes => same matching
    if n > 2:
        assert not np.array_equal(topo.col_idx, other.col_idx)
    distinct = set()
    for p in range(phases):
        W = topo.dense(p)
        np.testing.assert_array_equal(W, W.T)
        np.testing.assert_array_equal(W.sum(axis=0), 1.0)
        np.testing.assert_array_equal(W.sum(axis=1), 1.0)
        partner = W.argmax(axis=1) if n == 1 else [int(np.flatnonzero((W[i] > 0) & (np.arange(n) != i))[0])
                                                  if (W[i] > 0).sum() == 2 else i for i in range(n)]
        singles = [i for i in range(n) if partner[i] == i]
        assert len(singles) == n % 2                                # everyone paired (one left over if n is odd)
        for i in range(n):
            assert partner[partner[i]] == i
            if partner[i] != i:
                assert W[i, i] == 0.5 and W[i, partner[i]] == 0.5
        distinct.add(tuple(partner))
    if n >= 8:
        assert len(distinct) > 1                                    # the matching changes from iteration to iteration


def test_bipartite_groups_are_a_uniform_shuffle(oracle):
    """Over many phases every other node shows up as node 0's partner about equally often."""
    n, phases = 8, 7000
    topo = oracle.topology(oracle.BIPARTITE_MATCH, n, seed=99, phases=phases)
    counts = np.zeros(n)
    for p in range(phases):
        rp = topo.row_ptr[p * (n + 1):(p + 1) * (n + 1)]
        counts[topo.col_idx[rp[0] + 1]] += 1
    assert counts[0] == 0
    np.testing.assert_allclose(counts[1:], phases / (n - 1), rtol=0.12)   # 1000 +- 4 sigma
