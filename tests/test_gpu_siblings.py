"""GPU parity of awc_dmsgd_step / da_dmsgd_step against the oracle's reading of the two methods
(parity weakly pinned: the paper prints no recursion for them; see the oracle source)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from test_gpu_parity import P, check_elementwise, dev, topo_pair  # noqa: E402,F401

CASES = [
    # kind, n, d, pad, off, steps, gamma
    (0, 4, 4096, 0, 0, 6, 0.1),
    (2, 8, 1000, 0, 0, 7, 0.01),
    (1, 16, 1030, 2, 0, 4, 0.1),      # DA: 16-byte accesses up to n = 16
    (1, 32, 1030, 2, 0, 4, 0.1),      # DA: 8-byte accesses
    (1, 32, 777, 3, 1, 3, 0.1),       # misaligned: narrow accesses
    (0, 16, 2051, 1, 3, 3, 0.05),     # head + body + tail
    (2, 64, 517, 3, 0, 7, 0.05),
    (3, 64, 300, 0, 0, 3, 0.1),       # palette-encoded weights
    (0, 100, 333, 0, 0, 2, 0.1),
    (1, 128, 70, 0, 0, 2, 0.1),       # 1024 entries
    (1, 256, 67, 0, 0, 2, 0.1),       # 2304 entries: one weight per row, column indices only
    (4, 12, 515, 1, 0, 4, 0.05),      # irregular degrees
    (5, 9, 64, 0, 0, 6, 0.1),         # a new matching every iteration
    (0, 1, 70, 0, 0, 3, 0.1),
    (0, 3, 1, 0, 0, 3, 0.1),
]


@pytest.mark.parametrize("algo", ["awc_dmsgd", "da_dmsgd"])
@pytest.mark.parametrize("kind,n,d,pad,off,steps,gamma", CASES)
def test_sibling_step_matches_oracle_every_iteration(P, oracle, algo, kind, n, d, pad, off, steps, gamma):
    gamma, beta = float(np.float32(gamma)), float(np.float32(0.9))
    topo, otopo = topo_pair(P, oracle, kind, n)
    rng = np.random.default_rng(500 * n + d)
    x0 = rng.standard_normal((n, d)).astype(np.float32)
    grads = [rng.standard_normal((n, d)).astype(np.float32) for _ in range(steps)]
    ld = d + pad + off
    SENT = 12345.0
    bufs = [torch.full((n, ld), SENT, dtype=torch.float32, device="cuda") for _ in range(3)]
    x, m, g = (b[:, off:off + d] for b in bufs)
    x.copy_(dev(x0))
    m.zero_()
    ref = []
    oracle.run(algo, x0, lambda k, _x: grads[k], otopo, gamma, beta, steps, storage="fp32",
               record=lambda k, xs, ms: ref.append((xs.copy(), ms.copy())))
    fn = getattr(P, algo + "_step")
    for k in range(steps):
        g.copy_(dev(grads[k]))
        fn(x, m, g, topo, gamma, beta, k)
        torch.cuda.synchronize()
        check_elementwise(x.cpu().numpy(), ref[k][0], f"x after iteration {k}")
        check_elementwise(m.cpu().numpy(), ref[k][1], f"m after iteration {k}")
        np.testing.assert_array_equal(g.cpu().numpy(), grads[k])
    for b in bufs:
        full = b.cpu().numpy()
        assert np.all(full[:, :off] == SENT) and np.all(full[:, off + d:] == SENT)


def test_siblings_at_the_maximum_node_count(P, oracle):
    """n = DL_MAX_NODES: both methods run with one fp64 tile of 256 rows (DA-DmSGD uses it twice)."""
    n, d = 256, 70
    topo = P.topology_build(P.DL_TOPO_RING, n)
    otopo = oracle.topology(P.DL_TOPO_RING, n)
    rng = np.random.default_rng(256)
    x0, m0, g0 = (rng.standard_normal((n, d)).astype(np.float32) for _ in range(3))
    gamma, beta = float(np.float32(0.1)), float(np.float32(0.9))
    for algo in ("awc_dmsgd", "da_dmsgd"):
        x, m, g = (torch.from_numpy(a).cuda() for a in (x0, m0, g0))
        getattr(P, algo + "_step")(x, m, g, topo, gamma, beta, 0)
        torch.cuda.synchronize()
        xr, mr = oracle.STEP[algo](x0, m0, g0, otopo, gamma, beta, 0)
        for got, ref, what in ((x, xr, "x"), (m, mr, "m")):
            err = np.abs(got.cpu().numpy().astype(np.float64) - ref)
            assert (err <= 1e-5 * (1.0 + np.abs(ref))).all(), f"{algo} {what}"


@pytest.mark.parametrize("algo", ["awc_dmsgd", "da_dmsgd"])
def test_sibling_steps_at_the_headline_size(P, oracle, algo):
    """n = 32, d = 25.6 M in HBM; the oracle recomputes sampled columns (columns are independent)."""
    import workloads
    from test_gpu_fullsize import sample_columns

    w = workloads.get("c3_exp32")
    d = w.d
    topo, otopo = P.topology_build(1, w.n), oracle.topology(1, w.n)
    gamma, beta = float(np.float32(w.gamma)), float(np.float32(w.beta))
    ct = torch.from_numpy(sample_columns(d, seed=5, blocks=24)).cuda()
    x = workloads.device_x0(w, "cuda")
    m = torch.zeros_like(x)
    g = torch.empty_like(x)
    xs = x.index_select(1, ct).cpu().numpy().astype(np.float64)
    ms = np.zeros_like(xs)
    for k in range(4):
        workloads.device_grad(w, k, g)
        gs = g.index_select(1, ct).cpu().numpy().astype(np.float64)
        getattr(P, algo + "_step")(x, m, g, topo, gamma, beta, k)
        xs, ms = oracle.STEP[algo](xs, ms, gs, otopo, gamma, beta, k)
        xs, ms = xs.astype(np.float32).astype(np.float64), ms.astype(np.float32).astype(np.float64)
        check_elementwise(x.index_select(1, ct).cpu().numpy(), xs, f"x, iteration {k}")
        check_elementwise(m.index_select(1, ct).cpu().numpy(), ms, f"m, iteration {k}")
