"""The *_step_dev calls (neighbour lists in device memory) against the oracle, element by element: graphs beyond
what the ordinary calls take -- more than 256 nodes (tiles of 32 and 16 columns), lists longer than the
kernel-argument encodings hold (symmetric exponential graph on 256 nodes: 3840 entries; a dense graph with
arbitrary weights) -- and small graphs through the same path.  Time-varying topologies pick phase k mod period.
Padding between rows must stay untouched; g is read-only."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

SENT = 31.0


def dense_arbitrary(n, rng):
    rows = []
    for i in range(n):
        w = rng.random(n) + 0.05
        w = (w / w.sum()).astype(np.float32)
        order = rng.permutation(n)
        rows.append([(int(j), float(w[j])) for j in order])
    return rows


CASES = [
    # kind (or "dense"), n, d
    (0, 512, 333), (1, 512, 64), (3, 1024, 40), (3, 256, 1000), (2, 600, 130), (4, 1000, 17),
    (5, 301, 65), ("dense", 40, 515), (0, 1, 70), (1, 3, 5), (1, 257, 1), (0, 1024, 16),
]


@pytest.mark.parametrize("algo", ["decentlam", "dmsgd", "dsgd"])
@pytest.mark.parametrize("kind,n,d", CASES)
def test_device_resident_lists_match_oracle(oracle, algo, kind, n, d):
    import paper_2104_11981_amd as P

    rng = np.random.default_rng(n * 31 + d)
    if kind == "dense":
        otopo = oracle.custom_topology(n, [dense_arbitrary(n, rng)])
        topo = P.make_topology(n, otopo.row_ptr, otopo.col_idx, otopo.w, otopo.period)
    else:
        topo = P.topology_build(kind, n, seed=11, phases=3)
        otopo = oracle.topology(kind, n, seed=11, phases=3)
    W = P.topology_pack_device(topo)
    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    ld = d + 5
    x0, m0 = (rng.standard_normal((n, d)).astype(np.float32) for _ in range(2))
    bufs = [torch.full((n, ld), SENT, dtype=torch.float32, device="cuda") for _ in range(3)]
    bufs[0][:, :d].copy_(torch.from_numpy(x0).cuda())
    bufs[1][:, :d].copy_(torch.from_numpy(m0).cuda())
    x, m, g = (b[:, :d] for b in bufs)
    xr, mr = x0.astype(np.float64), m0.astype(np.float64)
    for k in range(min(topo.period, 3) + 1):
        g0 = rng.standard_normal((n, d)).astype(np.float32)
        g.copy_(torch.from_numpy(g0).cuda())
        if algo == "dsgd":
            P.dsgd_step_dev(x, g, W, gamma, k)
            xr = oracle.dsgd_step(xr.astype(np.float32), g0, otopo, gamma, k)
        else:
            getattr(P, algo + "_step_dev")(x, m, g, W, gamma, beta, k)
            xr, mr = oracle.STEP[algo](xr.astype(np.float32), mr.astype(np.float32), g0, otopo, gamma, beta, k)
        torch.cuda.synchronize()
        for got, ref, what in ((bufs[0], xr, "x"), (bufs[1], mr, "m")):
            a = got.cpu().numpy()
            err = np.abs(a[:, :d].astype(np.float64) - ref)
            assert (err <= 1e-5 * (1 + np.abs(ref))).all(), f"{what}, iteration {k}: off by {err.max():.3e}"
            assert (a[:, d:] == SENT).all()
        np.testing.assert_array_equal(bufs[2].cpu().numpy()[:, :d], g0)
        xr, mr = bufs[0].cpu().numpy()[:, :d].astype(np.float64), bufs[1].cpu().numpy()[:, :d].astype(np.float64)


def test_device_resident_lists_agree_with_the_ordinary_call_where_both_apply(oracle):
    """On a graph both paths take, the two kernels compute the same sums in the same order: same bits."""
    import paper_2104_11981_amd as P

    n, d = 32, 3000
    topo = P.topology_build(P.DL_TOPO_EXP_STATIC, n)
    W = P.topology_pack_device(topo)
    rng = np.random.default_rng(3)
    x0, m0, g0 = (torch.from_numpy(rng.standard_normal((n, d)).astype(np.float32)).cuda() for _ in range(3))
    for algo in ("decentlam", "dmsgd"):
        xa, ma, xb, mb = x0.clone(), m0.clone(), x0.clone(), m0.clone()
        getattr(P, algo + "_step")(xa, ma, g0, topo, 0.05, 0.9, 0)
        getattr(P, algo + "_step_dev")(xb, mb, g0, W, 0.05, 0.9, 0)
        torch.cuda.synchronize()
        assert torch.equal(xa, xb) and torch.equal(ma, mb)
