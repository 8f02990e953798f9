"""Edges of what the step kernels accept, each against the oracle element by element.

* 59-64 nodes with long neighbour lists: the fp64 tile of 16-byte lanes (118-128 KiB) leaves room for about
  2000 table entries; longer lists (up to the 2816 entries the one-weight-per-row encoding takes) must run with
  narrower lanes instead of being refused.
* A non-finite value in one node's column: in the gather form it reaches that node's neighbours only, exactly as
  the sums of Algorithms 1 and 2 over j in N_i say (and as the oracle does); in the matrix-core form of dense
  graphs every pair enters the product, absent ones with weight zero, so the whole column turns non-finite
  (documented in the header).  Columns without such a value are unaffected in both forms.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def circulant(n, per_row):
    w = float(np.float32(1.0) / np.float32(per_row))
    return [[((i + t) % n, w) for t in range(per_row)] for i in range(n)]


def pair(P, oracle, n, rows):
    otopo = oracle.custom_topology(n, [rows])
    return P.make_topology(n, otopo.row_ptr, otopo.col_idx, otopo.w, otopo.period), otopo


@pytest.mark.parametrize("n,per_row", [(64, 44), (64, 33), (60, 40), (59, 47), (64, 32)])
@pytest.mark.parametrize("algo", ["decentlam", "dmsgd"])
def test_long_lists_on_59_to_64_nodes_run_with_narrower_lanes(oracle, algo, n, per_row):
    import paper_2104_11981_amd as P

    assert n * per_row <= 2816
    topo, otopo = pair(P, oracle, n, circulant(n, per_row))
    d, ld = 1300, 1312
    rng = np.random.default_rng(n * per_row)
    x0, m0, g0 = (rng.standard_normal((n, d)).astype(np.float32) for _ in range(3))
    bufs = [torch.full((n, ld), 7.0, dtype=torch.float32, device="cuda") for _ in range(3)]
    for b, a in zip(bufs, (x0, m0, g0)):
        b[:, :d].copy_(torch.from_numpy(a).cuda())
    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    getattr(P, algo + "_step")(bufs[0][:, :d], bufs[1][:, :d], bufs[2][:, :d], topo, gamma, beta, 0)
    torch.cuda.synchronize()
    xr, mr = oracle.STEP[algo](x0, m0, g0, otopo, gamma, beta, 0)
    for got, ref in ((bufs[0], xr), (bufs[1], mr)):
        a = got.cpu().numpy()
        assert (np.abs(a[:, :d] - ref) <= 1e-5 * (1 + np.abs(ref))).all()
        assert (a[:, d:] == 7.0).all()


@pytest.mark.parametrize("per_row,dense", [(13, False), (14, True)])   # 32 nodes: the matrix cores take over at 14 per row
@pytest.mark.parametrize("algo", ["decentlam", "dmsgd"])
def test_non_finite_value_stays_with_the_neighbours_when_gathering(oracle, algo, per_row, dense):
    import paper_2104_11981_amd as P

    n, d = 32, 600
    topo, otopo = pair(P, oracle, n, circulant(n, per_row))
    rng = np.random.default_rng(per_row)
    x0, m0, g0 = (rng.standard_normal((n, d)).astype(np.float32) for _ in range(3))
    bad_node, bad_col = 5, 123
    x0[bad_node, bad_col] = np.inf
    x, m, g = (torch.from_numpy(a.copy()).cuda() for a in (x0, m0, g0))
    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    getattr(P, algo + "_step")(x, m, g, topo, gamma, beta, 0)
    torch.cuda.synchronize()
    with np.errstate(invalid="ignore", over="ignore"):
        xr, mr = oracle.STEP[algo](x0, m0, g0, otopo, gamma, beta, 0)
    xa, ma = x.cpu().numpy(), m.cpu().numpy()
    clean = np.ones(d, dtype=bool)
    clean[bad_col] = False
    for got, ref in ((xa, xr), (ma, mr)):   # every other column: the ordinary bar
        assert (np.abs(got[:, clean] - ref[:, clean]) <= 1e-5 * (1 + np.abs(ref[:, clean]))).all()
    readers = np.array([bad_node in [(i + t) % n for t in range(per_row)] for i in range(n)])
    assert readers.sum() == per_row and not np.isfinite(xr[readers, bad_col]).any() and np.isfinite(xr[~readers, bad_col]).all()
    if dense:
        assert not np.isfinite(xa[:, bad_col]).any()          # the whole column, as the header says
    else:
        assert not np.isfinite(xa[readers, bad_col]).any()    # exactly the oracle's pattern
        ok = ~readers
        assert (np.abs(xa[ok, bad_col] - xr[ok, bad_col]) <= 1e-5 * (1 + np.abs(xr[ok, bad_col]))).all()
        assert (np.abs(ma[ok, bad_col] - mr[ok, bad_col]) <= 1e-5 * (1 + np.abs(mr[ok, bad_col]))).all()
