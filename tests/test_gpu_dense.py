"""GPU parity of the step entry points on dense graphs with 23-48 nodes, where the mixing of a tile
runs as an fp64 matrix product on the matrix cores instead of one LDS gather per neighbour (from
46 - n entries per row on average up to 32 nodes: 14 at 32 nodes, all 23 at 23 nodes; from 38 - n / 4
entries per row at 33-48 nodes: 26 at 48 nodes; smaller graphs always gather).  Same bar as everywhere: every element of x and m against the
oracle, |diff| <= 1e-5 (1 + |ref|), padding untouched.  Graphs: all-to-all with equal weights,
dense random graphs with Metropolis-Hastings weights (few distinct values: palette encoding), random
row-stochastic weights in shuffled list order (arbitrary values: direct encoding), graphs right at
the switch-over density on either side, two alternating phases."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

SENT = 4242.0


@pytest.fixture(scope="module")
def P():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2104_11981_amd as pkg

    return pkg


def all_to_all(n, rng):
    w = np.float32(1.0 / n)   # n of them sum to 1 well within the library's check
    return [[(j, float(w)) for j in range(n)] for _ in range(n)]


def metropolis_dense(n, rng, p=0.75):
    a = rng.random((n, n)) < p
    a = np.triu(a, 1)
    a = a | a.T
    deg = a.sum(1)
    rows = []
    for i in range(n):
        lst, total = [], 0.0
        for j in np.flatnonzero(a[i]):
            wij = float(np.float32(1.0 / (1 + max(deg[i], deg[j]))))
            lst.append((int(j), wij))
            total += wij
        lst.append((i, float(np.float32(1.0 - total))))
        rows.append(lst)
    return rows


def random_rows(n, rng, lo, hi):
    """Row-stochastic, lo..hi entries per row, list order shuffled; arbitrary positive weights while
    a call takes them (512 entries), else one value per row."""
    rows = []
    for i in range(n):
        k = int(rng.integers(lo, hi + 1))
        others = rng.permutation([j for j in range(n) if j != i])[:k - 1]
        cols = rng.permutation(np.concatenate([[i], others]))
        w = rng.random(k) + 0.05 if n * hi <= 512 else np.ones(k)
        w = (w / w.sum()).astype(np.float32)
        rows.append([(int(j), float(v)) for j, v in zip(cols, w)])
    return rows


def exactly(n, rng, per_row):
    return random_rows(n, rng, per_row, per_row)


def switch(n):
    """Entries per row from which the library multiplies instead of gathering."""
    return 46 - n if n <= 32 else (152 - n + 3) // 4


def pair(P, oracle, n, phases):
    otopo = oracle.custom_topology(n, phases)
    return P.make_topology(n, otopo.row_ptr, otopo.col_idx, otopo.w, otopo.period), otopo


GRAPHS = {
    "all_to_all": lambda n, rng: [all_to_all(n, rng)],
    "metropolis": lambda n, rng: [metropolis_dense(n, rng)],
    "metropolis_90": lambda n, rng: [metropolis_dense(n, rng, 0.9)],
    "random_rows": lambda n, rng: [random_rows(n, rng, switch(n), 16 if n <= 32 else n)],   # 31, 32 nodes: at most 512 entries, direct encoding
    "at_switch": lambda n, rng: [exactly(n, rng, switch(n))],
    "below_switch": lambda n, rng: [exactly(n, rng, switch(n) - 1)],           # gathers, for comparison
    "two_phases": lambda n, rng: [metropolis_dense(n, rng), all_to_all(n, rng)],
}

CASES = [
    # graph, n, d, pad, off
    ("all_to_all", 32, 1030, 2, 0),
    ("all_to_all", 23, 515, 1, 0),      # the smallest graph that multiplies
    ("all_to_all", 24, 256, 0, 0),
    ("all_to_all", 20, 300, 0, 0),      # gathers
    ("metropolis", 32, 2051, 1, 3),     # head + body + tail: the peeled columns gather, the body multiplies
    ("metropolis", 31, 777, 3, 0),
    ("metropolis", 28, 1024, 0, 0),
    ("random_rows", 32, 1500, 0, 0),
    ("random_rows", 31, 300, 4, 4),
    ("at_switch", 32, 1100, 0, 0),
    ("at_switch", 27, 5, 3, 0),         # less than one lane group of columns
    ("at_switch", 25, 700, 0, 0),
    ("below_switch", 32, 1100, 0, 0),
    ("below_switch", 26, 600, 0, 0),
    ("two_phases", 29, 900, 0, 0),
    # 33-48 nodes: three row blocks
    ("all_to_all", 48, 1030, 2, 0),     # 2304 entries: one weight per row, column bytes only
    ("all_to_all", 33, 515, 1, 0),
    ("all_to_all", 39, 300, 0, 3),      # 1521 entries: palette encoding
    ("metropolis_90", 40, 777, 3, 0),   # mixed weights, about 1450 entries
    ("random_rows", 48, 600, 0, 0),     # 26-48 entries per row, one value per row
    ("random_rows", 44, 1100, 4, 4),
    ("at_switch", 41, 700, 0, 0),
    ("below_switch", 41, 700, 0, 0),
]

METHODS = ["decentlam", "dmsgd", "dsgd", "xprev", "awc_dmsgd", "da_dmsgd", "blocked", "multi", "multi_dmsgd", "g16"]


def check(gpu, ref, what):
    err = np.abs(gpu.astype(np.float64) - ref)
    tol = 1e-5 * (1.0 + np.abs(ref))
    assert (err <= tol).all(), f"{what}: {int((err > tol).sum())} elements off, first at {np.argwhere(err > tol)[0]}"


@pytest.mark.parametrize("method", METHODS)
@pytest.mark.parametrize("graph,n,d,pad,off", CASES)
def test_dense_graphs_match_oracle(P, oracle, method, graph, n, d, pad, off):
    rng = np.random.default_rng(97 * n + d)
    topo, otopo = pair(P, oracle, n, GRAPHS[graph](n, rng))
    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    x0, m0, g0 = (rng.standard_normal((n, d)).astype(np.float32) for _ in range(3))
    ld = d + pad + off
    bufs = [torch.full((n, ld), SENT, device="cuda") for _ in range(3)]
    x, m, g = (b[:, off:off + d] for b in bufs)
    for k in range(otopo.period + 1):
        what = f"{method} {graph} n={n} d={d} k={k}"
        for view, a in ((x, x0), (m, m0), (g, g0)):
            view.copy_(torch.from_numpy(a).cuda())
        if method in oracle.STEP:
            getattr(P, method + "_step")(x, m, g, topo, gamma, beta, k)
            xr, mr = oracle.STEP[method](x0, m0, g0, otopo, gamma, beta, k)
        elif method == "dsgd":
            P.dsgd_step(x, g, topo, gamma, k)
            xr, mr = oracle.dsgd_step(x0, g0, otopo, gamma, k), m0.astype(np.float64)
        elif method == "xprev":
            P.decentlam_step_xprev(x, m, g, topo, gamma, beta, k)
            xr, mr = x0.astype(np.float64), oracle.decentlam_xprev_step(x0, m0, g0, otopo, gamma, beta, k)
        elif method in ("multi", "multi_dmsgd"):   # per-tensor sums of squares ride along
            base = "decentlam" if method == "multi" else "dmsgd"
            T = 5
            offsets = np.concatenate([[0], np.sort(rng.integers(0, d + 1, size=T - 1)), [d]]).astype(np.int64) + off
            norms = torch.full((T, n, 3), -1.0, dtype=torch.float64, device="cuda")
            ws = torch.empty(P.decentlam_step_multi_workspace(n, d, T) + 256, dtype=torch.uint8, device="cuda")
            ws = ws[(-ws.data_ptr()) % 256:]
            getattr(P, base + "_step_multi")(bufs[0], bufs[1], bufs[2], offsets, topo, gamma, beta, k, norms=norms,
                                             workspace=ws)
            xr, mr = oracle.STEP[base](x0, m0, g0, otopo, gamma, beta, k)
            want = oracle.tensor_sumsq(g0, mr.astype(np.float32), xr.astype(np.float32), offsets - off)
            np.testing.assert_allclose(norms.cpu().numpy(), want, rtol=3e-6, atol=1e-30, err_msg=what)
        elif method == "g16":
            g16 = torch.from_numpy(g0).cuda().to(torch.bfloat16)
            gbuf = torch.zeros((n, ld), dtype=torch.bfloat16, device="cuda")
            gv = gbuf[:, off:off + d]
            gv.copy_(g16)
            P.decentlam_step_g16(x, m, gv, topo, gamma, beta, k)
            bits = g16.view(torch.int16).cpu().numpy().view(np.uint16)
            xr, mr = oracle.STEP["decentlam"](x0, m0, oracle.widen16(bits, "bf16"), otopo, gamma, beta, k)
        else:
            xb, mb, gb = (P.to_blocked(torch.from_numpy(a).cuda(), 512) for a in (x0, m0, g0))
            P.decentlam_step_blocked(xb, mb, gb, d, topo, gamma, beta, k)
            xr, mr = oracle.STEP["decentlam"](x0, m0, g0, otopo, gamma, beta, k)
            x.copy_(P.from_blocked(xb, d))
            m.copy_(P.from_blocked(mb, d))
        torch.cuda.synchronize()
        check(x.cpu().numpy(), xr, what + ": x")
        check(m.cpu().numpy(), mr, what + ": m")
        for b in bufs:
            full = b.cpu().numpy()
            assert np.all(full[:, :off] == SENT) and np.all(full[:, off + d:] == SENT), what + ": padding written"


def test_dense_run_follows_oracle_over_200_iterations(P, oracle):
    """All-to-all averaging of 32 nodes for 200 iterations of DecentLaM with gradients of a fixed
    quadratic: relative error of the iterate at the end within 1e-4."""
    n, d, steps = 32, 700, 200
    rng = np.random.default_rng(32)
    topo, otopo = pair(P, oracle, n, [metropolis_dense(n, rng, 0.8)])
    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    x0 = rng.standard_normal((n, d)).astype(np.float32)
    target = rng.standard_normal((n, d)).astype(np.float32)
    x, m = torch.from_numpy(x0).cuda(), torch.zeros((n, d), device="cuda")
    tgt = torch.from_numpy(target).cuda()
    ref = {}
    oracle.run("decentlam", x0, lambda k, xs: (xs.astype(np.float32) - target), otopo, gamma, beta, steps,
               storage="fp32", record=lambda k, xs, ms: ref.__setitem__("x", xs.copy()))
    for k in range(steps):
        g = x - tgt
        P.decentlam_step(x, m, g, topo, gamma, beta, k)
    torch.cuda.synchronize()
    got = x.cpu().numpy().astype(np.float64)
    rel = np.linalg.norm(got - ref["x"]) / np.linalg.norm(ref["x"])
    assert rel <= 1e-4, rel


def test_dense_headline_width_sampled_columns(P, oracle):
    """n = 32, all-to-all, d large enough for split tiles: sampled columns against the oracle."""
    n, d = 32, (1 << 20) + 16384 * 3 + 700
    rng = np.random.default_rng(5)
    topo, otopo = pair(P, oracle, n, [all_to_all(n, rng)])
    gamma, beta = float(np.float32(0.1)), float(np.float32(0.9))
    gen = torch.Generator(device="cuda").manual_seed(9)
    x, m, g = (P.empty_rows(n, d) for _ in range(3))
    for a in (x, m, g):
        a.copy_(torch.randn((n, d), generator=gen, device="cuda"))
    cols = np.unique(np.concatenate([rng.integers(0, d, 3000), np.arange(0, 600), np.arange(d - 900, d),
                                     np.arange(8192 - 200, 8192 + 200), np.arange((1 << 20) - 300, (1 << 20) + 300)]))
    pick = torch.from_numpy(cols).cuda()
    x0, m0, g0 = (a[:, pick].cpu().numpy() for a in (x, m, g))
    for method in ("decentlam", "dmsgd"):
        xs, ms = x.clone(), m.clone()
        xv, mv = P.empty_rows(n, d), P.empty_rows(n, d)
        xv.copy_(xs)
        mv.copy_(ms)
        getattr(P, method + "_step")(xv, mv, g, topo, gamma, beta, 0)
        torch.cuda.synchronize()
        xr, mr = oracle.STEP[method](x0, m0, g0, otopo, gamma, beta, 0)
        check(xv[:, pick].cpu().numpy(), xr, method + ": x")
        check(mv[:, pick].cpu().numpy(), mr, method + ": m")
