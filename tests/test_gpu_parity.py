"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Both sides start from the same seeded inputs and run freely (no state ever
flows from the GPU into the oracle).  The oracle keeps fp32 storage between
iterations, as the library does in HBM, and evaluates each iteration in fp64.

Tolerances (written out here as the contract states them):
  * per element, per iteration:  |gpu - ref| <= 1e-5 * (1 + |ref|)
  * after a long run:            ||gpu - ref||_F <= 1e-4 * ||ref||_F   (x; ref = all-fp64 oracle)
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def P():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2104_11981_amd as pkg

    return pkg


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_elementwise(gpu, ref, what):
    gpu = gpu.astype(np.float64)
    err = np.abs(gpu - ref)
    tol = 1e-5 * (1.0 + np.abs(ref))
    bad = err > tol
    assert not bad.any(), (f"{what}: {bad.sum()} of {bad.size} elements outside 1e-5*(1+|ref|); "
                           f"worst err {err.max():.3e} at ref {ref.flat[err.argmax()]:.6g}")
    return float((err / tol).max())


def topo_pair(P, oracle, kind, n):
    t = P.topology_build(kind, n, seed=11, phases=5)     # seed and phases only matter to the random match
    r = oracle.topology(kind, n, seed=11, phases=5)
    assert t.period == r.period
    np.testing.assert_array_equal(t.row_ptr, r.row_ptr)
    np.testing.assert_array_equal(t.col_idx, r.col_idx)
    np.testing.assert_array_equal(t.w.view(np.uint32), r.w.view(np.uint32))
    return t, r


STEP_CASES = [
    # kind, n, d, pad (ld - d), element offset of the views (misalignment), steps, gamma
    (0, 4, 4096, 0, 0, 10, 0.1),      # workload 1
    (2, 8, 1000, 0, 0, 7, 0.01),      # one-peer, small gamma (1/gamma amplification of rounding)
    (1, 32, 1030, 2, 0, 4, 0.1),      # several tiles + ragged tail, padded rows
    (1, 32, 777, 3, 1, 3, 0.1),       # misaligned base and odd stride: narrow-load path
    (0, 16, 2051, 1, 3, 3, 0.05),     # misaligned by 3 elements, ld multiple of 4: head + body + tail
    (2, 64, 517, 3, 0, 7, 0.05),      # n = 64 uses 8-byte accesses
    (1, 64, 300, 0, 2, 2, 0.05),
    (0, 100, 333, 0, 0, 2, 0.1),      # n > 64: 4-byte accesses
    (2, 256, 130, 2, 0, 9, 0.1),      # DL_MAX_NODES, 512 entries per phase
    (0, 170, 67, 0, 0, 2, 0.1),
    (0, 256, 67, 0, 0, 2, 0.1),       # 768 entries: beyond DL_MAX_NNZ, palette encoding of the weights
    (1, 128, 70, 0, 0, 2, 0.1),       # 1024 entries
    (1, 256, 70, 0, 0, 2, 0.1),       # exponential graph at DL_MAX_NODES: 2304 entries, one weight per row, column indices only
    (3, 128, 131, 1, 0, 3, 0.1),      # symmetric exponential graph on 128 nodes: 1920 entries, the same encoding
    (1, 200, 64, 0, 0, 2, 0.1),       # 1800 entries
    (3, 64, 300, 0, 0, 3, 0.1),       # symmetric exponential graph on 64 nodes, 768 entries
    (1, 7, 129, 0, 0, 3, 0.1),        # n not a power of two
    (0, 1, 70, 0, 0, 3, 0.1),         # single node: W = [1]
    (0, 2, 5, 0, 0, 3, 0.1),          # ring degenerates to a pair
    (0, 3, 1, 0, 0, 3, 0.1),          # one column
    (1, 5, 3, 5, 0, 3, 0.1),
    (2, 8, 4, 0, 0, 4, 0.1),
    (2, 8, 255, 1, 0, 4, 0.1),
    (2, 8, 257, 3, 0, 4, 0.1),
    (0, 4, 4095, 1, 0, 2, 0.1),       # one short of / one past a whole number of tiles
    (0, 4, 4097, 3, 0, 2, 0.1),
    (3, 32, 1030, 2, 0, 4, 0.1),      # symmetric exponential graph, 10 entries per row
    (3, 12, 260, 0, 0, 3, 0.1),       # n not a power of two: hops collide and are dropped
    (4, 12, 515, 1, 0, 4, 0.05),      # 3 x 4 mesh: degrees 2-4, Metropolis-Hastings weights
    (4, 32, 700, 0, 0, 3, 0.05),      # 4 x 8 mesh
    (4, 7, 100, 0, 0, 3, 0.05),       # prime n: the mesh is a path
    (5, 16, 300, 0, 0, 8, 0.1),       # bipartite random match, a new matching every iteration (period 5)
    (5, 9, 64, 0, 0, 6, 0.1),         # odd n: one node sits out each iteration
]


@pytest.mark.parametrize("algo", ["decentlam", "dmsgd"])
@pytest.mark.parametrize("kind,n,d,pad,off,steps,gamma", STEP_CASES)
def test_step_matches_oracle_every_iteration(P, oracle, algo, kind, n, d, pad, off, steps, gamma):
    gamma, beta = float(np.float32(gamma)), float(np.float32(0.9))
    topo, otopo = topo_pair(P, oracle, kind, n)
    rng = np.random.default_rng(1000 * n + d)
    x0 = rng.standard_normal((n, d)).astype(np.float32)
    grads = [rng.standard_normal((n, d)).astype(np.float32) for _ in range(steps)]
    ld = d + pad + off
    SENT = 12345.0
    bufs = [torch.full((n, ld), SENT, dtype=torch.float32, device="cuda") for _ in range(3)]
    x, m, g = (b[:, off:off + d] for b in bufs)
    x.copy_(dev(x0))
    m.zero_()
    fn = getattr(P, algo + "_step")
    ref_states = []
    oracle.run(algo, x0, lambda k, _x: grads[k], otopo, gamma, beta, steps, storage="fp32",
               record=lambda k, xs, ms: ref_states.append((xs.copy(), ms.copy())))
    for k in range(steps):
        g.copy_(dev(grads[k]))
        fn(x, m, g, topo, gamma, beta, k)
        torch.cuda.synchronize()
        check_elementwise(x.cpu().numpy(), ref_states[k][0], f"x after iteration {k}")
        check_elementwise(m.cpu().numpy(), ref_states[k][1], f"m after iteration {k}")
        np.testing.assert_array_equal(g.cpu().numpy(), grads[k])          # g is read-only
    for b in bufs:                                                        # padding untouched
        full = b.cpu().numpy()
        assert np.all(full[:, :off] == SENT) and np.all(full[:, off + d:] == SENT)


def test_zero_columns_is_a_noop(P):
    topo = P.topology_build(0, 4)
    x = torch.zeros((4, 0), dtype=torch.float32, device="cuda")
    P.decentlam_step(x, x.clone(), x.clone(), topo, 0.1, 0.9, 0)
    P.dmsgd_step(x, x.clone(), x.clone(), topo, 0.1, 0.9, 0)
    torch.cuda.synchronize()


def test_custom_weights_and_degrees(P, oracle):
    """Irregular graph with unequal weights and degrees (general CSR path)."""
    n, d = 6, 515
    rows = [[(0, 0.5), (1, 0.25), (5, 0.25)], [(1, 0.75), (0, 0.25)], [(2, 1.0)],
            [(3, 0.125), (0, 0.125), (1, 0.25), (2, 0.25), (4, 0.125), (5, 0.125)],
            [(4, 0.5), (3, 0.5)], [(5, 0.375), (4, 0.625)]]
    otopo = oracle.custom_topology(n, [rows])
    topo = P.make_topology(n, otopo.row_ptr, otopo.col_idx, otopo.w)
    rng = np.random.default_rng(5)
    x0, m0, g0 = (rng.standard_normal((n, d)).astype(np.float32) for _ in range(3))
    for algo in ("decentlam", "dmsgd"):
        x, m, g = dev(x0), dev(m0), dev(g0)
        getattr(P, algo + "_step")(x, m, g, topo, 0.05, 0.9, 0)
        xr, mr = oracle.STEP[algo](x0, m0, g0, otopo, float(np.float32(0.05)), float(np.float32(0.9)))
        check_elementwise(x.cpu().numpy(), xr, algo + " x")
        check_elementwise(m.cpu().numpy(), mr, algo + " m")


def test_results_are_correctly_rounded_almost_everywhere(P, oracle):
    """fp64-in-register arithmetic: the stored fp32 value is the rounded oracle value except where
    a different fp64 summation order lands on the other side of a rounding boundary."""
    n, d = 32, 1 << 16
    topo, otopo = topo_pair(P, oracle, 1, n)
    rng = np.random.default_rng(6)
    x0, m0, g0 = (rng.standard_normal((n, d)).astype(np.float32) for _ in range(3))
    gamma, beta = float(np.float32(0.01)), float(np.float32(0.9))
    for algo in ("decentlam", "dmsgd"):
        x, m, g = dev(x0), dev(m0), dev(g0)
        getattr(P, algo + "_step")(x, m, g, topo, gamma, beta, 0)
        xr, mr = oracle.STEP[algo](x0, m0, g0, otopo, gamma, beta)
        for got, ref in ((x, xr), (m, mr)):
            mismatch = np.mean(got.cpu().numpy() != ref.astype(np.float32))
            assert mismatch < 1e-4, mismatch


def test_in_place_update_is_deterministic_and_resumable(P):
    """Column ownership makes the in-place update race-free: repeated runs agree bit for bit, and
    a run interrupted after T/2 iterations (state copied out and back) equals an uninterrupted one."""
    n, d, T = 32, 200_003, 6
    topo = P.topology_build(1, n)
    gen = torch.Generator(device="cuda").manual_seed(7)
    x0 = torch.randn((n, d), device="cuda", generator=gen)
    gs = [torch.randn((n, d), device="cuda", generator=gen) for _ in range(T)]

    def run(upto, x=None, m=None, start=0):
        x = x0.clone() if x is None else x
        m = torch.zeros_like(x0) if m is None else m
        for k in range(start, upto):
            P.decentlam_step(x, m, gs[k], topo, 0.1, 0.9, k)
        return x, m

    xa, ma = run(T)
    xb, mb = run(T)
    assert torch.equal(xa, xb) and torch.equal(ma, mb)
    xh, mh = run(T // 2)
    xh2, mh2 = dev(xh.cpu().numpy()), dev(mh.cpu().numpy())   # checkpoint through the host
    xc, mc = run(T, xh2, mh2, start=T // 2)
    assert torch.equal(xa, xc) and torch.equal(ma, mc)


# ---------------------------------------------------------------- least-squares gradient
LSQ_CASES = [
    # n, b, d, ldA pad, ld pad, scale
    (8, 32, 1024, 0, 0, 1.0 / 32),       # workload 2, small batch
    (8, 1024, 1024, 0, 0, 1.0 / 1024),   # workload 2, large batch
    (3, 17, 130, 2, 2, 1.0),             # ragged, aligned strides
    (2, 5, 33, 1, 3, 0.5),               # odd strides: scalar path
    (1, 1, 1, 0, 0, 1.0),
    (4, 300, 7, 0, 0, 1.0),              # tall and thin
    (4, 3, 2500, 0, 0, 1.0),             # short and wide; single sweep, 4 chunks per thread
    (2, 77, 132, 0, 4, 1.0),             # single sweep with most threads idle (d < 1024)
    (3, 1000, 1500, 4, 0, 0.001),        # single sweep, 2 chunks per thread, ragged row blocks
    (2, 45, 5000, 0, 0, 1.0),            # single sweep, 8 chunks per thread
    (1, 9, 8200, 0, 0, 1.0),             # 8192 < d <= 16384: single sweep with 1024 threads, 4 chunks each
    (2, 37, 16384, 0, 0, 0.25),          # the widest with x_i in registers
    (3, 40, 12292, 4, 0, 1.0),           # 1024 threads, last chunk of most threads past d, padded rows
    (1, 9, 16388, 0, 0, 1.0),            # 16384 < d <= 32768: single sweep, 8 chunks per thread, x_i in LDS
    (2, 20, 32768, 0, 0, 0.5),           # the widest single sweep
    (3, 33, 20484, 4, 4, 1.0),           # ... with padded rows and most of the last chunks past d
    (1, 9, 32772, 0, 0, 1.0),            # d > 32768: columns split over waves, 17 slots, the last wave with 4 columns
    (2, 40, 40000, 0, 0, 1.0),           # 20 slots, a ragged last wave, two row blocks per node
    (3, 50, 65536, 0, 0, 0.5),           # 32 slots: eight whole workgroups per row block
    (2, 33, 131072, 0, 0, 1.0),          # 64 slots: the widest
    (2, 33, 100000, 0, 0, 1.0),          # 49 slots, the last with 1696 columns
    (1, 20, 131068, 4, 0, 1.0),          # 64 slots, the last four columns short
    (2, 70, 36868, 4, 4, 1.0),           # padded rows, four row blocks of 17 or 18 rows
    (2, 30, 50000, 0, 3, 1.0),           # x and g off the 16-byte grid
    (40, 3, 131072, 0, 0, 1.0),          # more nodes than one launch holds (32 row blocks of 16 workgroups): two launches
    (1, 12, 131076, 0, 0, 1.0),          # 65 slots: two per lane from here on
    (2, 20, 200000, 0, 0, 1.0),          # 98 slots
    (1, 12, 262144, 0, 0, 1.0),          # 128 slots: the widest
    (1, 6, 262148, 0, 0, 1.0),           # beyond: two sweeps with 16-byte loads, a workgroup per row
    (1, 9, 32770, 2, 2, 1.0),            # d not a multiple of 4 above 32768: two sweeps
    (2, 7, 4099, 1, 3, 1.0),             # few long rows, odd strides: a workgroup per row, 4-byte loads
    (3, 2000, 8196, 0, 0, 1.0),          # many long rows: a wave per row
    (70, 2, 64, 0, 0, 1.0),              # more nodes than rows
    # d not a multiple of 4 with rows on 16-byte boundaries: single sweep, the last d % 4 columns element by element
    (3, 100, 1030, 2, 2, 1.0),           # two tail columns, 2 chunks per thread
    (2, 300, 4099, 1, 1, 0.5),           # three tail columns, 8 chunks per thread
    (1, 64, 8191, 1, 1, 1.0),            # the widest with 256 threads
    (4, 70, 257, 3, 3, 1.0),             # one tail column
    (1, 2000, 9, 3, 3, 1.0),             # two chunks and a tail column in all
    (2, 40, 8197, 3, 3, 1.0),            # 1024 threads: the tail sums kept in LDS by thread 0
    (2, 21, 20001, 3, 3, 1.0),           # ... with x_i in LDS as well
    (1, 12, 32767, 1, 1, 1.0),           # the widest such d
    (1, 12, 32769, 3, 3, 1.0),           # beyond: two sweeps with 4-byte loads
    # rows that are not on 16-byte boundaries: single sweep with 8-byte (even ldA) or 4-byte accesses, up to d = 16384
    (2, 300, 7850, 0, 0, 1.0),           # contiguous, even d: 8-byte accesses, 32 columns per thread
    (2, 100, 4095, 0, 0, 1.0),           # odd stride: 4-byte accesses, 16 columns per thread
    (3, 50, 1001, 0, 0, 0.5),            # 4 columns per thread, 4 rows per tile, ragged row blocks
    (2, 64, 2047, 1, 0, 1.0),            # 8-byte accesses with an odd d: thread 0 takes the last column
    (2, 40, 12290, 0, 0, 1.0),           # 1024 threads, 8-byte accesses
    (1, 30, 16383, 0, 0, 1.0),           # 1024 threads, 4-byte accesses, the widest
    (1, 30, 16385, 0, 0, 1.0),           # beyond: two sweeps
    (5, 3, 1500, 2, 1, 1.0),             # fewer rows than a tile holds
    # short rows (d <= 1024): a wave per row, or per 2, 4, 8 rows; 16-, 8- or 4-byte accesses by alignment
    (3, 1000, 8, 0, 0, 1.0),             # 16-byte accesses: 8 lanes per row (6 of them idle), 32 rows per access
    (2, 700, 32, 0, 0, 0.5),             # 8 lanes per row, all busy
    (3, 333, 64, 4, 0, 1.0),             # 16 lanes per row
    (2, 300, 100, 0, 0, 1.0),            # 32 lanes per row, 25 busy
    (2, 260, 256, 0, 4, 1.0),            # a wave per row
    (3, 77, 300, 0, 0, 1.0),             # two chunks per lane
    (2, 130, 1000, 0, 1, 1.0),           # four chunks per lane; x and g off the 16-byte grid
    (2, 600, 30, 0, 0, 1.0),             # 8-byte accesses (even ldA, even d): 16 lanes per row
    (2, 90, 1022, 0, 0, 1.0),            # 8-byte accesses, eight chunks per lane
    (2, 210, 250, 0, 0, 1.0),            # 8-byte accesses, two chunks per lane
    (2, 500, 31, 0, 0, 1.0),             # 4-byte accesses: 32 lanes per row
    (3, 400, 7, 0, 0, 1.0),              # 4-byte accesses: 8 lanes per row
    (2, 100, 129, 0, 0, 1.0),            # 4-byte accesses, four chunks per lane
    (2, 90, 1023, 0, 0, 1.0),            # 4-byte accesses, sixteen chunks per lane
    (2, 120, 514, 1, 0, 1.0),            # odd ldA with an even d: 4-byte accesses
    (1, 5000, 1, 0, 0, 1.0),             # one column
    (2, 40, 1024, 0, 0, 1.0),            # the widest short row; row blocks shorter than a workgroup's access
    # shapes between the powers of two: one chunk column more per shape
    (2, 70, 600, 0, 0, 1.0),             # a wave per row, three chunks per lane
    (2, 70, 1100, 0, 0, 1.0),            # five
    (2, 70, 1500, 4, 0, 1.0),            # six
    (3, 70, 1700, 0, 0, 1.0),            # seven
    (2, 70, 2300, 0, 0, 1.0),            # ten; the sums pass through LDS in three groups
    (2, 30, 2800, 0, 0, 1.0),            # a workgroup per row tile, three chunks per thread
    (2, 30, 2802, 2, 0, 1.0),            # the same with two tail columns
    (2, 20, 4500, 0, 0, 1.0),            # five chunks per thread
    (2, 20, 5501, 3, 0, 1.0),            # six, one tail column
    (2, 20, 6800, 0, 4, 1.0),            # seven
    (2, 16, 10000, 0, 0, 1.0),           # 1024 threads, three chunks each
    (1, 12, 10001, 3, 0, 1.0),           # the same with a tail column
    (1, 12, 24000, 0, 0, 1.0),           # x_i in LDS, six chunks per thread
    (1, 10, 26000, 0, 0, 1.0),           # seven
    (1, 10, 27002, 2, 0, 1.0),           # seven, two tail columns
    (2, 10, 18000, 0, 0, 1.0),           # five
    # the same for rows off the 16-byte boundaries
    (2, 30, 2502, 0, 0, 1.0),            # 8-byte accesses, 12 columns per thread
    (2, 30, 2999, 0, 0, 1.0),            # 4-byte accesses, 12 columns per thread
    (2, 20, 5001, 1, 0, 1.0),            # 8-byte accesses with an odd d, 20 columns per thread
    (2, 20, 6002, 0, 0, 1.0),            # 24 columns per thread
    (2, 20, 6999, 0, 0, 1.0),            # 4-byte accesses, 28 columns per thread
    (1, 16, 11001, 0, 0, 1.0),           # 1024 threads, 12 columns each
    # a wave per row up to 3072 columns off the 16-byte boundaries
    (2, 60, 1026, 0, 0, 1.0),            # 8-byte accesses, ten chunks per lane
    (2, 50, 1402, 0, 0, 1.0),            # twelve
    (2, 50, 1802, 0, 0, 1.0),            # sixteen
    (2, 40, 3002, 0, 0, 1.0),            # twenty-four
    (2, 50, 1501, 0, 0, 1.0),            # 4-byte accesses, 24 chunks per lane
    (2, 50, 2047, 0, 0, 1.0),            # 32
    (2, 40, 2301, 0, 0, 1.0),            # 40
    (2, 30, 3071, 1, 0, 1.0),            # 8-byte accesses and an odd d: 4-byte accesses, 48 chunks per lane
]


@pytest.mark.parametrize("n,b,d,padA,pad,scale", LSQ_CASES)
def test_local_grad_lsq_matches_oracle(P, oracle, n, b, d, padA, pad, scale):
    rng = np.random.default_rng(n * 100 + b)
    A0 = rng.standard_normal((n, b, d)).astype(np.float32)
    y0 = rng.standard_normal((n, b)).astype(np.float32)
    x0 = rng.standard_normal((n, d)).astype(np.float32)
    Ab = torch.full((n, b, d + padA), 7.0, dtype=torch.float32, device="cuda")
    A = Ab[:, :, :d]
    A.copy_(dev(A0))
    xb = torch.full((n, d + pad), 7.0, dtype=torch.float32, device="cuda")
    gb = torch.full((n, d + pad), 7.0, dtype=torch.float32, device="cuda")
    x, g = xb[:, :d], gb[:, :d]
    x.copy_(dev(x0))
    loss = torch.empty(n, dtype=torch.float32, device="cuda")
    ws = torch.empty(P.local_grad_lsq_workspace(n, b, d), dtype=torch.uint8, device="cuda")
    scale = float(np.float32(scale))
    P.local_grad_lsq(A, dev(y0), x, g, loss, scale, ws)
    gr, lr = oracle.lsq_grad(A0, y0, x0, scale)
    check_elementwise(g.cpu().numpy(), gr, "g")
    check_elementwise(loss.cpu().numpy(), lr, "loss")
    assert np.all(gb.cpu().numpy()[:, d:] == 7.0)
    # no loss requested, same gradient; and the result is reproducible bit for bit
    g2 = torch.zeros_like(gb)[:, :d]
    P.local_grad_lsq(A, dev(y0), x, g2, None, scale, ws)
    assert torch.equal(g2, g)


def test_wide_row_sweep_repeats_bit_for_bit_on_a_shared_workspace(P):
    """Two shapes of more than 32768 columns (both kernel shapes) take turns on one workspace, 40 calls each: the exchange
    slots of a call lie where the other shape's slots and partial sums lay a moment ago, and every call must mark its
    own slots empty before its waves read them.  Every call's result equals the first one's bit for bit."""
    shapes = ((3, 40, 65536), (2, 70, 36868))
    rng = np.random.default_rng(3)
    data, first = [], []
    need = max(P.local_grad_lsq_workspace(*s) for s in shapes)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    for n, b, d in shapes:
        A = dev(rng.standard_normal((n, b, d)).astype(np.float32))
        y = dev(rng.standard_normal((n, b)).astype(np.float32))
        x = dev(rng.standard_normal((n, d)).astype(np.float32))
        data.append((A, y, x))
    for it in range(40):
        for k, (A, y, x) in enumerate(data):
            g = torch.empty_like(x)
            loss = torch.empty(x.shape[0], dtype=torch.float32, device="cuda")
            P.local_grad_lsq(A, y, x, g, loss, 0.01, ws)
            if it == 0:
                assert bool(torch.isfinite(g).all()) and bool(torch.isfinite(loss).all())
                first.append((g, loss))
            else:
                assert torch.equal(g, first[k][0]) and torch.equal(loss, first[k][1]), f"call {it} of shape {shapes[k]}"


def test_wide_row_sweep_answers_nan_when_its_waves_stop_waiting(P, oracle):
    """Rows of more than 32768 columns: the waves of a row block hand one another their shares of each dot product and
    wait for them, a bounded number of polls.  With the limit at zero a wave that finds a share missing gives up at
    once; every kernel still runs to its end, and a launch in which any wave gave up must answer NaN for all of its
    nodes, never numbers computed from an incomplete residual.  With the limit restored the same call is right again."""
    n, b, d = 3, 64, 40000
    rng = np.random.default_rng(5)
    A0 = rng.standard_normal((n, b, d)).astype(np.float32)
    y0 = rng.standard_normal((n, b)).astype(np.float32)
    x0 = rng.standard_normal((n, d)).astype(np.float32)
    A, y, x = dev(A0), dev(y0), dev(x0)
    g = torch.zeros((n, d), dtype=torch.float32, device="cuda")
    loss = torch.zeros(n, dtype=torch.float32, device="cuda")
    ws = torch.empty(P.local_grad_lsq_workspace(n, b, d), dtype=torch.uint8, device="cuda")
    gr, lr = oracle.lsq_grad(A0, y0, x0, 1.0)
    old = P.local_grad_lsq_poll_limit(0)
    try:
        assert old == 1 << 21
        for _ in range(3):
            P.local_grad_lsq(A, y, x, g, loss, 1.0, ws)
            torch.cuda.synchronize()
            gh, lh = g.cpu().numpy(), loss.cpu().numpy()
            if np.isnan(lh).any() or np.isnan(gh).any():
                assert np.isnan(gh).all() and np.isnan(lh).all()   # one launch holds all three nodes
            else:                                                   # nobody had to wait: then the numbers are right
                check_elementwise(gh, gr, "g")
                check_elementwise(lh, lr, "loss")
    finally:
        assert P.local_grad_lsq_poll_limit(-1) == 0
    P.local_grad_lsq(A, y, x, g, loss, 1.0, ws)
    check_elementwise(g.cpu().numpy(), gr, "g")
    check_elementwise(loss.cpu().numpy(), lr, "loss")


@pytest.mark.parametrize("n,b,d,ldA,offA,offx,offg", [(2, 40, 3000, 3000, 1, 0, 0),     # 4-byte aligned A only
                                                      (2, 40, 3000, 3000, 2, 1, 3),     # 8-byte aligned A, odd x, g
                                                      (3, 25, 1021, 1024, 3, 2, 1),     # aligned stride, odd base
                                                      (2, 20, 9001, 9004, 4, 1, 2),     # aligned A, x and g are not
                                                      (1, 10, 20001, 20002, 1, 1, 1)])  # two sweeps
def test_local_grad_lsq_on_views_off_the_16_byte_grid(P, oracle, n, b, d, ldA, offA, offx, offg):
    """Any 4-byte aligned base is accepted for A, x and g; the kernels pick narrower accesses."""
    rng = np.random.default_rng(5 * d + offA)
    A0 = rng.standard_normal((n, b, d)).astype(np.float32)
    y0 = rng.standard_normal((n, b)).astype(np.float32)
    x0 = rng.standard_normal((n, d)).astype(np.float32)
    Abuf = torch.full((offA + n * b * ldA,), 7.0, dtype=torch.float32, device="cuda")
    A = Abuf[offA:].view(n, b, ldA)[:, :, :d]
    A.copy_(dev(A0))
    ld = d + 5
    xbuf = torch.full((offx + n * ld,), 7.0, dtype=torch.float32, device="cuda")
    gbuf = torch.full((offg + n * ld,), 7.0, dtype=torch.float32, device="cuda")
    x, g = xbuf[offx:].view(n, ld)[:, :d], gbuf[offg:].view(n, ld)[:, :d]
    x.copy_(dev(x0))
    loss = torch.empty(n, dtype=torch.float32, device="cuda")
    ws = torch.empty(P.local_grad_lsq_workspace(n, b, d), dtype=torch.uint8, device="cuda")
    P.local_grad_lsq(A, dev(y0), x, g, loss, 1.0, ws)
    gr, lr = oracle.lsq_grad(A0, y0, x0, 1.0)
    check_elementwise(g.cpu().numpy(), gr, "g")
    check_elementwise(loss.cpu().numpy(), lr, "loss")
    whole = gbuf.cpu().numpy()
    assert np.all(whole[:offg] == 7.0) and np.all(whole[offg:].reshape(n, ld)[:, d:] == 7.0)


@pytest.mark.parametrize("name,ring", [("c2_onepeer8_b32", False), ("c2_onepeer8_b1024", False),
                                       ("c2_onepeer8_b32", True)])
@pytest.mark.parametrize("algo", ["decentlam", "dmsgd"])
def test_workload2_trajectory_200_steps(P, oracle, name, ring, algo):
    """Least-squares workload, gradient from local_grad_lsq, 200 iterations.

    The gradient couples all coordinates of a node and gamma = 0.01 multiplies any difference in
    x by 100 on its way into m, so two fp32-storage runs that differ by one rounding somewhere
    (exact ties are common here: averaging two fp32 numbers with weights 1/2) drift apart at the
    last-bit level.  Hence two checks, one per tolerance of the contract:
      (S) every checked iteration starts from the ORACLE's state k (uploaded to the GPU) and the
          GPU's gradient and state k+1 must match the oracle's element by element;
      (F) the GPU's own free-running 200-iteration trajectory must agree with the all-fp64
          oracle trajectory to 1e-4 in relative Frobenius norm.
    On the one-peer graph DecentLaM grows geometrically (the paper requires a symmetric W for
    convergence, Sec. "Experiments"); the ring variant is the convergent counterpart."""
    import workloads

    w = workloads.get(name)
    A0, y0, _ = workloads.lsq_problem(w)
    kind = 0 if ring else w.topo
    topo, otopo = topo_pair(P, oracle, kind, w.n)
    gamma, beta, scale = (float(np.float32(v)) for v in (w.gamma, w.beta, w.lsq_scale))
    A, y = dev(A0), dev(y0)
    g = torch.empty((w.n, w.d), dtype=torch.float32, device="cuda")
    ws = torch.empty(P.local_grad_lsq_workspace(w.n, w.b, w.d), dtype=torch.uint8, device="cuda")
    fn = getattr(P, algo + "_step")

    zeros = np.zeros((w.n, w.d))
    states, grads = [(zeros, zeros)], []

    def grad_fn(k, xs):
        gk = oracle.lsq_grad(A0, y0, xs, scale)[0]
        grads.append(gk)
        return gk

    oracle.run(algo, zeros, grad_fn, otopo, gamma, beta, w.steps, storage="fp32",
               record=lambda k, xs, ms: states.append((xs.copy(), ms.copy())))
    x64, _ = oracle.run(algo, zeros, lambda k, xs: oracle.lsq_grad(A0, y0, xs, scale)[0], otopo, gamma,
                        beta, w.steps, storage="fp64")

    # (S) one GPU iteration from the oracle's state k
    for k in [0, 1, 2, 3, 4, 5] + list(range(19, w.steps, 20)):
        x, m = dev(states[k][0].astype(np.float32)), dev(states[k][1].astype(np.float32))
        P.local_grad_lsq(A, y, x, g, None, scale, ws)
        check_elementwise(g.cpu().numpy(), grads[k], f"g at iteration {k}")
        fn(x, m, g, topo, gamma, beta, k)
        check_elementwise(x.cpu().numpy(), states[k + 1][0], f"x after iteration {k}")
        check_elementwise(m.cpu().numpy(), states[k + 1][1], f"m after iteration {k}")

    # (F) free-running GPU trajectory
    x = torch.zeros((w.n, w.d), dtype=torch.float32, device="cuda")
    m = torch.zeros_like(x)
    for k in range(w.steps):
        P.local_grad_lsq(A, y, x, g, None, scale, ws)
        fn(x, m, g, topo, gamma, beta, k)
    xg = x.cpu().numpy().astype(np.float64)
    assert np.isfinite(xg).all()
    rel = np.linalg.norm(xg - x64) / np.linalg.norm(x64)
    assert rel <= 1e-4, rel
    rel32 = np.linalg.norm(xg - states[-1][0]) / np.linalg.norm(states[-1][0])
    assert rel32 <= 1e-4, rel32


# ---------------------------------------------------------------- diagnostics
@pytest.mark.parametrize("n,d,pad,off", [(8, 1000, 0, 0), (32, 4099, 1, 0), (5, 7, 0, 0), (16, 2048, 4, 1),
                                         (1, 300, 0, 0), (64, 513, 3, 0), (13, 777, 3, 0), (100, 132, 0, 0),
                                         # large states: whole 64 KiB units in the split order, plain launches
                                         # before and after them, a tail of three columns
                                         (3, 2**20 + 40003, 25, 4), (2, 2**20 + 16384, 0, 0), (2, 2**20, 28, 4)])
def test_stats_match_oracle(P, oracle, n, d, pad, off):
    rng = np.random.default_rng(n + d)
    x0 = (rng.standard_normal((n, d)) * 0.01 + rng.standard_normal(d) * 5.0).astype(np.float32)  # near consensus
    m0 = rng.standard_normal((n, d)).astype(np.float32)
    r0 = rng.standard_normal(d).astype(np.float32)
    ld = d + pad + off
    xb = torch.full((n, ld), 9.0, dtype=torch.float32, device="cuda")
    mb = torch.full((n, ld), 9.0, dtype=torch.float32, device="cuda")
    x, m = xb[:, off:off + d], mb[:, off:off + d]
    x.copy_(dev(x0))
    m.copy_(dev(m0))
    out = torch.full((5,), -1.0, dtype=torch.float64, device="cuda")
    ws = torch.empty(P.decentlam_stats_workspace(n, d), dtype=torch.uint8, device="cuda")
    P.decentlam_stats(x, m, dev(r0), out, ws)
    ref = oracle.stats(x0, m0, r0)
    np.testing.assert_allclose(out.cpu().numpy(), ref, rtol=1e-10, atol=1e-18)
    P.decentlam_stats(x, None, None, out, ws)
    got = out.cpu().numpy()
    np.testing.assert_allclose(got[:2], ref[:2], rtol=1e-10, atol=1e-18)
    assert np.all(got[2:] == 0.0)
    P.decentlam_stats(x, m, None, out, ws)             # each optional input on its own
    got = out.cpu().numpy()
    np.testing.assert_allclose(got[[0, 1, 4]], ref[[0, 1, 4]], rtol=1e-10, atol=1e-18)
    assert np.all(got[2:4] == 0.0)
    P.decentlam_stats(x, None, dev(r0), out, ws)
    got = out.cpu().numpy()
    np.testing.assert_allclose(got[:4], ref[:4], rtol=1e-10, atol=1e-18)
    assert got[4] == 0.0
    P.decentlam_stats(x, None, None, out, ws)
    out2 = torch.empty_like(out)
    P.decentlam_stats(x, None, None, out2, ws)
    assert torch.equal(out, out2)                      # fixed summation order


def test_stats_track_consensus_during_a_run(P, oracle):
    """Diagnostics on the device state of a DmSGD run on the ring: the consensus distance the
    library reports equals the oracle's on the downloaded state."""
    n, d = 16, 5000
    topo = P.topology_build(0, n)
    gen = torch.Generator(device="cuda").manual_seed(3)
    x = torch.randn((n, d), device="cuda", generator=gen)
    m = torch.zeros_like(x)
    out = torch.empty(5, dtype=torch.float64, device="cuda")
    ws = torch.empty(P.decentlam_stats_workspace(n, d), dtype=torch.uint8, device="cuda")
    seen = []
    for k in range(5):
        g = torch.randn((n, d), device="cuda", generator=gen) * 0.1
        P.dmsgd_step(x, m, g, topo, 0.05, 0.9, k)
        P.decentlam_stats(x, m, None, out, ws)
        got = out.cpu().numpy()
        ref = oracle.stats(x.cpu().numpy(), m.cpu().numpy())
        np.testing.assert_allclose(got[[0, 1, 4]], ref[[0, 1, 4]], rtol=1e-10)
        seen.append(got[0])
    assert seen[-1] < seen[0]                          # averaging contracts the disagreement


# ---------------------------------------------------------------- DSGD
@pytest.mark.parametrize("kind,n,d,pad,off", [(0, 8, 1000, 0, 0), (1, 32, 1030, 2, 0), (2, 64, 517, 3, 0),
                                              (0, 16, 2051, 1, 3), (0, 100, 333, 0, 0), (0, 1, 70, 0, 0)])
def test_dsgd_step_matches_oracle(P, oracle, kind, n, d, pad, off):
    gamma = float(np.float32(0.05))
    topo, otopo = topo_pair(P, oracle, kind, n)
    rng = np.random.default_rng(77 + n + d)
    x0 = rng.standard_normal((n, d)).astype(np.float32)
    ld = d + pad + off
    xb = torch.full((n, ld), 5.0, dtype=torch.float32, device="cuda")
    gb = torch.full((n, ld), 5.0, dtype=torch.float32, device="cuda")
    x, g = xb[:, off:off + d], gb[:, off:off + d]
    x.copy_(dev(x0))
    xs = x0.astype(np.float64)
    for k in range(4):
        gk = rng.standard_normal((n, d)).astype(np.float32)
        g.copy_(dev(gk))
        P.dsgd_step(x, g, topo, gamma, k)
        xs = oracle.dsgd_step(xs, gk, otopo, gamma, k).astype(np.float32).astype(np.float64)
        check_elementwise(x.cpu().numpy(), xs, f"x after iteration {k}")
    full = xb.cpu().numpy()
    assert np.all(full[:, :off] == 5.0) and np.all(full[:, off + d:] == 5.0)
    # beta = 0 in the momentum kernels is the same map
    xa, ma = dev(x0), torch.zeros((n, d), dtype=torch.float32, device="cuda")
    xd = dev(x0)
    P.decentlam_step(xa, ma, g.contiguous(), topo, gamma, 0.0, 0)
    P.dsgd_step(xd, g.contiguous(), topo, gamma, 0)
    check_elementwise(xa.cpu().numpy(), xd.cpu().numpy().astype(np.float64), "DecentLaM(beta=0) vs DSGD")


def test_decentlam_stays_bounded_on_symmetric_graphs(P):
    """The paper's requirement (Sec. "Experiments"): DecentLaM needs a symmetric weight matrix.  On the
    symmetric exponential graph and the mesh a long run with zero-mean gradients keeps the state
    bounded, while the directed static exponential graph of the same size lets it grow geometrically."""
    n, d, T = 32, 2048, 300
    gen = torch.Generator(device="cuda").manual_seed(21)
    x0 = torch.randn((n, d), device="cuda", generator=gen)
    gs = [torch.randn((n, d), device="cuda", generator=gen) for _ in range(8)]

    def final_norm(kind):
        topo = P.topology_build(kind, n)
        x, m = x0.clone(), torch.zeros_like(x0)
        for k in range(T):
            P.decentlam_step(x, m, gs[k % 8], topo, 0.01, 0.9, k)
        return float(x.norm())

    base = float(x0.norm())
    assert final_norm(P.DL_TOPO_EXP_SYM) < 10 * base
    assert final_norm(P.DL_TOPO_MESH) < 10 * base
    assert final_norm(P.DL_TOPO_RING) < 10 * base
    assert not final_norm(P.DL_TOPO_EXP_STATIC) < 1e6 * base      # inf or astronomically large


# ---------------------------------------------------------------- mini-batch gradient
@pytest.mark.parametrize("n,b,d,bs,pad", [(8, 1024, 1024, 64, 0), (3, 40, 132, 7, 0), (2, 50, 33, 20, 1),
                                          (4, 300, 2500, 33, 0), (2, 100, 5000, 9, 0), (1, 5, 8200, 5, 0),
                                          (5, 64, 1500, 200, 0),
                                          (2, 30, 16388, 11, 0),      # 1024 threads, x_i in LDS
                                          (3, 60, 1030, 25, 2),       # d % 4 = 2 with rows on 16-byte boundaries: tail columns
                                          (1, 20, 20001, 9, 3),       # both
                                          (2, 80, 3001, 17, 0),       # rows off the 16-byte boundaries: 4-byte accesses
                                          (3, 900, 48, 100, 0),       # short rows: 16 lanes per row, ragged row groups
                                          (2, 500, 200, 37, 0),       # a wave per row
                                          (2, 300, 30, 50, 0),        # 8-byte accesses
                                          (2, 200, 999, 13, 0),       # 4-byte accesses, sixteen chunks per lane
                                          # more than 128 sampled rows per workgroup: the look-ups wait in registers, 64 at a time
                                          (40, 700, 1100, 3000, 0),   # two chunks per thread, two rows per tile
                                          (40, 300, 4100, 2600, 4),   # eight chunks per thread, no prefetch
                                          (64, 200, 2052, 1500, 0),   # four chunks per thread
                                          (40, 500, 1030, 2000, 2),   # d not a multiple of 4
                                          (16, 150, 12292, 1200, 0),  # 1024 threads, four chunks each
                                          # rows of more than 32768 columns: the columns split over waves
                                          (2, 60, 40000, 25, 0),      # 20 slots, one row block
                                          (3, 40, 65536, 100, 4),     # more samples than rows, padded rows, six row blocks
                                          (2, 30, 70000, 20, 0),      # 35 slots of 2048 columns, the last nearly empty
                                          (1, 30, 32770, 12, 2)])     # d not a multiple of 4 up there: two sweeps
def test_local_grad_lsq_rows_matches_oracle(P, oracle, n, b, d, bs, pad):
    rng = np.random.default_rng(n * 1000 + bs)
    A0 = rng.standard_normal((n, b, d)).astype(np.float32)
    y0 = rng.standard_normal((n, b)).astype(np.float32)
    x0 = rng.standard_normal((n, d)).astype(np.float32)
    rows0 = rng.integers(0, b, size=(n, bs)).astype(np.int32)       # with replacement
    Ab = torch.zeros((n, b, d + pad), dtype=torch.float32, device="cuda")
    A = Ab[:, :, :d]
    A.copy_(dev(A0))
    x, g = dev(x0), torch.empty((n, d), dtype=torch.float32, device="cuda")
    loss = torch.empty(n, dtype=torch.float32, device="cuda")
    ws = torch.empty(P.local_grad_lsq_workspace(n, bs, d), dtype=torch.uint8, device="cuda")
    scale = float(np.float32(1.0 / bs))
    P.local_grad_lsq(A, dev(y0), x, g, loss, scale, ws, rows=dev(rows0))
    gr, lr = oracle.lsq_grad_rows(A0, y0, x0, rows0, scale)
    check_elementwise(g.cpu().numpy(), gr, "g")
    check_elementwise(loss.cpu().numpy(), lr, "loss")


# ---------------------------------------------------------------- HIP graph capture
def test_iteration_is_capturable_in_a_hip_graph(P):
    """The small least-squares workload is launch-latency bound.  All entry points only enqueue
    kernels on the caller's stream (no allocation, no synchronisation, no memset), so one period of
    the time-varying topology (gradient + step for k = 0, 1, 2) can be captured once and replayed.
    Every replay is checked against eager execution, with eager work and synchronisations in between."""
    import workloads

    w = workloads.get("c2_onepeer8_b32")
    A0, y0, _ = workloads.lsq_problem(w)
    topo = P.topology_build(w.topo, w.n)
    assert topo.period == 3
    gamma, beta, scale = (float(np.float32(v)) for v in (w.gamma, w.beta, w.lsq_scale))
    A, y = dev(A0), dev(y0)
    ws = torch.empty(P.local_grad_lsq_workspace(w.n, w.b, w.d), dtype=torch.uint8, device="cuda")

    def period(x, m, g):
        for k in range(3):
            P.local_grad_lsq(A, y, x, g, None, scale, ws)
            P.dmsgd_step(x, m, g, topo, gamma, beta, k)

    # eager reference: 5 periods, state recorded after each
    xe = torch.zeros((w.n, w.d), dtype=torch.float32, device="cuda")
    me, ge = torch.zeros_like(xe), torch.zeros_like(xe)
    eager = []
    for _ in range(5):
        period(xe, me, ge)
        eager.append((xe.clone(), me.clone()))

    xg = torch.zeros((w.n, w.d), dtype=torch.float32, device="cuda")
    mg, gg = torch.zeros_like(xg), torch.zeros_like(xg)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):          # warm-up on the capture stream, then restore the state
        period(xg, mg, gg)
    torch.cuda.current_stream().wait_stream(side)
    xg.zero_()
    mg.zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        period(xg, mg, gg)
    xg.zero_()
    mg.zero_()
    scratch = torch.zeros(1000, device="cuda")
    for r in range(5):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(xg, eager[r][0]) and torch.equal(mg, eager[r][1]), f"replay {r} differs from eager"
        scratch.add_(1.0)                  # unrelated eager work between replays
        torch.cuda.synchronize()


@pytest.mark.parametrize("d", [40000, 65536])
def test_wide_row_gradient_is_capturable(P, d):
    """Rows of more than 32768 columns: the call marks its exchange slots empty with a kernel of its own (no memset), so
    it can be captured like the others.  Four replays of a captured gradient + step, each against eager execution, with
    eager work in between: every replay has to find the slots marked empty again, not filled by the replay before it."""
    n, b = 3, 48
    topo = P.topology_build(P.DL_TOPO_RING, n)
    gamma, beta = float(np.float32(1e-5)), float(np.float32(0.8))
    gen = torch.Generator(device="cuda").manual_seed(d)
    A = torch.randn((n, b, d), device="cuda", generator=gen)
    y = torch.randn((n, b), device="cuda", generator=gen)
    x0 = torch.randn((n, d), device="cuda", generator=gen)
    ws = torch.empty(P.local_grad_lsq_workspace(n, b, d), dtype=torch.uint8, device="cuda")
    scale = float(np.float32(1.0 / b))

    def iteration(x, m, g, loss):
        P.local_grad_lsq(A, y, x, g, loss, scale, ws)
        P.decentlam_step(x, m, g, topo, gamma, beta, 0)

    xe, me, ge, le = x0.clone(), torch.zeros_like(x0), torch.zeros_like(x0), torch.zeros(n, device="cuda")
    eager = []
    for _ in range(4):
        iteration(xe, me, ge, le)
        eager.append((xe.clone(), me.clone(), le.clone()))
    assert bool(torch.isfinite(xe).all()) and not torch.equal(eager[0][0], eager[3][0])

    xg, mg, gg, lg = x0.clone(), torch.zeros_like(x0), torch.zeros_like(x0), torch.zeros(n, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        iteration(xg, mg, gg, lg)
    xg.copy_(x0)
    mg.zero_()
    scratch = torch.zeros(1000, device="cuda")
    for r in range(4):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(xg, eager[r][0]) and torch.equal(mg, eager[r][1]) and torch.equal(lg, eager[r][2]), f"replay {r}"
        scratch.add_(1.0)
        torch.cuda.synchronize()


@pytest.mark.parametrize("graph", ["exp_sym", "all_to_all"])
def test_large_lds_kernels_are_capturable(P, graph):
    """The 32-node kernels ask for more than 48 KiB of dynamic LDS, which takes a function-attribute
    call before the launch, also while a stream is being captured; the all-to-all graph takes the
    matrix-core form of the kernel.  Three replays of two captured iterations against eager execution."""
    n, d = 32, 3000
    if graph == "exp_sym":
        topo = P.topology_build(P.DL_TOPO_EXP_SYM, n)
    else:
        topo = P.make_topology(n, np.arange(0, n * n + 1, n), np.tile(np.arange(n), n), np.full(n * n, 1.0 / n, np.float32))
    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    gen = torch.Generator(device="cuda").manual_seed(77)
    x0 = torch.randn((n, d), device="cuda", generator=gen)
    g = torch.randn((n, d), device="cuda", generator=gen)

    def two_steps(x, m):
        P.decentlam_step(x, m, g, topo, gamma, beta, 0)
        P.dmsgd_step(x, m, g, topo, gamma, beta, 1)

    xe, me = x0.clone(), torch.zeros_like(x0)
    eager = []
    for _ in range(3):
        two_steps(xe, me)
        eager.append((xe.clone(), me.clone()))
    xg, mg = x0.clone(), torch.zeros_like(x0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        two_steps(xg, mg)
    torch.cuda.current_stream().wait_stream(side)
    xg.copy_(x0)
    mg.zero_()
    graph_obj = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph_obj, stream=side):
        two_steps(xg, mg)
    xg.copy_(x0)
    mg.zero_()
    scratch = torch.zeros(1000, device="cuda")
    for r in range(3):
        graph_obj.replay()
        torch.cuda.synchronize()
        assert torch.equal(xg, eager[r][0]) and torch.equal(mg, eager[r][1]), f"replay {r} differs from eager"
        scratch.add_(1.0)
        torch.cuda.synchronize()


# ---------------------------------------------------------------- momentum-free DecentLaM
@pytest.mark.parametrize("kind,n,d,pad,off,steps", [(1, 32, 1030, 2, 0, 6), (2, 8, 1000, 0, 0, 7), (0, 16, 2051, 1, 3, 4),
                                                     (3, 64, 517, 3, 0, 4), (4, 12, 515, 1, 0, 4), (0, 100, 333, 0, 0, 3),
                                                     (0, 1, 70, 0, 0, 3), (5, 16, 300, 0, 0, 6)])
def test_decentlam_xprev_matches_oracle(P, oracle, kind, n, d, pad, off, steps):
    """Buffers rotate as a caller would rotate them; a changing learning rate exercises gamma_prev."""
    beta = float(np.float32(0.9))
    topo, otopo = topo_pair(P, oracle, kind, n)
    rng = np.random.default_rng(500 + n + d)
    x0 = rng.standard_normal((n, d)).astype(np.float32)
    ld = d + pad + off
    bufs = [torch.full((n, ld), 3.0, dtype=torch.float32, device="cuda") for _ in range(3)]
    cur, prev, g = (b[:, off:off + d] for b in bufs)
    cur.copy_(dev(x0))
    prev.copy_(dev(x0))                                # x^{-1} = x^0
    xc, xp = x0.astype(np.float64), x0.astype(np.float64)
    gammas = [float(np.float32(0.05 * (1 + 0.2 * k))) for k in range(steps)]
    for k in range(steps):
        gk = rng.standard_normal((n, d)).astype(np.float32)
        g.copy_(dev(gk))
        gp = gammas[k - 1] if k else gammas[0]
        P.decentlam_step_xprev(cur, prev, g, topo, gammas[k], beta, k, gamma_prev=gp)
        xn = oracle.decentlam_xprev_step(xc, xp, gk, otopo, gammas[k], beta, k, gamma_prev=gp)
        xn = xn.astype(np.float32).astype(np.float64)
        check_elementwise(prev.cpu().numpy(), xn, f"x after iteration {k}")
        np.testing.assert_array_equal(cur.cpu().numpy(), xc.astype(np.float32))      # x^k is only read
        cur, prev = prev, cur
        xc, xp = xn, xc
    for b in bufs:
        full = b.cpu().numpy()
        assert np.all(full[:, :off] == 3.0) and np.all(full[:, off + d:] == 3.0)


def test_decentlam_xprev_tracks_decentlam_step(P):
    """Same method, two state layouts: after 30 iterations on a symmetric graph the iterates agree to fp32 noise."""
    n, d = 32, 4096
    topo = P.topology_build(P.DL_TOPO_EXP_SYM, n)
    gen = torch.Generator(device="cuda").manual_seed(9)
    x0 = torch.randn((n, d), device="cuda", generator=gen)
    xa, ma = x0.clone(), torch.zeros_like(x0)
    cur, prev = x0.clone(), x0.clone()
    for k in range(30):
        g = torch.randn((n, d), device="cuda", generator=gen)
        P.decentlam_step(xa, ma, g, topo, 0.05, 0.9, k)
        P.decentlam_step_xprev(cur, prev, g, topo, 0.05, 0.9, k)
        cur, prev = prev, cur
    rel = float((cur - xa).norm() / xa.norm())
    assert rel < 1e-5, rel


def test_global_averaging_and_many_weight_values(P, oracle):
    """W = 11^T/n with n = 32 (1024 entries, one weight value: palette encoding) turns DmSGD into
    Parallel SGD -- every node holds the same model after one iteration (Sec. "Decentralized Momentum
    SGD"); a dense 16-node W with 256 different weights goes through the direct encoding."""
    n, d = 32, 777
    rows = [[(j, 1.0 / n) for j in range(n)] for _ in range(n)]
    otopo = oracle.custom_topology(n, [rows])
    topo = P.make_topology(n, otopo.row_ptr, otopo.col_idx, otopo.w)
    rng = np.random.default_rng(8)
    x0, g0 = (rng.standard_normal((n, d)).astype(np.float32) for _ in range(2))
    x, m, g = dev(x0), torch.zeros((n, d), dtype=torch.float32, device="cuda"), dev(g0)
    P.dmsgd_step(x, m, g, topo, 0.1, 0.9, 0)
    xr, mr = oracle.dmsgd_step(x0, np.zeros_like(x0), g0, otopo, float(np.float32(0.1)), float(np.float32(0.9)))
    check_elementwise(x.cpu().numpy(), xr, "x")
    got = x.cpu().numpy()
    assert np.all(got == got[0])                      # identical rows, bit for bit (same sum order)

    n = 16
    W = rng.uniform(0.5, 1.5, size=(n, n))
    W = (W / W.sum(axis=1, keepdims=True)).astype(np.float32)
    W[:, 0] += (1.0 - W.astype(np.float64).sum(axis=1)).astype(np.float32)      # row sums 1 within 1e-6
    assert len(np.unique(W)) > 64
    rows = [[(j, float(W[i, j])) for j in range(n)] for i in range(n)]
    otopo = oracle.custom_topology(n, [rows])
    topo = P.make_topology(n, otopo.row_ptr, otopo.col_idx, otopo.w)
    x0, m0, g0 = (rng.standard_normal((n, d)).astype(np.float32) for _ in range(3))
    for algo in ("decentlam", "dmsgd"):
        x, m, g = dev(x0), dev(m0), dev(g0)
        getattr(P, algo + "_step")(x, m, g, topo, 0.05, 0.9, 0)
        xr, mr = oracle.STEP[algo](x0, m0, g0, otopo, float(np.float32(0.05)), float(np.float32(0.9)))
        check_elementwise(x.cpu().numpy(), xr, algo + " x")
        check_elementwise(m.cpu().numpy(), mr, algo + " m")


def test_per_tensor_steps_overlap_with_gradient_production(P):
    """The paper's workflow (Sec. "Improving Inconsistency Bias", "Efficient implementation": per-layer
    communication overlapped with back-propagation): gradients of the tensors of a ragged layout become
    available one tensor at a time, last layer first, on one stream; a second stream runs the ranged
    DecentLaM step of each tensor as soon as its gradient is there.  The result equals one flat call."""
    n, T = 8, 12
    rng = np.random.default_rng(17)
    sizes = rng.integers(50, 4000, size=T)
    off = np.concatenate([[0], np.cumsum(sizes)])
    d = int(off[-1])
    topo = P.topology_build(P.DL_TOPO_EXP_SYM, n)
    gen = torch.Generator(device="cuda").manual_seed(4)
    x0 = torch.randn((n, d), device="cuda", generator=gen)
    m0 = torch.randn((n, d), device="cuda", generator=gen)
    g_src = torch.randn((n, d), device="cuda", generator=gen)

    x_flat, m_flat = x0.clone(), m0.clone()
    P.decentlam_step(x_flat, m_flat, g_src, topo, 0.05, 0.9, 3)

    x, m, g = x0.clone(), m0.clone(), torch.zeros_like(g_src)
    producer, consumer = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for t in reversed(range(T)):
        a, b = int(off[t]), int(off[t + 1])
        with torch.cuda.stream(producer):
            g[:, a:b].copy_(g_src[:, a:b])              # "back-propagation" delivers this tensor's gradient
            ready = torch.cuda.Event()
            ready.record(producer)
        consumer.wait_event(ready)
        P.decentlam_step(x[:, a:b], m[:, a:b], g[:, a:b], topo, 0.05, 0.9, 3, stream=consumer.cuda_stream)
    torch.cuda.synchronize()
    assert torch.equal(x, x_flat) and torch.equal(m, m_flat)
