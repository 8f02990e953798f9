"""GPU parity of the large-launch column orders of the row-major step.

From 2^16 columns on, a row-major launch with 16-byte lanes maps its tiles to two 512-byte segments
32 KiB apart inside 64 KiB-aligned units of the written array (what precedes the first aligned column
is a launch of its own, what follows the last whole unit rides along as ordinary tiles).  Every
column must still be updated exactly once: a column left out keeps its old value, a column taken
twice gets the update twice, and either fails the comparison with the oracle, which is made on every
element.  Bases are placed at chosen distances from a 64 KiB boundary so that all three parts occur.
Row strides that are not a multiple of 32 elements take the other large-launch order (tiles handed out
XCD by XCD), checked the same way, also with the per-tensor sums riding along.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

UNIT = 16384   # columns per 64 KiB


@pytest.fixture(scope="module")
def P():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2104_11981_amd as pkg

    return pkg


def check_elementwise(gpu, ref, what):
    err = np.abs(gpu.astype(np.float64) - ref)
    tol = 1e-5 * (1.0 + np.abs(ref))
    bad = err > tol
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} elements outside 1e-5*(1+|ref|), first at {np.argwhere(bad)[0]}"


def placed(n, d, ld, skew, fill):
    """n x d view with row stride ld whose first element lies `skew` elements past a 64 KiB boundary."""
    buf = torch.full((n * ld + 2 * UNIT,), fill, dtype=torch.float32, device="cuda")
    first = (-(buf.data_ptr() // 4)) % UNIT + skew
    return buf, buf[first:first + n * ld].view(n, ld)[:, :d]


CASES = [
    # kind, n, d, ld - d, skew of x, m, g (elements past a 64 KiB boundary)
    (0, 4, (1 << 20) + 2 * UNIT + 300, 0, (0, 0, 0)),               # aligned; ld not a multiple of a unit
    (0, 4, (1 << 20) + 5 * UNIT, 3 * UNIT, (0, 0, 0)),              # whole units only, aligned rows
    (1, 32, (1 << 20) + 77 * 4, 8188 - 77 * 4 + 4, (4, 4, 4)),      # 16 bytes past the boundary: a launch of 16380 columns first
    (0, 16, (1 << 20) + UNIT + 1031, 1, (9000, 9000, 9000)),        # odd stride: narrow lanes, no split tiles at all
    (2, 8, (1 << 20) + 3 * UNIT + 8, 8, (8, 4, 12)),                # arrays placed differently (the written x decides)
    (1, 32, (1 << 20) + 40, UNIT - 40, (3, 3, 3)),                  # three elements off 16-byte alignment: head columns, then the rest
    # rows that start at different offsets inside a 128-byte line (ld not a multiple of 32): one piece per
    # row and tile, every XCD's workgroups on a contiguous share of the tiles; tile counts 8q + 2, + 6, + 0, + 7
    (0, 4, (1 << 20) + 260, 4, (0, 0, 0)),
    (2, 8, (1 << 20) + 1284, 4, (0, 0, 0)),
    (0, 4, (1 << 20) + 1796, 12, (0, 4, 8)),
    (1, 16, (1 << 20) + 1540, 20, (4, 4, 4)),
    # the shortest launches that take these orders (65536 columns), and one just below
    (1, 32, (1 << 16) + UNIT + 300, UNIT - 300, (4, 4, 4)),
    (0, 8, 1 << 16, 0, (0, 0, 0)),
    (1, 16, (1 << 16) + 260, 4, (0, 0, 0)),
    (1, 32, (1 << 16) - 4, 4, (0, 0, 0)),
    (1, 24, (1 << 16) + 8192, 0, (0, 0, 0)),                        # rows alternating between boundaries and midpoints, too short for chained tiles
]


@pytest.mark.parametrize("algo", ["decentlam", "dmsgd", "dsgd", "xprev", "awc_dmsgd"])
@pytest.mark.parametrize("kind,n,d,pad,skew", CASES)
def test_large_row_major_launch_matches_oracle(P, oracle, algo, kind, n, d, pad, skew):
    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    topo = P.topology_build(kind, n)
    otopo = oracle.topology(kind, n)
    rng = np.random.default_rng(n * 7 + d)
    x0, m0, g0 = (rng.standard_normal((n, d)).astype(np.float32) for _ in range(3))
    ld = d + pad
    SENT = 4242.0
    (bx, x), (bm, m), (bg, g) = (placed(n, d, ld, s, SENT) for s in skew)
    for view, a in ((x, x0), (m, m0), (g, g0)):
        view.copy_(torch.from_numpy(a).cuda())
    k = 1
    if algo == "dsgd":
        P.dsgd_step(x, g, topo, gamma, k)
        xr = oracle.dsgd_step(x0, g0, otopo, gamma, k)
        mr = m0.astype(np.float64)
    elif algo == "xprev":
        # state (x^k, x^{k-1}) = (x0, m0); the result lands in the x_prev buffer, x is only read
        P.decentlam_step_xprev(x, m, g, topo, gamma, beta, k)
        mr = oracle.decentlam_xprev_step(x0, m0, g0, otopo, gamma, beta, k)
        xr = x0.astype(np.float64)
    else:
        getattr(P, algo + "_step")(x, m, g, topo, gamma, beta, k)
        xr, mr = oracle.STEP[algo](x0, m0, g0, otopo, gamma, beta, k)
    torch.cuda.synchronize()
    check_elementwise(x.cpu().numpy(), xr, algo + " x")
    check_elementwise(m.cpu().numpy(), mr, algo + " m")
    np.testing.assert_array_equal(g.cpu().numpy(), g0)
    for buf, view in ((bx, x), (bm, m), (bg, g)):   # nothing outside the views was written
        full = buf.cpu().numpy()
        inside = np.zeros(full.shape, dtype=bool)
        first = (view.data_ptr() - buf.data_ptr()) // 4
        for i in range(n):
            inside[first + i * ld:first + i * ld + d] = True
        assert np.all(full[~inside] == SENT)


# Rows that alternate between 64 KiB boundaries and their midpoints (ld an odd multiple of 8192 elements: a
# contiguous 32 x 25.6 M array is one): the whole units of a launch on 17-32 nodes go to the chained-tile
# kernel, in which the odd rows load half a wave one unit ahead and store half a wave one unit late.  A value
# loaded ahead from the wrong place, a result stored late at the wrong place, or a chain end handled wrongly
# fails the comparison, which covers every element.  Chains shorten towards the end of a launch: 64-67 units
# make chains of four, two and one unit.
CHAIN_CASES = [
    # kind, n, d, ld - d, skew of x, m, g
    (1, 32, (1 << 20) + 8192, 0, (0, 0, 0)),                          # ld = d: 64 units chained, 8192 columns after them
    (1, 32, (1 << 20) + 3 * UNIT + 8192, 0, (0, 0, 0)),               # 67 units: one chain of four, then twos and ones
    (0, 21, (1 << 20) + 3 * UNIT + 400, 8192 - 400, (260, 260, 260)), # off the boundary alike: 16124 columns first
    (3, 31, (1 << 20) + 2 * UNIT + 12, 8192 - 12 + UNIT, (0, 0, 0)),  # odd node count: the last wave holds one row
    (1, 17, (1 << 20) + 8192, 0, (8192, 8192, 8192)),                 # all bases half a unit off: half a unit first
    (1, 32, (1 << 20) + 8192, 0, (0, 8192, 0)),                       # m placed differently: not served, split tiles
    (4, 24, (1 << 20) + 8192, 0, (0, 0, 0)),                          # irregular degrees (mesh)
]


@pytest.mark.parametrize("algo", ["decentlam", "dmsgd", "awc_dmsgd", "xprev"])
@pytest.mark.parametrize("kind,n,d,pad,skew", CHAIN_CASES)
def test_rows_alternating_between_boundaries_and_midpoints(P, oracle, algo, kind, n, d, pad, skew):
    assert (d + pad) % UNIT == UNIT // 2
    test_large_row_major_launch_matches_oracle(P, oracle, algo, kind, n, d, pad, skew)


# 33-128 nodes with rows on 64 KiB boundaries: the whole units of a large launch go to the kernel that uses its LDS
# tile twice per tile of 256 columns (columns 0-1 of every lane, then 2-3); what precedes the first boundary of the
# written array and what follows the last whole unit are launches of the ordinary kernel.  A result of the first pass
# lost while it waits in registers, a second pass that reads the first pass's tile, or a seam between the launches
# fails the comparison, which covers every element.
ALL_TALL = ("decentlam", "dmsgd", "dsgd", "xprev", "awc_dmsgd")
TALL_CASES = [
    # kind, n, d, ld - d, skew of x, m, g, methods
    (0, 128, (1 << 20) + UNIT + 300, UNIT - 300, (0, 0, 0), ALL_TALL),    # eight rows per thread; 300 columns after the units
    (1, 96, (1 << 20) + 2 * UNIT, 0, (4, 4, 4), ALL_TALL),                # six rows per thread; 16380 columns before the units
    (3, 72, (1 << 20) + UNIT + 12, UNIT - 12, (0, 8192, 4096), ("decentlam", "xprev")),   # m, g placed differently; five rows per thread, 72-79 absent
    (4, 100, (1 << 20) + 200, UNIT - 200, (3, 3, 3), ("decentlam", "dmsgd")),   # irregular degrees; seven rows per thread; off 16-byte alignment alike
    (1, 65, (1 << 20) + 4, UNIT - 4, (0, 0, 0), ("dmsgd", "awc_dmsgd")),   # the smallest node count served
    (0, 128, (1 << 20) + 8, UNIT - 8, (1, 2, 3), ("decentlam",)),         # misaligned differently: not served, narrow lanes
    # 33-64 nodes: the same kernel with three or four rows per thread, two workgroups per CU
    (1, 64, (1 << 20) + UNIT + 300, UNIT - 300, (0, 0, 0), ALL_TALL),     # four rows per thread (AWC-DmSGD: not served there)
    (1, 48, (1 << 20) + 2 * UNIT, 0, (4, 4, 4), ALL_TALL),                # three rows per thread
    (4, 40, (1 << 20) + 200, UNIT - 200, (0, 4096, 8192), ("decentlam", "dmsgd", "awc_dmsgd")),   # 10 waves x 4 rows (AWC: 16 x 3); irregular degrees
    (0, 33, (1 << 20) + 4, UNIT - 4, (3, 3, 3), ("xprev", "awc_dmsgd")),  # the smallest node count served: 12 waves x 3 rows, rows 33-35 absent
    (2, 56, (1 << 20) + 2 * UNIT, 0, (0, 0, 0), ("decentlam", "dsgd")),   # 14 waves x 4 rows; one peer per iteration
    (1, 48, (1 << 16) + 2 * UNIT, 0, (0, 0, 0), ("decentlam", "dmsgd")),  # the shortest launch served, six units
    (1, 128, (1 << 16) + 300, UNIT - 300, (4, 4, 4), ("decentlam",)),     # four units between two ordinary launches
]


@pytest.mark.parametrize("kind,n,d,pad,skew,algo", [c[:5] + (a,) for c in TALL_CASES for a in c[5]])
def test_tall_tiles_in_two_passes(P, oracle, algo, kind, n, d, pad, skew):
    assert (d + pad) % UNIT == 0 and 32 < n <= 128
    test_large_row_major_launch_matches_oracle(P, oracle, algo, kind, n, d, pad, skew)


# Up to 64 nodes the same kernel also takes rows that start on other 512-byte boundaries (its column order is then
# relative to row 0 of the written array; the other rows' pieces are 512 bytes at some other phase of their units).
@pytest.mark.parametrize("kind,n,d,pad,skew,algo", [
    (1, 48, (1 << 20) + 8192, 0, (0, 0, 0), "decentlam"),              # ld = d, rows alternate between boundaries and midpoints
    (1, 64, (1 << 20) + 8192 + 77, 128 - 77, (4, 4, 4), "dmsgd"),      # rows 512 bytes further on each, 16380 columns first
    (0, 36, (1 << 20) + 3 * 128, 0, (0, 128, 256), "xprev"),           # m, g placed differently
])
def test_tall_tiles_on_rows_off_the_64_kib_boundaries(P, oracle, algo, kind, n, d, pad, skew):
    assert (d + pad) % 128 == 0 and (d + pad) % UNIT != 0 and 32 < n <= 64
    test_large_row_major_launch_matches_oracle(P, oracle, algo, kind, n, d, pad, skew)


# The same kernel with bf16 / fp16 gradients (8 bytes per lane, widened on load): DecentLaM, DmSGD and the
# momentum-free form.  g has its own stride and its own place; it is served when its misalignment in elements equals
# that of x and m.
@pytest.mark.parametrize("fmt,algo,kind,n,d,pad,skew,skew_g,padg", [
    ("bf16", "decentlam", 1, 40, (1 << 20) + UNIT + 300, UNIT - 300, 0, 0, 4),      # 10 waves x 4 rows; g with another stride
    ("f16", "dmsgd", 0, 64, (1 << 20) + 2 * UNIT, 0, 4, 4, 0),                      # 16380 columns first
    ("bf16", "xprev", 1, 100, (1 << 20) + 200, UNIT - 200, 0, 8, 8),                # seven rows per thread; g placed elsewhere
    ("f16", "decentlam", 4, 36, (1 << 20) + 3 * 128, 0, 0, 0, 0),                   # rows on other 512-byte boundaries
    ("bf16", "dmsgd", 1, 128, (1 << 20) + 8, UNIT - 8, 0, 2, 0),                    # g misaligned differently: not served
])
def test_tall_tiles_with_16_bit_gradients(P, oracle, fmt, algo, kind, n, d, pad, skew, skew_g, padg):
    dtype = {"bf16": torch.bfloat16, "f16": torch.float16}[fmt]
    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    topo, otopo = P.topology_build(kind, n), oracle.topology(kind, n)
    rng = np.random.default_rng(n * 13 + d)
    x0, m0 = (rng.standard_normal((n, d)).astype(np.float32) for _ in range(2))
    g16 = torch.from_numpy(rng.standard_normal((n, d)).astype(np.float32)).to(dtype)
    bits = g16.view(torch.int16).numpy().view(np.uint16).copy()
    g0 = oracle.widen16(bits, fmt)
    ld, ldg = d + pad, d + pad + padg
    SENT = 4242.0
    (bx, x), (bm, m) = (placed(n, d, ld, skew, SENT) for _ in range(2))
    bg = torch.full((n * ldg + 2 * UNIT,), 7.0, dtype=dtype, device="cuda")
    first_g = (-(bg.data_ptr() // 2)) % UNIT + skew_g
    g = bg[first_g:first_g + n * ldg].view(n, ldg)[:, :d]
    x.copy_(torch.from_numpy(x0).cuda())
    m.copy_(torch.from_numpy(m0).cuda())
    g.copy_(g16.cuda())
    k = 1
    if algo == "xprev":
        P.decentlam_step_xprev_ex(x, m, g, topo, gamma, beta, k)
        mr = oracle.decentlam_xprev_step(x0, m0, g0, otopo, gamma, beta, k)
        xr = x0.astype(np.float64)
    else:
        getattr(P, algo + "_step_g16")(x, m, g, topo, gamma, beta, k)
        xr, mr = oracle.STEP[algo](x0, m0, g0, otopo, gamma, beta, k)
    torch.cuda.synchronize()
    check_elementwise(x.cpu().numpy(), xr, algo + " x")
    check_elementwise(m.cpu().numpy(), mr, algo + " m")
    np.testing.assert_array_equal(g.cpu().view(torch.int16).numpy().view(np.uint16), bits)
    for buf, view in ((bx, x), (bm, m)):   # nothing outside the views was written
        full = buf.cpu().numpy()
        inside = np.zeros(full.shape, dtype=bool)
        first = (view.data_ptr() - buf.data_ptr()) // 4
        for i in range(n):
            inside[first + i * ld:first + i * ld + d] = True
        assert np.all(full[~inside] == SENT)


@pytest.mark.parametrize("n,d,pad", [(4, (1 << 20) + 1284, 4), (8, (1 << 20) + 3 * UNIT + 8, 8), (4, (1 << 20) + 2 * UNIT, 0)])
def test_large_launch_with_per_tensor_sums(P, oracle, n, d, pad):
    """The multi-tensor call over one large launch in either order: state and sums against the oracle."""
    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    topo, otopo = P.topology_build(0, n), oracle.topology(0, n)
    rng = np.random.default_rng(d + n)
    x0, m0, g0 = (rng.standard_normal((n, d)).astype(np.float32) for _ in range(3))
    ld = d + pad
    bufs = [torch.zeros((n, ld), device="cuda") for _ in range(3)]
    for b, a in zip(bufs, (x0, m0, g0)):
        b[:, :d].copy_(torch.from_numpy(a).cuda())
    T = 9
    offsets = np.concatenate([[0], np.sort(rng.integers(0, d + 1, size=T - 1)), [d]]).astype(np.int64)
    norms = torch.full((T, n, 3), -1.0, dtype=torch.float64, device="cuda")
    ws = torch.empty(P.decentlam_step_multi_workspace(n, d, T) + 256, dtype=torch.uint8, device="cuda")
    ws = ws[(-ws.data_ptr()) % 256:]
    P.decentlam_step_multi(bufs[0], bufs[1], bufs[2], offsets, topo, gamma, beta, 2, norms=norms, workspace=ws)
    torch.cuda.synchronize()
    xr, mr = oracle.STEP["decentlam"](x0, m0, g0, otopo, gamma, beta, 2)
    check_elementwise(bufs[0][:, :d].cpu().numpy(), xr, "x")
    check_elementwise(bufs[1][:, :d].cpu().numpy(), mr, "m")
    want = oracle.tensor_sumsq(g0, mr.astype(np.float32), xr.astype(np.float32), offsets)
    np.testing.assert_allclose(norms.cpu().numpy(), want, rtol=3e-6, atol=1e-30)



@pytest.mark.parametrize("n,d,ld", [(48, (1 << 20) + 3 * UNIT + 300, (1 << 20) + 4 * UNIT),      # two-pass kernel + ordinary launches around it
                                    (32, (1 << 20) + 8192, (1 << 20) + 8192)])                   # chained tiles + an ordinary launch
def test_large_launches_made_of_several_kernels_are_capturable(P, n, d, ld):
    """A large call on these layouts is two or three kernel launches, some of which set a function attribute first;
    all of it must be recordable into a HIP graph.  Three replays of two captured iterations against eager execution,
    with the program's own work and synchronisations between the replays."""
    topo = P.topology_build(P.DL_TOPO_EXP_STATIC, n)
    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    gen = torch.Generator(device="cuda").manual_seed(n)
    skew = 4                                                  # 16 bytes past a 64 KiB boundary: columns before the units too
    bufs = [placed(n, d, ld, skew, 0.0) for _ in range(5)]    # eager x, m; graph x, m; g
    (_, xe), (_, me), (_, xg), (_, mg), (_, g) = bufs
    x0 = torch.randn((n, d), device="cuda", generator=gen)
    g.copy_(torch.randn((n, d), device="cuda", generator=gen))

    def two_steps(x, m):
        P.decentlam_step(x, m, g, topo, gamma, beta, 0)
        P.dmsgd_step(x, m, g, topo, gamma, beta, 1)

    xe.copy_(x0)
    eager = []
    for _ in range(3):
        two_steps(xe, me)
        eager.append((xe.clone(), me.clone()))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):          # warm-up on the capture stream, then restore the state
        two_steps(xg, mg)
    torch.cuda.current_stream().wait_stream(side)
    xg.copy_(x0)
    mg.zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        two_steps(xg, mg)
    xg.copy_(x0)
    mg.zero_()
    scratch = torch.zeros(1000, device="cuda")
    for r in range(3):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(xg, eager[r][0]) and torch.equal(mg, eager[r][1]), f"replay {r} differs from eager"
        scratch.add_(1.0)
        torch.cuda.synchronize()
