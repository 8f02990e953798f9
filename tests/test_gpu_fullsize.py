"""GPU parity at the full workload sizes, in the launch configuration the benchmark times.

The arrays only ever exist in HBM (torch's seeded device generator fills them).
Columns of the update are independent, so the oracle recomputes a sample of
columns exactly: the sampled columns of x0 and of every gradient are copied to
the host and the oracle runs its own free trajectory on them.
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


def check_elementwise(gpu, ref, what):
    err = np.abs(gpu.astype(np.float64) - ref)
    tol = 1e-5 * (1.0 + np.abs(ref))
    assert (err <= tol).all(), f"{what}: worst err/tol {(err / tol).max():.3f}"


def sample_columns(d, seed, block=64, blocks=48, edge=1024):
    rng = np.random.default_rng(seed)
    cols = [np.arange(0, min(edge, d)), np.arange(max(0, d - edge), d)]
    for s in rng.integers(0, max(1, d - block), size=blocks):
        cols.append(np.arange(s, s + block))
    # the seams of the large-launch column order: around multiples of 8192 and 16384 columns, and
    # where the last whole 64 KiB unit ends and ordinary tiles take over
    last_unit = d // 16384 * 16384
    for s in (8192, 16384, 3 * 8192, (d // 2) // 16384 * 16384 + 8192, last_unit - 8192, last_unit):
        if 128 <= s <= d - 128:
            cols.append(np.arange(s - 128, s + 128))
    return np.unique(np.concatenate(cols))


def run_sampled_trajectory(P, oracle, w, algo, kind, stepper=None, ld=None):
    import workloads

    d = workloads.generate.dim(w)
    topo = P.topology_build(kind, w.n)
    otopo = oracle.topology(kind, w.n)
    gamma, beta = float(np.float32(w.gamma)), float(np.float32(w.beta))
    cols = sample_columns(d, seed=w.cfg)
    cols_t = torch.from_numpy(cols).cuda()
    xb = workloads.device_x0(w, "cuda", ld=ld)
    mb = torch.zeros_like(xb)
    gb = torch.zeros_like(xb)
    x, m, g = xb[:, :d], mb[:, :d], gb[:, :d]
    xs = x.index_select(1, cols_t).cpu().numpy().astype(np.float64)
    ms = np.zeros_like(xs)
    fn = getattr(P, algo + "_step")
    for k in range(w.steps):
        workloads.device_grad(w, k, gb)
        gs = g.index_select(1, cols_t).cpu().numpy().astype(np.float64)
        if stepper is None:
            fn(x, m, g, topo, gamma, beta, k)
        else:
            stepper(fn, x, m, g, topo, gamma, beta, k)
        xs, ms = oracle.STEP[algo](xs, ms, gs, otopo, gamma, beta, k)
        xs = xs.astype(np.float32).astype(np.float64)   # fp32 storage between iterations
        ms = ms.astype(np.float32).astype(np.float64)
        check_elementwise(x.index_select(1, cols_t).cpu().numpy(), xs, f"{w.name} {algo} x, iteration {k}")
        check_elementwise(m.index_select(1, cols_t).cpu().numpy(), ms, f"{w.name} {algo} m, iteration {k}")
    assert torch.isfinite(x).all() and torch.isfinite(m).all()
    return x, m


@pytest.mark.parametrize("padded", [True, False], ids=["ld_64KiB", "ld_d"])
@pytest.mark.parametrize("algo", ["decentlam", "dmsgd"])
def test_workload3_n32_d25_6M_sampled_columns(P, oracle, algo, padded):
    """The headline configuration: n = 32, static exponential graph, d = 25.6 M, 20 iterations, with the
    row stride the benchmark uses (rows on 64 KiB boundaries) and with ld = d."""
    import workloads

    w = workloads.get("c3_exp32")
    d = workloads.generate.dim(w)
    run_sampled_trajectory(P, oracle, w, algo, 1, ld=P.recommended_ld(d) if padded else d)


@pytest.mark.parametrize("n", [48, 64, 128])
def test_headline_size_at_other_node_counts_sampled_columns(P, oracle, n):
    """The benchmark's side measurement `decentlam_step_by_node_count`: 819.2 M node-elements on n nodes, static
    exponential graph, rows on 64 KiB boundaries (empty_rows): from 33 nodes on these launches take the kernel
    that uses its LDS tile twice per 256 columns.  Five iterations, the oracle on sampled columns incl. the seams."""
    d = 32 * 25_600_000 // n
    topo = P.topology_build(P.DL_TOPO_EXP_STATIC, n)
    otopo = oracle.topology(1, n)
    gamma, beta = float(np.float32(0.01)), float(np.float32(0.9))
    gen = torch.Generator(device="cuda").manual_seed(1000 + n)
    x, m, g = (P.empty_rows(n, d) for _ in range(3))
    x.normal_(generator=gen)
    m.zero_()
    cols = sample_columns(d, seed=n)
    cols_t = torch.from_numpy(cols).cuda()
    xs = x.index_select(1, cols_t).cpu().numpy().astype(np.float64)
    ms = np.zeros_like(xs)
    for k in range(5):
        g.normal_(generator=gen)
        gs = g.index_select(1, cols_t).cpu().numpy().astype(np.float64)
        P.decentlam_step(x, m, g, topo, gamma, beta, k)
        xs, ms = oracle.STEP["decentlam"](xs, ms, gs, otopo, gamma, beta, k)
        xs = xs.astype(np.float32).astype(np.float64)
        ms = ms.astype(np.float32).astype(np.float64)
        check_elementwise(x.index_select(1, cols_t).cpu().numpy(), xs, f"n = {n}: x, iteration {k}")
        check_elementwise(m.index_select(1, cols_t).cpu().numpy(), ms, f"n = {n}: m, iteration {k}")
    assert torch.isfinite(x).all() and torch.isfinite(m).all()


def test_workload4_ragged_flat_and_ranged_calls(P, oracle):
    """n = 16 ring over 160 packed tensors (sizes not multiples of 4): one flat call per iteration
    against the oracle on sampled columns; then the same run as 160 per-tensor ranged calls
    (pointer offset, same row stride) must agree with the flat run bit for bit."""
    import workloads

    w = workloads.get("c4_ring16_ragged")
    sizes, offsets, _ = workloads.ragged_layout(w)
    assert len(sizes) == 160 and (sizes % 4 != 0).any()
    x_flat, m_flat = run_sampled_trajectory(P, oracle, w, "decentlam", 0)

    def ranged(fn, x, m, g, topo, gamma, beta, k):
        for t in range(len(sizes)):
            a, b = int(offsets[t]), int(offsets[t + 1])
            fn(x[:, a:b], m[:, a:b], g[:, a:b], topo, gamma, beta, k)

    x_rng, m_rng = run_sampled_trajectory(P, oracle, w, "decentlam", 0, stepper=ranged)
    assert torch.equal(x_flat, x_rng) and torch.equal(m_flat, m_rng)
    # the benchmark's layout: rows padded to a multiple of 64 elements (256-byte aligned rows)
    d = int(offsets[-1])
    x_pad, m_pad = run_sampled_trajectory(P, oracle, w, "decentlam", 0, ld=(d + 63) // 64 * 64)
    assert torch.equal(x_flat, x_pad) and torch.equal(m_flat, m_pad)


def test_workload5_lsq_gradient_then_step(P, oracle):
    """n = 64, A_i 4096 x 4096: local_grad_lsq feeds decentlam_step.  The gradient couples all
    columns of a node, so there is no column sampling here: the oracle runs its own first
    iterations over all nodes, and each checked GPU iteration starts from the oracle's state
    (uploaded), as in the 200-step test of the small least-squares workload.  Then the GPU runs
    all 50 iterations freely."""
    import workloads

    w = workloads.get("c5_onepeer64_lsq")
    A, y, _ = workloads.device_lsq_problem(w, "cuda")
    A0, y0 = A.cpu().numpy(), y.cpu().numpy()
    topo = P.topology_build(w.topo, w.n)
    otopo = oracle.topology(w.topo, w.n)
    gamma, beta, scale = (float(np.float32(v)) for v in (w.gamma, w.beta, w.lsq_scale))
    g = torch.empty((w.n, w.d), dtype=torch.float32, device="cuda")
    loss = torch.empty(w.n, dtype=torch.float32, device="cuda")
    ws = torch.empty(P.local_grad_lsq_workspace(w.n, w.b, w.d), dtype=torch.uint8, device="cuda")
    to_dev = lambda a: torch.from_numpy(a.astype(np.float32)).cuda()
    r32 = lambda a: a.astype(np.float32).astype(np.float64)

    xs = np.zeros((w.n, w.d))
    ms = np.zeros_like(xs)
    for k in range(3):
        x, m = to_dev(xs), to_dev(ms)
        P.local_grad_lsq(A, y, x, g, loss, scale, ws)
        P.decentlam_step(x, m, g, topo, gamma, beta, k)
        gs, ls = oracle.lsq_grad(A0, y0, xs, scale)
        check_elementwise(g.cpu().numpy(), gs, f"g, iteration {k}")
        check_elementwise(loss.cpu().numpy(), ls, f"loss, iteration {k}")
        xs, ms = oracle.decentlam_step(xs, ms, r32(gs), otopo, gamma, beta, k)
        xs, ms = r32(xs), r32(ms)
        check_elementwise(x.cpu().numpy(), xs, f"x, iteration {k}")
        check_elementwise(m.cpu().numpy(), ms, f"m, iteration {k}")

    x = torch.zeros((w.n, w.d), dtype=torch.float32, device="cuda")
    m = torch.zeros_like(x)
    losses = []
    for k in range(w.steps):
        P.local_grad_lsq(A, y, x, g, loss, scale, ws)
        P.decentlam_step(x, m, g, topo, gamma, beta, k)
        losses.append(float(loss.sum()))
    assert np.isfinite(losses).all() and bool(torch.isfinite(x).all())


def test_more_than_2_pow_31_elements_per_array(P, oracle):
    """64-bit indexing: n x d = 3 x 800 000 003 (2.4 G elements, 9.6 GB per array, odd d so that the
    body / tail split is exercised far from the origin).  Sampled columns against the oracle,
    including the very last ones."""
    n, d = 3, 800_000_003
    topo = P.topology_build(P.DL_TOPO_RING, n)
    otopo = oracle.topology(oracle.RING, n)
    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    gen = torch.Generator(device="cuda").manual_seed(31)
    x = torch.empty((n, d), dtype=torch.float32, device="cuda").normal_(generator=gen)
    m = torch.empty((n, d), dtype=torch.float32, device="cuda").normal_(generator=gen)
    g = torch.empty((n, d), dtype=torch.float32, device="cuda").normal_(generator=gen)
    cols = np.unique(np.concatenate([np.arange(0, 512), np.arange(d - 515, d),
                                     np.arange(715_827_880, 715_827_890),      # around 2^31 / 3
                                     np.arange(2**29 - 4, 2**29 + 4)]))
    ct = torch.from_numpy(cols).cuda()
    for algo in ("decentlam", "dmsgd"):
        xs, ms, gs = (t.index_select(1, ct).cpu().numpy().astype(np.float64) for t in (x, m, g))
        getattr(P, algo + "_step")(x, m, g, topo, gamma, beta, 0)
        xr, mr = oracle.STEP[algo](xs, ms, gs, otopo, gamma, beta, 0)
        check_elementwise(x.index_select(1, ct).cpu().numpy(), xr, algo + " x")
        check_elementwise(m.index_select(1, ct).cpu().numpy(), mr, algo + " m")
    out = torch.empty(5, dtype=torch.float64, device="cuda")
    ws = torch.empty(P.decentlam_stats_workspace(n, d), dtype=torch.uint8, device="cuda")
    P.decentlam_stats(x, m, None, out, ws)
    got = out.cpu().numpy()
    m2 = float((m.double() ** 2).sum())
    assert abs(got[4] - m2) <= 1e-9 * m2


def test_stats_over_more_column_blocks_than_workgroups(P, oracle):
    """decentlam_stats caps its grid (32768 workgroups of 1024 columns with 16-byte lanes); beyond that
    width every workgroup walks several blocks of columns.  2 x 40 M: against the oracle on the
    downloaded arrays."""
    n, d = 2, 40_000_000
    gen = torch.Generator(device="cuda").manual_seed(5)
    x = torch.empty((n, d), dtype=torch.float32, device="cuda").normal_(generator=gen)
    m = torch.empty((n, d), dtype=torch.float32, device="cuda").normal_(generator=gen)
    ref = torch.empty(d, dtype=torch.float32, device="cuda").normal_(generator=gen)
    out = torch.empty(5, dtype=torch.float64, device="cuda")
    ws = torch.empty(P.decentlam_stats_workspace(n, d), dtype=torch.uint8, device="cuda")
    P.decentlam_stats(x, m, ref, out, ws)
    want = oracle.stats(x.cpu().numpy(), m.cpu().numpy(), ref.cpu().numpy())
    np.testing.assert_allclose(out.cpu().numpy(), want, rtol=1e-10)


def test_workload3_bf16_gradients_sampled_columns(P, oracle):
    """n = 32, d = 25.6 M with the gradients stored as bfloat16 (decentlam_step_g16), in the
    benchmark's layout.  The oracle gets the values of the same 16-bit patterns on sampled columns."""
    import workloads

    w = workloads.get("c3_exp32")
    d = w.d
    topo, otopo = P.topology_build(1, w.n), oracle.topology(1, w.n)
    gamma, beta = float(np.float32(w.gamma)), float(np.float32(w.beta))
    cols = sample_columns(d, seed=77)
    ct = torch.from_numpy(cols).cuda()
    x = workloads.device_x0(w, "cuda")
    m = torch.zeros_like(x)
    g32 = torch.empty_like(x)
    g = torch.empty((w.n, d), dtype=torch.bfloat16, device="cuda")
    xs = x.index_select(1, ct).cpu().numpy().astype(np.float64)
    ms = np.zeros_like(xs)
    for k in range(6):
        workloads.device_grad(w, k, g32)
        g.copy_(g32)                                                    # the tensor library rounds to bf16
        bits = g.index_select(1, ct).cpu().view(torch.int16).numpy().view(np.uint16)
        P.decentlam_step_g16(x, m, g, topo, gamma, beta, k)
        xs, ms = oracle.decentlam_step(xs, ms, oracle.widen16(bits, "bf16"), otopo, gamma, beta, k)
        xs, ms = xs.astype(np.float32).astype(np.float64), ms.astype(np.float32).astype(np.float64)
        check_elementwise(x.index_select(1, ct).cpu().numpy(), xs, f"x, iteration {k}")
        check_elementwise(m.index_select(1, ct).cpu().numpy(), ms, f"m, iteration {k}")


def test_workload4_multi_tensor_call_with_norms(P, oracle):
    """The ragged workload as ONE multi-tensor call per iteration with the per-tensor sums of
    squares: the state must equal the flat call's bit for bit; the sums are checked for every
    tensor against fp64 sums of what the call stored, and for a sample of tensors (the smallest
    ones and two that straddle many tiles' worth of columns) against the oracle, which runs its own
    trajectory on exactly those tensors' columns."""
    import workloads

    w = workloads.get("c4_ring16_ragged")
    sizes, offsets, _ = workloads.ragged_layout(w)
    d, T, n = int(offsets[-1]), len(sizes), w.n
    ld = (d + 63) // 64 * 64
    topo, otopo = P.topology_build(0, n), oracle.topology(0, n)
    gamma, beta = float(np.float32(w.gamma)), float(np.float32(w.beta))
    order = np.argsort(sizes)
    sample = sorted(int(t) for t in np.concatenate([order[:10], order[T // 2:T // 2 + 2]]))
    assert sum(int(sizes[t]) for t in sample) < 400_000
    cols = np.concatenate([np.arange(offsets[t], offsets[t + 1]) for t in sample])
    rel = np.concatenate([[0], np.cumsum([sizes[t] for t in sample])])
    ct = torch.from_numpy(cols).cuda()
    x = workloads.device_x0(w, "cuda", ld=ld)
    xf = x.clone()
    m, mf = torch.zeros_like(x), torch.zeros_like(x)
    g = torch.zeros_like(x)
    norms = torch.empty((T, n, 3), dtype=torch.float64, device="cuda")
    ws = torch.empty(P.decentlam_step_multi_workspace(n, d, T) + 256, dtype=torch.uint8, device="cuda")
    ws = ws[(-ws.data_ptr()) % 256:]
    xs = x.index_select(1, ct).cpu().numpy().astype(np.float64)
    ms = np.zeros_like(xs)
    steps = 5
    for k in range(steps):
        workloads.device_grad(w, k, g)
        gs = g.index_select(1, ct).cpu().numpy().astype(np.float64)
        P.decentlam_step_multi(x, m, g, offsets, topo, gamma, beta, k, norms=norms, workspace=ws)
        P.decentlam_step(xf[:, :d], mf[:, :d], g[:, :d], topo, gamma, beta, k)
        xs, ms = oracle.decentlam_step(xs, ms, gs, otopo, gamma, beta, k)
        xs, ms = xs.astype(np.float32).astype(np.float64), ms.astype(np.float32).astype(np.float64)
    assert torch.equal(x, xf) and torch.equal(m, mf)
    got = norms.cpu().numpy()
    want = oracle.tensor_sumsq(gs, ms, xs, rel)
    np.testing.assert_allclose(got[sample], want, rtol=2e-6)
    np.testing.assert_allclose(got[sample][:, :, 0], want[:, :, 0], rtol=1e-13)
    csum = lambda a: torch.cat([torch.zeros((n, 1), dtype=torch.float64, device="cuda"),
                                torch.cumsum(a[:, :d].double() ** 2, dim=1)], dim=1)
    idx = torch.from_numpy(offsets).cuda()
    for q, a in enumerate((g, m, x)):
        c = csum(a)
        own = (c[:, idx[1:]] - c[:, idx[:-1]]).T.cpu().numpy()          # [T, n], differences of a running sum
        np.testing.assert_allclose(got[:, :, q], own, rtol=1e-7, atol=1e-6)
        del c
