"""GPU parity of the general step calls (`*_step_ex`): every combination of layout (row-major,
blocked) and gradient format (fp32, bf16, fp16) for DecentLaM, DmSGD, the momentum-free DecentLaM,
AWC-DmSGD and DA-DmSGD, against the oracle; and bit for bit against the special-case calls where one exists."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from test_gpu_parity import P, check_elementwise, dev, topo_pair  # noqa: E402,F401

DT = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}


def make_grad(oracle, rng, n, d, fmt):
    """(device tensor in the given format, float64 values the oracle uses)."""
    g32 = rng.standard_normal((n, d)).astype(np.float32)
    if fmt == "f32":
        return torch.from_numpy(g32).cuda(), g32.astype(np.float64)
    t = torch.from_numpy(g32).to(DT[fmt])
    bits = t.view(torch.int16).numpy().view(np.uint16)
    return t.cuda(), oracle.widen16(bits, fmt)


CASES = [
    # kind, n, d, bw (0 = row-major), steps
    (1, 32, 5000, 0, 3),
    (1, 32, 20000, 8192, 3),
    (0, 16, 2051, 256, 3),
    (2, 8, 1000, 64, 6),
    (3, 64, 700, 512, 2),
    (0, 100, 333, 128, 2),
    (4, 12, 515, 0, 3),
]


@pytest.mark.parametrize("fmt", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("algo", ["decentlam", "dmsgd", "decentlam_xprev", "awc_dmsgd", "da_dmsgd"])
@pytest.mark.parametrize("kind,n,d,bw,steps", CASES)
def test_general_step_matches_oracle(P, oracle, fmt, algo, kind, n, d, bw, steps):
    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    topo, otopo = topo_pair(P, oracle, kind, n)
    rng = np.random.default_rng(17 * n + d + bw)
    x0 = rng.standard_normal((n, d)).astype(np.float32)
    lay = (lambda t: P.to_blocked(t, bw)) if bw else (lambda t: t.clone())
    unlay = (lambda t: P.from_blocked(t, d)) if bw else (lambda t: t)
    x = lay(dev(x0))
    second = lay(dev(x0)) if algo == "decentlam_xprev" else torch.zeros_like(x)       # x^{-1} = x^0, or m^0 = 0
    xs, ss = x0.astype(np.float64), (x0.astype(np.float64) if algo == "decentlam_xprev" else np.zeros((n, d)))
    r32 = lambda a: a.astype(np.float32).astype(np.float64)
    for k in range(steps):
        gd, gv = make_grad(oracle, rng, n, d, fmt)
        g = lay(gd)
        kw = dict(d=d) if bw else {}
        if algo == "decentlam_xprev":
            P.decentlam_step_xprev_ex(x, second, g, topo, gamma, beta, k, **kw)
            xn = r32(oracle.decentlam_xprev_step(xs, ss, gv, otopo, gamma, beta, k))
            check_elementwise(unlay(second).cpu().numpy(), xn, f"x after iteration {k}")
            x, second = second, x
            xs, ss = xn, xs
        else:
            getattr(P, algo + "_step_ex")(x, second, g, topo, gamma, beta, k, **kw)
            xs, ss = (r32(a) for a in oracle.STEP[algo](xs, ss, gv, otopo, gamma, beta, k))
            check_elementwise(unlay(x).cpu().numpy(), xs, f"x after iteration {k}")
            check_elementwise(unlay(second).cpu().numpy(), ss, f"m after iteration {k}")


def test_general_forms_reproduce_the_special_cases(P):
    n, d, bw = 32, 20000, 8192
    topo = P.topology_build(P.DL_TOPO_EXP_STATIC, n)
    gen = torch.Generator(device="cuda").manual_seed(4)
    x0 = torch.randn((n, d), device="cuda", generator=gen)
    g = torch.randn((n, d), device="cuda", generator=gen)
    g16 = g.to(torch.bfloat16)
    # row-major fp32
    xa, ma, xb, mb = x0.clone(), torch.zeros_like(x0), x0.clone(), torch.zeros_like(x0)
    P.decentlam_step(xa, ma, g, topo, 0.1, 0.9, 0)
    P.decentlam_step_ex(xb, mb, g, topo, 0.1, 0.9, 0)
    assert torch.equal(xa, xb) and torch.equal(ma, mb)
    # row-major bf16
    xa, ma, xb, mb = x0.clone(), torch.zeros_like(x0), x0.clone(), torch.zeros_like(x0)
    P.dmsgd_step_g16(xa, ma, g16, topo, 0.1, 0.9, 0)
    P.dmsgd_step_ex(xb, mb, g16, topo, 0.1, 0.9, 0)
    assert torch.equal(xa, xb) and torch.equal(ma, mb)
    # blocked fp32
    xa, ma = P.to_blocked(x0, bw), P.to_blocked(torch.zeros_like(x0), bw)
    xb, mb = xa.clone(), ma.clone()
    gb = P.to_blocked(g, bw)
    P.decentlam_step_blocked(xa, ma, gb, d, topo, 0.1, 0.9, 0)
    P.decentlam_step_ex(xb, mb, gb, topo, 0.1, 0.9, 0, d=d)
    assert torch.equal(xa, xb) and torch.equal(ma, mb)
    # momentum-free, row-major fp32
    ca, pa, cb, pb = x0.clone(), x0.clone(), x0.clone(), x0.clone()
    P.decentlam_step_xprev(ca, pa, g, topo, 0.1, 0.9, 0, gamma_prev=0.05)
    P.decentlam_step_xprev_ex(cb, pb, g, topo, 0.1, 0.9, 0, gamma_prev=0.05)
    assert torch.equal(pa, pb)
    torch.cuda.synchronize()


def test_leanest_iteration_at_the_headline_size(P, oracle):
    """n = 32, d = 25.6 M, blocked layout, bf16 gradients, momentum-free form (14 B per node-element):
    sampled columns against the oracle over several iterations."""
    import workloads
    from test_gpu_fullsize import sample_columns

    w = workloads.get("c3_exp32")
    d, n, bw = w.d, w.n, 8192
    nb = d // bw
    topo, otopo = P.topology_build(1, n), oracle.topology(1, n)
    gamma, beta = float(np.float32(w.gamma)), float(np.float32(w.beta))
    cols = sample_columns(d, seed=3, blocks=24)
    flat = (torch.from_numpy((cols // bw) * (n * bw) + cols % bw).cuda().view(1, -1)
            + torch.arange(n, device="cuda").view(n, 1) * bw)
    gen = torch.Generator(device="cuda").manual_seed(14)
    cur = torch.empty((nb, n, bw), dtype=torch.float32, device="cuda").normal_(generator=gen)
    prev = cur.clone()
    g32 = torch.empty_like(cur)
    g = torch.empty((nb, n, bw), dtype=torch.bfloat16, device="cuda")
    xc = cur.view(-1)[flat].cpu().numpy().astype(np.float64)
    xp = xc.copy()
    for k in range(5):
        g32.normal_(generator=gen)
        g.copy_(g32)
        bits = g.view(-1)[flat].cpu().view(torch.int16).numpy().view(np.uint16)
        P.decentlam_step_xprev_ex(cur, prev, g, topo, gamma, beta, k, d=d)
        xn = oracle.decentlam_xprev_step(xc, xp, oracle.widen16(bits, "bf16"), otopo, gamma, beta, k)
        xn = xn.astype(np.float32).astype(np.float64)
        check_elementwise(prev.view(-1)[flat].cpu().numpy(), xn, f"x, iteration {k}")
        cur, prev = prev, cur
        xc, xp = xn, xc


def test_multi_tensor_and_general_calls_are_capturable_in_a_hip_graph(P):
    """decentlam_step_multi with per-tensor sums (tile records + final pass, the tensor table passed
    as kernel arguments) and the general call in the blocked layout with bf16 gradients only enqueue
    kernels: captured once, replayed five times, each replay compared with eager execution.  n = 32
    uses more than 48 KiB of LDS per workgroup, so the capture also covers the launch path that raises
    the kernel's dynamic LDS limit."""
    n, bw = 32, 256
    topo = P.topology_build(P.DL_TOPO_RING, n)
    sizes = [300, 1, 0, 63, 64, 65, 2000, 2, 700]
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    d, T = int(offsets[-1]), len(sizes)
    gen = torch.Generator(device="cuda").manual_seed(8)
    x0 = torch.randn((n, d), device="cuda", generator=gen)
    g = torch.randn((n, d), device="cuda", generator=gen)
    xb0, gb = P.to_blocked(x0, bw), P.to_blocked(g, bw).to(torch.bfloat16)
    ws = torch.empty(P.decentlam_step_multi_workspace(n, d, T), dtype=torch.uint8, device="cuda")

    def work(x, m, norms, cur, prev):
        for k in range(2):
            P.decentlam_step_multi(x, m, g, offsets, topo, 0.05, 0.9, k, norms=norms, workspace=ws)
        P.decentlam_step_xprev_ex(cur, prev, gb, topo, 0.05, 0.9, 0, d=d)
        P.decentlam_step_xprev_ex(prev, cur, gb, topo, 0.05, 0.9, 1, d=d)

    def fresh():
        return (x0.clone(), torch.zeros_like(x0), torch.zeros((T, n, 3), dtype=torch.float64, device="cuda"),
                xb0.clone(), xb0.clone())

    eager_state = fresh()
    eager = []
    for _ in range(5):
        work(*eager_state)
        eager.append([t.clone() for t in eager_state])
    state = fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        work(*state)                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    for t, f in zip(state, fresh()):
        t.copy_(f)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        work(*state)
    for t, f in zip(state, fresh()):
        t.copy_(f)
    scratch = torch.zeros(1000, device="cuda")
    for r in range(5):
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(state, eager[r]):
            assert torch.equal(got, want), f"replay {r} differs from eager"
        scratch.add_(1.0)
        torch.cuda.synchronize()


MULTI_EX_CASES = [
    # n, bw (0 = row-major), tensor sizes
    (16, 256, [300, 1, 0, 63, 64, 65, 700, 2, 2, 2, 500, 0, 1097]),     # ends inside a block
    (32, 512, [1] * 40 + [600] + [5] * 30 + [1024 - 790]),              # exactly two blocks
    (64, 256, [517, 100, 100, 51]),                                     # 128-column tiles
    (100, 256, [64, 64, 1, 200, 500]),                                  # 64-column tiles
    (16, 8192, [3000, 5000, 10000, 7]),                                 # two full blocks + a rest with a tail
    (16, 0, [300, 1, 0, 63, 64, 65, 700]),                              # row-major through the general call
]


@pytest.mark.parametrize("fmt", ["f32", "bf16"])
@pytest.mark.parametrize("algo", ["decentlam", "dmsgd", "awc_dmsgd", "da_dmsgd"])
@pytest.mark.parametrize("n,bw,sizes", MULTI_EX_CASES)
def test_general_multi_tensor_call_matches_oracle(P, oracle, fmt, algo, n, bw, sizes):
    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    topo, otopo = topo_pair(P, oracle, 0, n)
    rng = np.random.default_rng(7 * n + bw + len(sizes))
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    d, T = int(offsets[-1]), len(sizes)
    x0 = rng.standard_normal((n, d)).astype(np.float32)
    lay = (lambda t: P.to_blocked(t, bw)) if bw else (lambda t: t.clone())
    unlay = (lambda t: P.from_blocked(t, d)) if bw else (lambda t: t)
    x, m = lay(dev(x0)), lay(torch.zeros((n, d), dtype=torch.float32, device="cuda"))
    norms = torch.full((T, n, 3), -1.0, dtype=torch.float64, device="cuda")
    ws = torch.empty(P.decentlam_step_multi_workspace(n, d, T), dtype=torch.uint8, device="cuda")
    xs, ms = x0.astype(np.float64), np.zeros((n, d))
    r32 = lambda a: a.astype(np.float32).astype(np.float64)
    for k in range(3):
        gd, gv = make_grad(oracle, rng, n, d, fmt)
        getattr(P, algo + "_step_multi_ex")(x, m, lay(gd), offsets, topo, gamma, beta, k, norms=norms, workspace=ws)
        xs, ms = (r32(a) for a in oracle.STEP[algo](xs, ms, gv, otopo, gamma, beta, k))
        xg, mg = unlay(x).cpu().numpy(), unlay(m).cpu().numpy()
        check_elementwise(xg, xs, f"x after iteration {k}")
        check_elementwise(mg, ms, f"m after iteration {k}")
        got = norms.cpu().numpy()
        want = oracle.tensor_sumsq(gv, ms, xs, offsets)
        np.testing.assert_allclose(got, want, rtol=2e-6, atol=1e-30)
        np.testing.assert_allclose(got[:, :, 0], want[:, :, 0], rtol=1e-13, atol=0)
        own = oracle.tensor_sumsq(gv, mg, xg, offsets)              # plain sums of what the call stored
        np.testing.assert_allclose(got, own, rtol=1e-13, atol=0)


def test_blocked_multi_tensor_requirements(P):
    n = 4
    topo = P.topology_build(P.DL_TOPO_RING, n)
    x = torch.zeros((2, n, 100), device="cuda")                         # bw not a multiple of 256
    m, g = torch.zeros_like(x), torch.zeros_like(x)
    norms = torch.zeros((1, n, 3), dtype=torch.float64, device="cuda")
    ws = torch.empty(P.decentlam_step_multi_workspace(n, 200, 1), dtype=torch.uint8, device="cuda")
    with pytest.raises(P.DecentLamError) as e:
        P.decentlam_step_multi_ex(x, m, g, [0, 200], topo, 0.1, 0.9, 0, norms=norms, workspace=ws)
    assert e.value.status == P.DL_EINVAL and "256" in str(e.value)
    P.decentlam_step_multi_ex(x, m, g, [0, 200], topo, 0.1, 0.9, 0)     # without sums any width works
    with pytest.raises(P.DecentLamError) as e:
        P.decentlam_step_multi_ex(x, m, g, [5, 200], topo, 0.1, 0.9, 0)
    assert e.value.status == P.DL_EINVAL
    torch.cuda.synchronize()
