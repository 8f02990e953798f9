"""GPU parity of the mixed-precision and multi-tensor step calls against the CPU oracle.

16-bit gradients: both sides receive the same 16-bit patterns; the oracle works on their values
(computed field by field, pinned on the CPU against every pattern).  Multi-tensor calls: the update
is checked like a flat call, the per-tensor sums of squares against the oracle's plain sums over the
oracle's own new state.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from test_gpu_parity import P, check_elementwise, dev, topo_pair  # noqa: E402,F401

FORMATS = {"bf16": torch.bfloat16, "f16": torch.float16}


def round16(a32, fmt):
    """fp32 array -> (uint16 patterns, torch 16-bit CPU tensor); rounding done by the tensor library."""
    t = torch.from_numpy(a32).to(FORMATS[fmt])
    return t.view(torch.int16).numpy().view(np.uint16).copy(), t


G16_CASES = [
    # kind, n, d, pad x/m, pad g, offset x/m, offset g, steps
    (0, 4, 4096, 0, 0, 0, 0, 4),
    (1, 32, 1030, 2, 2, 0, 0, 3),      # 16-byte x/m accesses, 8-byte g accesses, ragged tail
    (1, 32, 1029, 3, 7, 0, 0, 2),      # both strides multiples of 4 with different paddings
    (0, 16, 2051, 1, 1, 3, 3, 3),      # same misalignment everywhere: head + body + tail
    (0, 16, 1000, 0, 0, 1, 2, 2),      # g misaligned differently from x: narrower accesses
    (2, 64, 517, 3, 1, 0, 0, 6),       # n = 64: 8-byte x/m, 4-byte g accesses
    (0, 100, 333, 0, 1, 0, 1, 2),      # n > 64: element-wise accesses, odd g stride
    (3, 64, 300, 0, 0, 0, 0, 2),       # palette-encoded weights
    (2, 8, 3, 0, 0, 0, 0, 3),
    (4, 12, 515, 1, 1, 0, 0, 3),
]


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
@pytest.mark.parametrize("algo", ["decentlam", "dmsgd"])
@pytest.mark.parametrize("kind,n,d,pad,padg,off,offg,steps", G16_CASES)
def test_g16_step_matches_oracle_every_iteration(P, oracle, fmt, algo, kind, n, d, pad, padg, off, offg, steps):
    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    topo, otopo = topo_pair(P, oracle, kind, n)
    rng = np.random.default_rng(77 * n + d)
    x0 = rng.standard_normal((n, d)).astype(np.float32)
    bits, tens, vals = [], [], []
    for _ in range(steps):
        b, t = round16(rng.standard_normal((n, d)).astype(np.float32), fmt)
        bits.append(b)
        tens.append(t)
        vals.append(oracle.widen16(b, fmt))
    ld, ldg = d + pad + off, d + padg + offg
    SENT = 12345.0
    bx, bm = (torch.full((n, ld), SENT, dtype=torch.float32, device="cuda") for _ in range(2))
    bg = torch.full((n, ldg), 7.0, dtype=FORMATS[fmt], device="cuda")
    x, m, g = bx[:, off:off + d], bm[:, off:off + d], bg[:, offg:offg + d]
    x.copy_(dev(x0))
    m.zero_()
    ref = []
    oracle.run(algo, x0, lambda k, _x: vals[k], otopo, gamma, beta, steps, storage="fp32",
               record=lambda k, xs, ms: ref.append((xs.copy(), ms.copy())))
    fn = getattr(P, algo + "_step_g16")
    for k in range(steps):
        g.copy_(tens[k].cuda())
        fn(x, m, g, topo, gamma, beta, k)
        torch.cuda.synchronize()
        check_elementwise(x.cpu().numpy(), ref[k][0], f"x after iteration {k}")
        check_elementwise(m.cpu().numpy(), ref[k][1], f"m after iteration {k}")
        np.testing.assert_array_equal(g.cpu().view(torch.int16).numpy().view(np.uint16), bits[k])
    for b in (bx, bm):
        full = b.cpu().numpy()
        assert np.all(full[:, :off] == SENT) and np.all(full[:, off + d:] == SENT)
    gfull = bg.cpu().float().numpy()
    assert np.all(gfull[:, :offg] == 7.0) and np.all(gfull[:, offg + d:] == 7.0)


def test_g16_with_fp32_format_is_the_plain_step(P):
    """DL_GRAD_F32 through the g16 entry point (g with its own stride) gives decentlam_step's bits."""
    n, d = 32, 3000
    topo = P.topology_build(P.DL_TOPO_EXP_STATIC, n)
    gen = torch.Generator(device="cuda").manual_seed(3)
    x0 = torch.randn((n, d), device="cuda", generator=gen)
    g = torch.randn((n, d + 8), device="cuda", generator=gen)[:, :d]
    xa, ma, xb, mb = x0.clone(), torch.zeros_like(x0), x0.clone(), torch.zeros_like(x0)
    for k in range(3):
        P.decentlam_step(xa, ma, g.contiguous(), topo, 0.1, 0.9, k)
        P.decentlam_step_g16(xb, mb, g, topo, 0.1, 0.9, k)
    torch.cuda.synchronize()
    assert torch.equal(xa, xb) and torch.equal(ma, mb)


def ragged_offsets(rng, start, sizes):
    return np.concatenate([[start], start + np.cumsum(sizes)]).astype(np.int64)


MULTI_CASES = [
    # kind, n, start column, tensor sizes, trailing columns
    (0, 16, 0, [300, 1, 0, 63, 64, 65, 5000, 2, 2, 2, 700, 0, 4097], 0),
    (0, 16, 5, [7, 250, 1024, 3, 3, 3, 1000], 9),          # misaligned start, untouched columns on both sides
    (1, 32, 2, [1] * 40 + [600] + [5] * 30, 1),            # many tensors inside one tile
    (2, 64, 0, [517, 100, 100], 0),                        # 8-byte accesses, 128-column tiles
    (0, 100, 3, [64, 64, 1, 200], 0),                      # 4-byte accesses, 64-column tiles
    (0, 4, 0, [10000], 0),                                 # one tensor, many tiles
    (0, 4, 0, [0, 0, 3, 0], 0),
    # beyond 2^20 columns: split tiles (two 128-column segments 8192 columns apart per tile), records per half tile
    (0, 4, 0, [300000, 5, 700000, 128, 127, 129, 8192, 16384, 40000, 65539], 0),
    (0, 4, 4, [300000, 5, 700000, 128, 127, 129, 8192, 16384, 40000, 65539], 3),   # 16 bytes past the start: a shorter launch first
    (1, 32, 0, [1 << 20, 1000, 70000], 0),                                         # two rows per thread
    (0, 4, 0, [(7 * t) % 23 for t in range(1000)], 0),     # more tensors than one final-pass launch takes (440): three launches
]


@pytest.mark.parametrize("fmt", ["f32", "bf16"])
@pytest.mark.parametrize("algo", ["decentlam", "dmsgd"])
@pytest.mark.parametrize("kind,n,start,sizes,trail", MULTI_CASES)
def test_multi_tensor_step_and_norms_match_oracle(P, oracle, fmt, algo, kind, n, start, sizes, trail):
    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    topo, otopo = topo_pair(P, oracle, kind, n)
    rng = np.random.default_rng(len(sizes) * 131 + n)
    offsets = ragged_offsets(rng, start, sizes)
    lo, hi = int(offsets[0]), int(offsets[-1])
    d, cols = hi - lo, hi + trail
    steps = 3
    x0 = rng.standard_normal((n, d)).astype(np.float32)
    grads, gdev = [], []
    for _ in range(steps):
        g32 = rng.standard_normal((n, d)).astype(np.float32)
        if fmt == "f32":
            grads.append(g32)
            gdev.append(torch.from_numpy(g32))
        else:
            b, t = round16(g32, fmt)
            grads.append(oracle.widen16(b, fmt))
            gdev.append(t)
    SENT = 4321.0
    x = torch.full((n, cols), SENT, dtype=torch.float32, device="cuda")
    m = torch.full((n, cols), SENT, dtype=torch.float32, device="cuda")
    g = torch.full((n, cols), 3.0, dtype=gdev[0].dtype, device="cuda")
    x[:, lo:hi] = dev(x0)
    m[:, lo:hi] = 0
    T = len(sizes)
    norms = torch.full((T, n, 3), -1.0, dtype=torch.float64, device="cuda")
    ws = torch.empty(P.decentlam_step_multi_workspace(n, d, T) + 256, dtype=torch.uint8, device="cuda")
    ws = ws[(-ws.data_ptr()) % 256:]
    ref = []
    oracle.run(algo, x0, lambda k, _x: grads[k], otopo, gamma, beta, steps, storage="fp32",
               record=lambda k, xs, ms: ref.append((xs.copy(), ms.copy())))
    fn = getattr(P, algo + "_step_multi")
    rel = offsets - lo
    for k in range(steps):
        g[:, lo:hi] = gdev[k].cuda()
        fn(x, m, g, offsets, topo, gamma, beta, k, norms=norms, workspace=ws)
        torch.cuda.synchronize()
        xg, mg = x[:, lo:hi].cpu().numpy(), m[:, lo:hi].cpu().numpy()
        check_elementwise(xg, ref[k][0], f"x after iteration {k}")
        check_elementwise(mg, ref[k][1], f"m after iteration {k}")
        got = norms.cpu().numpy()
        want = oracle.tensor_sumsq(grads[k], ref[k][1].astype(np.float32), ref[k][0].astype(np.float32), rel)
        # the oracle's new state and the library's differ by fp32 rounding-boundary cases only
        np.testing.assert_allclose(got, want, rtol=2e-6, atol=1e-30)
        # g is the same on both sides; fp64 sums of N non-negative terms in two different orders differ by
        # at most N * 2^-53 relative
        order_tol = max(1e-13, max(sizes) * 2.0 ** -53)
        np.testing.assert_allclose(got[:, :, 0], want[:, :, 0], rtol=order_tol, atol=0)
        # and the sums are the sums of what the call stored (fp64 accumulation, any order)
        own = np.zeros_like(got)
        for t in range(T):
            a, b = int(rel[t]), int(rel[t + 1])
            own[t, :, 1] = (mg[:, a:b].astype(np.float64) ** 2).sum(axis=1)
            own[t, :, 2] = (xg[:, a:b].astype(np.float64) ** 2).sum(axis=1)
        np.testing.assert_allclose(got[:, :, 1:], own[:, :, 1:], rtol=order_tol, atol=0)
    for b in (x, m):
        full = b.cpu().numpy()
        assert np.all(full[:, :lo] == SENT) and np.all(full[:, hi:] == SENT)


def test_multi_tensor_norms_are_deterministic_and_optional(P):
    n = 16
    topo = P.topology_build(P.DL_TOPO_RING, n)
    rng = np.random.default_rng(9)
    sizes = np.exp(rng.uniform(np.log(1), np.log(20000), 60)).astype(np.int64)
    offsets = np.concatenate([[0], np.cumsum(sizes)])
    d, T = int(offsets[-1]), len(sizes)
    gen = torch.Generator(device="cuda").manual_seed(5)
    x0 = torch.randn((n, d), device="cuda", generator=gen)
    g = torch.randn((n, d), device="cuda", generator=gen)
    ws = torch.empty(P.decentlam_step_multi_workspace(n, d, T) + 256, dtype=torch.uint8, device="cuda")
    ws = ws[(-ws.data_ptr()) % 256:]
    outs = []
    for rep in range(3):
        x, m = x0.clone(), torch.zeros_like(x0)
        norms = torch.full((T, n, 3), float(rep), dtype=torch.float64, device="cuda")   # stale contents are cleared
        for k in range(2):
            P.decentlam_step_multi(x, m, g, offsets, topo, 0.1, 0.9, k, norms=norms, workspace=ws)
        outs.append((x, m, norms))
    xf, mf = x0.clone(), torch.zeros_like(x0)
    xn, mn = x0.clone(), torch.zeros_like(x0)
    for k in range(2):
        P.decentlam_step(xf, mf, g, topo, 0.1, 0.9, k)
        P.decentlam_step_multi(xn, mn, g, offsets, topo, 0.1, 0.9, k)      # no norms: no workspace needed
    torch.cuda.synchronize()
    for x, m, norms in outs:
        assert torch.equal(x, xf) and torch.equal(m, mf)                   # the update is the flat call's, bit for bit
        assert torch.equal(norms, outs[0][2])
    assert torch.equal(xn, xf) and torch.equal(mn, mf)


def test_multi_tensor_argument_errors(P):
    n, d = 4, 100
    topo = P.topology_build(P.DL_TOPO_RING, n)
    x = torch.zeros((n, d), device="cuda")
    m, g = torch.zeros_like(x), torch.zeros_like(x)
    norms = torch.zeros((2, n, 3), dtype=torch.float64, device="cuda")
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(P.DecentLamError) as e:
        P.decentlam_step_multi(x, m, g, [0, 50, 100], topo, 0.1, 0.9, 0, norms=norms, workspace=small[(-small.data_ptr()) % 256:])
    assert e.value.status == P.DL_ECAP
    with pytest.raises(P.DecentLamError) as e:
        P.decentlam_step_multi(x, m, g, [0, 60, 50], topo, 0.1, 0.9, 0)
    assert e.value.status == P.DL_EINVAL
    with pytest.raises(P.DecentLamError) as e:
        P.decentlam_step_multi(x, m, g, [0, 60, 101], topo, 0.1, 0.9, 0)
    assert e.value.status == P.DL_EINVAL
