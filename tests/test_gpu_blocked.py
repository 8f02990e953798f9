"""GPU parity of the blocked-layout calls: against the oracle element by element, and bit for bit
against the row-major calls on the same values (the arithmetic per element is the same)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from test_gpu_parity import P, check_elementwise, dev, topo_pair  # noqa: E402,F401

SENT = 777.0


def blocked_buffer(P, a, bw, off):
    """Blocked copy of the logical n x d array `a` inside a flat buffer whose base is `off` elements
    past an aligned address; sentinel in the padding of the last block."""
    n, d = a.shape
    nb = (d + bw - 1) // bw
    flat = torch.full((nb * n * bw + off,), SENT, dtype=torch.float32, device="cuda")
    view = flat[off:].view(nb, n, bw)
    view.copy_(P.to_blocked(a, bw, fill=SENT))
    return flat, view


CASES = [
    # kind, n, d, bw, off, steps
    (1, 32, 20000, 8192, 0, 3),     # two full blocks + a narrower one
    (1, 32, 16384, 8192, 0, 2),     # exactly two blocks
    (0, 16, 5000, 8192, 0, 3),      # less than one block: the ordinary row-major path with ld = bw
    (0, 4, 4096, 256, 0, 4),        # one tile per block
    (2, 8, 1000, 64, 0, 5),         # blocks narrower than a tile
    (0, 16, 2051, 100, 0, 3),       # bw not a multiple of 4: element-wise accesses
    (1, 32, 3000, 1024, 3, 2),      # misaligned base: head + body + tail in every block
    (2, 64, 1500, 512, 0, 6),       # 8-byte accesses
    (0, 100, 700, 128, 0, 2),       # 4-byte accesses
    (4, 12, 999, 320, 1, 3),
    (0, 3, 7, 1, 0, 2),             # one column per block
    (1, 256, 300, 64, 0, 2),        # exponential graph on 256 nodes: 2304 entries, one weight per row
    (1, 24, 2100, 1024, 0, 2),      # twelve waves of two rows
    # launches of 4096 tiles and more on 33-40 and 49-56 nodes: the kernel that uses its LDS tile twice per tile
    (1, 40, (1 << 20) + 3 * 2048 + 100, 2048, 0, 2),    # 515 blocks of 8 tiles + a narrow last block; 10 waves x 4 rows
    (0, 36, (1 << 20) + 8192, 8192, 0, 2),              # 129 blocks of 32 tiles; 12 waves x 3 rows
    (4, 56, (1 << 20) + 512, 1024, 0, 2),               # irregular degrees; 14 waves x 4 rows; half a block at the end
    (1, 40, (1 << 20) + 2048, 2048, 4, 1),              # base 16 bytes past an aligned address: still served
    (1, 40, (1 << 20) + 2048, 2048, 1, 1),              # misaligned base: not served, the ordinary kernel
]


@pytest.mark.parametrize("algo", ["decentlam", "dmsgd"])
@pytest.mark.parametrize("kind,n,d,bw,off,steps", CASES)
def test_blocked_step_matches_oracle_and_row_major_call(P, oracle, algo, kind, n, d, bw, off, steps):
    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    topo, otopo = topo_pair(P, oracle, kind, n)
    rng = np.random.default_rng(31 * n + d + bw)
    x0 = rng.standard_normal((n, d)).astype(np.float32)
    grads = [rng.standard_normal((n, d)).astype(np.float32) for _ in range(steps)]
    bufs = [blocked_buffer(P, dev(a), bw, off) for a in (x0, np.zeros_like(x0), grads[0])]
    (fx, x), (fm, m), (fg, g) = bufs
    xr, mr = dev(x0), torch.zeros((n, d), dtype=torch.float32, device="cuda")
    ref = []
    oracle.run(algo, x0, lambda k, _x: grads[k], otopo, gamma, beta, steps, storage="fp32",
               record=lambda k, xs, ms: ref.append((xs.copy(), ms.copy())))
    for k in range(steps):
        g.copy_(P.to_blocked(dev(grads[k]), bw, fill=SENT))
        getattr(P, algo + "_step_blocked")(x, m, g, d, topo, gamma, beta, k)
        getattr(P, algo + "_step")(xr, mr, dev(grads[k]), topo, gamma, beta, k)
        torch.cuda.synchronize()
        xl, ml = P.from_blocked(x, d), P.from_blocked(m, d)
        check_elementwise(xl.cpu().numpy(), ref[k][0], f"x after iteration {k}")
        check_elementwise(ml.cpu().numpy(), ref[k][1], f"m after iteration {k}")
        assert torch.equal(xl, xr) and torch.equal(ml, mr)
    nb = x.shape[0]
    if d < nb * bw:                                                  # padding of the last block untouched
        for t in (x, m):
            assert bool((t[-1, :, d - (nb - 1) * bw:] == SENT).all())
    for f in (fx, fm, fg):
        assert bool((f[:off] == SENT).all())


def test_blocked_argument_errors(P):
    n, bw = 4, 64
    topo = P.topology_build(P.DL_TOPO_RING, n)
    x = torch.zeros((3, n, bw), device="cuda")
    m, g = torch.zeros_like(x), torch.zeros_like(x)
    with pytest.raises(P.DecentLamError) as e:
        P.decentlam_step_blocked(x, m, g, 3 * bw + 1, topo, 0.1, 0.9, 0)      # d beyond the blocks
    assert e.value.status == P.DL_EINVAL
    with pytest.raises(P.DecentLamError) as e:
        P.decentlam_step_blocked(x, m, g, 2 * bw, topo, 0.1, 0.9, 0)          # d ends before the last block
    assert e.value.status == P.DL_EINVAL
    with pytest.raises(P.DecentLamError) as e:
        P.decentlam_step_blocked(x, x, g, 3 * bw, topo, 0.1, 0.9, 0)
    assert e.value.status == P.DL_EALIAS
    P.decentlam_step_blocked(x, m, g, 3 * bw - 5, topo, 0.1, 0.9, 0)
    torch.cuda.synchronize()


@pytest.mark.parametrize("algo", ["decentlam", "dmsgd"])
def test_blocked_layout_at_the_headline_size(P, oracle, algo):
    """n = 32, d = 25.6 M, bw = 8192 (3125 blocks of 1 MiB per array), the benchmark's blocked
    configuration: sampled columns against the oracle over all 20 iterations."""
    import workloads
    from test_gpu_fullsize import sample_columns

    w = workloads.get("c3_exp32")
    d, n, bw = w.d, w.n, 8192
    assert d % bw == 0
    nb = d // bw
    topo, otopo = P.topology_build(1, n), oracle.topology(1, n)
    gamma, beta = float(np.float32(w.gamma)), float(np.float32(w.beta))
    cols = sample_columns(d, seed=9, blocks=32)
    flat_index = torch.from_numpy((cols // bw) * (n * bw) + cols % bw).cuda()        # offset of (row 0, c)
    rows = torch.arange(n, device="cuda").view(n, 1) * bw

    def sample(t):                                                     # logical [n, len(cols)] from a blocked tensor
        return t.view(-1)[flat_index.view(1, -1) + rows].cpu().numpy().astype(np.float64)

    gen = torch.Generator(device="cuda").manual_seed(2104)
    x = torch.empty((nb, n, bw), dtype=torch.float32, device="cuda").normal_(generator=gen)
    m = torch.zeros_like(x)
    g = torch.empty_like(x)
    xs, ms = sample(x), np.zeros((n, len(cols)))
    for k in range(w.steps):
        g.normal_(generator=gen)
        gs = sample(g)
        getattr(P, algo + "_step_blocked")(x, m, g, d, topo, gamma, beta, k)
        xs, ms = oracle.STEP[algo](xs, ms, gs, otopo, gamma, beta, k)
        xs, ms = xs.astype(np.float32).astype(np.float64), ms.astype(np.float32).astype(np.float64)
        check_elementwise(sample(x), xs, f"x, iteration {k}")
        check_elementwise(sample(m), ms, f"m, iteration {k}")
