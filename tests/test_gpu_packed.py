"""The *_step_packed calls (W checked and encoded once by topology_pack) against their flat forms and the oracle:
same bits as the flat call at every iteration of a time-varying topology, oracle tolerance element by element."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.mark.parametrize("kind,n,d", [(2, 8, 1024), (5, 9, 777), (1, 32, 4096 + 3), (0, 4, 4096), (3, 64, 513), (1, 256, 130)])
@pytest.mark.parametrize("algo", ["decentlam", "dmsgd", "dsgd"])
def test_packed_step_equals_flat_step_and_oracle(oracle, algo, kind, n, d):
    import paper_2104_11981_amd as P

    gamma, beta = float(np.float32(0.05)), float(np.float32(0.9))
    topo = P.topology_build(kind, n, seed=7, phases=4)
    otopo = oracle.topology(kind, n, seed=7, phases=4)
    packed = P.topology_pack(topo)
    rng = np.random.default_rng(kind * 1000 + n + d)
    x0, m0 = (rng.standard_normal((n, d)).astype(np.float32) for _ in range(2))
    xa, ma = torch.from_numpy(x0).cuda(), torch.from_numpy(m0).cuda()
    xb, mb = xa.clone(), ma.clone()
    xr, mr = x0.astype(np.float64), m0.astype(np.float64)
    for k in range(2 * topo.period + 1):
        g0 = rng.standard_normal((n, d)).astype(np.float32)
        g = torch.from_numpy(g0).cuda()
        if algo == "dsgd":
            P.dsgd_step(xa, g, topo, gamma, k)
            P.dsgd_step_packed(xb, g, packed, gamma, k)
            xr = oracle.dsgd_step(xr.astype(np.float32), g0, otopo, gamma, k)
        else:
            getattr(P, algo + "_step")(xa, ma, g, topo, gamma, beta, k)
            getattr(P, algo + "_step_packed")(xb, mb, g, packed, gamma, beta, k)
            xr, mr = oracle.STEP[algo](xr.astype(np.float32), mr.astype(np.float32), g0, otopo, gamma, beta, k)
        torch.cuda.synchronize()
        assert torch.equal(xa, xb) and torch.equal(ma, mb), f"iteration {k}"
        xr, mr = xr.astype(np.float32).astype(np.float64), mr.astype(np.float32).astype(np.float64)
        for got, ref in ((xb, xr), (mb, mr)):
            err = np.abs(got.cpu().numpy().astype(np.float64) - ref)
            assert (err <= 1e-5 * (1 + np.abs(ref))).all(), f"iteration {k}"
        # keep the two sides on the same fp32 state (what the oracle sees is what the GPU stored)
        xr, mr = xb.cpu().numpy().astype(np.float64), mb.cpu().numpy().astype(np.float64)


def test_prepared_calls_equal_direct_calls(oracle):
    """prepare_step / prepare_local_grad_lsq marshal once and issue the same C calls: same bits, iteration after
    iteration of a time-varying topology (the prepared step must pick phase k mod period like the direct one)."""
    import paper_2104_11981_amd as P

    n, b, d = 8, 32, 1024
    rng = np.random.default_rng(5)
    A = torch.from_numpy(rng.standard_normal((n, b, d)).astype(np.float32)).cuda()
    y = torch.from_numpy(rng.standard_normal((n, b)).astype(np.float32)).cuda()
    topo = P.topology_build(P.DL_TOPO_EXP_ONEPEER, n)
    packed = P.topology_pack(topo)
    gamma, beta, scale = float(np.float32(0.01)), float(np.float32(0.9)), float(np.float32(1.0 / b))
    state = []
    for prepared in (False, True, "packed"):
        x = torch.zeros((n, d), dtype=torch.float32, device="cuda")
        m, g = torch.zeros_like(x), torch.zeros_like(x)
        loss = torch.zeros(n, dtype=torch.float32, device="cuda")
        ws = torch.empty(P.local_grad_lsq_workspace(n, b, d), dtype=torch.uint8, device="cuda")
        if prepared:
            grad = P.prepare_local_grad_lsq(A, y, x, g, loss, scale, ws)
            step = P.prepare_step("dmsgd", x, m, g, packed if prepared == "packed" else topo, gamma, beta)
        for k in range(7):
            if prepared:
                grad()
                step(k)
            else:
                P.local_grad_lsq(A, y, x, g, loss, scale, ws)
                P.dmsgd_step(x, m, g, topo, gamma, beta, k)
        torch.cuda.synchronize()
        state.append((x.clone(), m.clone(), g.clone(), loss.clone()))
    for other in state[1:]:
        for a, c in zip(state[0], other):
            assert torch.equal(a, c)
    with pytest.raises(P.DecentLamError):
        step(-1)
