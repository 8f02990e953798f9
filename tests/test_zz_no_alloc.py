"""local_grad_lsq_static (the entry point that allocates nothing) against local_grad_lsq, through the C ABI.

The two share their kernels, so the outputs must agree bit for bit, and both must meet the parity bar
against the oracle.  Two calls in a row, the second on a smaller problem: the library's scratch array
keeps the first call's contents and the second call must not be disturbed by them."""
import ctypes

import numpy as np
import pytest

torch = pytest.importorskip("torch")
import paper_2104_11981_amd as P  # noqa: E402

pytestmark = pytest.mark.gpu

VP = ctypes.c_void_p


def _problem(rng, n, b, d):
    A = rng.standard_normal((n, b, d)).astype(np.float32)
    y = rng.standard_normal((n, b)).astype(np.float32)
    x = rng.standard_normal((n, d)).astype(np.float32)
    return A, y, x


def _run_both(A0, y0, x0, scale):
    n, b, d = A0.shape
    A, y, x = (torch.from_numpy(a).cuda() for a in (A0, y0, x0))
    out = {}
    for name in ("workspace", "static"):
        g = torch.full((n, d), float("nan"), dtype=torch.float32, device="cuda")
        loss = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
        if name == "workspace":
            ws = torch.empty(P.local_grad_lsq_workspace(n, b, d), dtype=torch.uint8, device="cuda")
            rc = P.raw.local_grad_lsq(VP(A.data_ptr()), VP(y.data_ptr()), VP(x.data_ptr()), VP(g.data_ptr()),
                                      VP(loss.data_ptr()), n, b, d, d, d, scale, VP(ws.data_ptr()), ws.numel(), None)
        else:
            rc = P.raw.local_grad_lsq_static(VP(A.data_ptr()), VP(y.data_ptr()), VP(x.data_ptr()), VP(g.data_ptr()),
                                             VP(loss.data_ptr()), n, b, d, d, d, scale, None)
        assert rc == P.DL_OK, P.last_error()
        torch.cuda.synchronize()
        out[name] = (g.cpu().numpy(), loss.cpu().numpy())
    return out


# first call, then a smaller one: a single-sweep shape and then the small-problem kernel; the single sweep
# with 4-byte accesses (rows not 16-byte aligned) and then a narrower one with 16-byte accesses; a two-sweep
# shape (such rows, more than 16384 columns) and then a single sweep; rows beyond 32768 columns twice (the waves of
# the second call must not take the first call's shares of the dot products, still in the array, for their own)
@pytest.mark.parametrize("shapes", [((8, 96, 1024), (3, 20, 100)), ((5, 33, 1001), (4, 16, 512)),
                                    ((2, 20, 16387), (2, 12, 2048)), ((64, 256, 4096), (8, 32, 1024)),
                                    ((2, 40, 40000), (1, 20, 36000))])
def test_static_scratch_call_matches_workspace_call_twice_in_a_row(oracle, shapes):
    rng = np.random.default_rng(11981)
    for n, b, d in shapes:
        print(f"local_grad_lsq_static n={n} b={b} d={d}", flush=True)
        A0, y0, x0 = _problem(rng, n, b, d)
        scale = float(np.float32(1.0 / b))
        got = _run_both(A0, y0, x0, scale)
        g_ref, loss_ref = oracle.lsq_grad(A0, y0, x0, scale)
        for name, (g, loss) in got.items():
            assert (np.abs(g - g_ref) <= 1e-5 * (1 + np.abs(g_ref))).all(), name
            assert (np.abs(loss - loss_ref) <= 1e-5 * (1 + np.abs(loss_ref))).all(), name
        np.testing.assert_array_equal(got["static"][0].view(np.uint32), got["workspace"][0].view(np.uint32))
        np.testing.assert_array_equal(got["static"][1].view(np.uint32), got["workspace"][1].view(np.uint32))


def test_static_scratch_call_refuses_what_does_not_fit():
    n, b, d = 64, 4096, 16384   # 64 x 8 x 16385 doubles of partial sums: beyond the 32 MiB array
    assert P.local_grad_lsq_workspace(n, b, d) > P.DL_STATIC_SCRATCH_BYTES
    a = torch.zeros(16, dtype=torch.float32, device="cuda")   # never dereferenced: the size check comes first
    rc = P.raw.local_grad_lsq_static(VP(a.data_ptr()), VP(a.data_ptr()), VP(a.data_ptr()), VP(a.data_ptr()), None,
                                     n, b, d, d, d, 1.0, None)
    assert rc == P.DL_ECAP and "DL_STATIC_SCRATCH_BYTES" in P.last_error()
