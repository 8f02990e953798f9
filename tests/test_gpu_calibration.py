"""The bare calibration streams (dl_calibration_stream) do what their header says: kind 0 computes
x <- x + g / 2, m <- m / 2 + g on whole tiles in either column order and leaves the remaining columns and the
padding alone; kind 1 stores nothing; kind 2 overwrites x and m on the covered columns only.  (They carry no
arithmetic of the method: the reference here is the formula of the header, evaluated with numpy.)"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.mark.parametrize("split", [False, True])
@pytest.mark.parametrize("n,d,ld", [(32, 3 * 16384 + 700, 3 * 16384 + 704), (5, 16384 + 256 * 3 + 4, 2 * 16384)])
def test_calibration_stream_covers_whole_tiles_only(split, n, d, ld):
    import paper_2104_11981_amd as P

    rng = np.random.default_rng(n + d)
    SENT = 77.0
    host = [np.full((n, ld), SENT, np.float32) for _ in range(3)]
    for h in host:
        h[:, :d] = rng.standard_normal((n, d)).astype(np.float32)
    bufs = [torch.from_numpy(h.copy()).cuda() for h in host]
    x, m, g = (b[:, :d] for b in bufs)
    want_cols = d // 16384 * 16384 if split else d // 256 * 256

    assert P.dl_calibration_stream(1, split, x, m, g) == want_cols      # reads only: nothing changes
    torch.cuda.synchronize()
    for b, h in zip(bufs, host):
        np.testing.assert_array_equal(b.cpu().numpy(), h)

    assert P.dl_calibration_stream(0, split, x, m, g) == want_cols
    torch.cuda.synchronize()
    x0, m0, g0 = host
    xr, mr = x0.copy(), m0.copy()
    xr[:, :want_cols] = x0[:, :want_cols] + np.float32(0.5) * g0[:, :want_cols]
    mr[:, :want_cols] = np.float32(0.5) * m0[:, :want_cols] + g0[:, :want_cols]
    np.testing.assert_allclose(bufs[0].cpu().numpy(), xr, rtol=1e-6, atol=1e-6)
    np.testing.assert_allclose(bufs[1].cpu().numpy(), mr, rtol=1e-6, atol=1e-6)
    np.testing.assert_array_equal(bufs[2].cpu().numpy(), g0)             # g is read-only, padding untouched
    assert (bufs[0].cpu().numpy()[:, d:] == SENT).all() and (bufs[1].cpu().numpy()[:, d:] == SENT).all()

    assert P.dl_calibration_stream(2, split, x, m, g) == want_cols      # writes only
    torch.cuda.synchronize()
    xa, ma = bufs[0].cpu().numpy(), bufs[1].cpu().numpy()
    np.testing.assert_array_equal(xa[:, want_cols:], xr[:, want_cols:])   # beyond the covered columns: as before
    np.testing.assert_array_equal(ma[:, want_cols:], mr[:, want_cols:])
    assert np.isfinite(xa).all() and np.isfinite(ma).all()
