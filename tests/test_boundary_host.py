"""Host-side tests of the C ABI (no GPU): the library loads and exports what
include/decentlam.h declares, topology_build matches the oracle bit for bit,
and argument validation returns the documented status codes before any device
work is attempted."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2104_11981_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
I32P = ctypes.POINTER(ctypes.c_int32)
F32P = ctypes.POINTER(ctypes.c_float)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "decentlam.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b([a-z_][a-z0-9_]*)\s*\(", header)) - {"defined", "sizeof"}
    assert declared == set(P.EXPORTS)
    lib = ctypes.CDLL(P.LIB_PATH)
    for name in declared:
        assert getattr(lib, name) is not None


@pytest.mark.parametrize("kind", [0, 1, 2, 3, 4, 5])
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6, 7, 8, 9, 15, 16, 17, 31, 32, 33, 64, 100, 128, 256])
def test_topology_build_matches_oracle_bit_exactly(oracle, kind, n):
    ours = P.topology_build(kind, n, seed=2104 + n, phases=5)
    ref = oracle.topology(kind, n, seed=2104 + n, phases=5)
    assert ours.period == ref.period
    np.testing.assert_array_equal(ours.row_ptr, ref.row_ptr)
    np.testing.assert_array_equal(ours.col_idx, ref.col_idx)
    np.testing.assert_array_equal(ours.w.view(np.uint32), ref.w.view(np.uint32))  # fp32 bit patterns


@pytest.mark.parametrize("kind,n", [(0, 1), (0, 2), (0, 5), (1, 8), (1, 12), (2, 8), (2, 6), (3, 8), (3, 12),
                                    (4, 6), (4, 12), (4, 7), (5, 8), (5, 9)])
def test_topology_flags_describe_the_matrix(oracle, kind, n):
    ours = P.topology_build(kind, n, seed=3, phases=4)
    ref = oracle.topology(kind, n, seed=3, phases=4)
    sym = all(np.array_equal(ref.dense(p), ref.dense(p).T) for p in range(ref.period))
    assert bool(ours.flags & P.DL_FLAG_SYMMETRIC) == sym
    for p in range(ref.period):
        W = ref.dense(p)
        assert bool(ours.flags & P.DL_FLAG_ROW_STOCHASTIC) and np.abs(W.sum(1) - 1).max() <= 1e-6
        assert bool(ours.flags & P.DL_FLAG_COL_STOCHASTIC) and np.abs(W.sum(0) - 1).max() <= 1e-6


def test_topology_build_size_query_and_capacity():
    period, nnz, flags = ctypes.c_int32(), ctypes.c_int64(), ctypes.c_uint32()
    rc = P.raw.topology_build(P.DL_TOPO_EXP_STATIC, 32, None, 0, None, None, 0, ctypes.byref(period),
                              ctypes.byref(nnz), ctypes.byref(flags))
    assert rc == P.DL_OK and period.value == 1 and nnz.value == 192
    row_ptr = np.zeros(33, np.int32)
    col = np.zeros(100, np.int32)
    w = np.zeros(100, np.float32)
    rc = P.raw.topology_build(P.DL_TOPO_EXP_STATIC, 32, row_ptr.ctypes.data_as(I32P), 33,
                              col.ctypes.data_as(I32P), w.ctypes.data_as(F32P), 100,
                              ctypes.byref(period), ctypes.byref(nnz), ctypes.byref(flags))
    assert rc == P.DL_ECAP and nnz.value == 192 and "nnz_cap" in P.last_error()
    assert not col.any()   # nothing written when the capacity is short
    assert P.raw.topology_build(9, 4, None, 0, None, None, 0, ctypes.byref(period), ctypes.byref(nnz),
                                None) == P.DL_EINVAL
    assert P.raw.topology_build(0, 0, None, 0, None, None, 0, ctypes.byref(period), ctypes.byref(nnz),
                                None) == P.DL_EINVAL
    assert P.raw.topology_build(0, 4, None, 0, None, None, 0, None, None, None) == P.DL_EINVAL


def _call(fn, n=4, d=0, ld=0, topo=None, gamma=0.1, beta=0.9, k=0, x=None, m=None, g=None):
    topo = topo or P.topology_build(0, n)
    return fn(x, m, g, n, d, ld, *topo._args(), gamma, beta, k, None)


@pytest.mark.parametrize("fn", [P.raw.decentlam_step, P.raw.dmsgd_step])
def test_step_argument_validation(fn):
    assert _call(fn) == P.DL_OK                      # d == 0: successful no-op, no device needed
    assert _call(fn, n=0, topo=P.topology_build(0, 1)) == P.DL_EINVAL
    assert _call(fn, d=-1) == P.DL_EINVAL
    assert _call(fn, d=8, ld=4) == P.DL_EINVAL
    for bad in (0.0, -0.1, float("inf"), float("nan")):
        assert _call(fn, gamma=bad) == P.DL_EINVAL
    for bad in (-0.1, 1.0, float("nan")):
        assert _call(fn, beta=bad) == P.DL_EINVAL
    assert _call(fn, beta=0.0) == P.DL_OK            # beta = 0 is the DSGD case
    assert _call(fn, k=-1) == P.DL_EINVAL
    assert _call(fn, d=8, ld=8) == P.DL_EINVAL       # NULL arrays with d > 0
    assert "NULL" in P.last_error()
    assert _call(fn, d=8, ld=8, x=4096, m=4096 + 64, g=8192) == P.DL_EALIAS   # m starts inside x
    assert _call(fn, d=8, ld=8, x=4096, m=8192, g=4096) == P.DL_EALIAS        # g is x
    assert _call(fn, d=8, ld=8, x=1026, m=4096, g=8192) == P.DL_EINVAL        # misaligned pointer


def _topo(n, rows):
    row_ptr, col, w = [0], [], []
    for r in rows:
        for j, wij in r:
            col.append(j)
            w.append(wij)
        row_ptr.append(len(col))
    return P.make_topology(n, row_ptr, col, w)


def test_step_topology_validation():
    fn = P.raw.decentlam_step
    good = [[(0, 0.5), (1, 0.5)], [(1, 0.5), (0, 0.5)]]
    assert _call(fn, n=2, topo=_topo(2, good)) == P.DL_OK
    cases = {
        "outside": [[(0, 0.5), (2, 0.5)], [(1, 1.0)]],
        "twice": [[(0, 0.5), (0, 0.5)], [(1, 1.0)]],
        "must be finite": [[(0, 1.5), (1, -0.5)], [(1, 1.0)]],
        "sums to": [[(0, 0.5), (1, 0.4)], [(1, 1.0)]],
        "empty": [[(0, 1.0)], []],
    }
    for needle, rows in cases.items():
        assert _call(fn, n=2, topo=_topo(2, rows)) == P.DL_ETOPO
        assert needle in P.last_error(), (needle, P.last_error())
    nan_w = _topo(2, [[(0, float("nan"))], [(1, 1.0)]])
    assert _call(fn, n=2, topo=nan_w) == P.DL_ETOPO
    # limits: more nodes / entries than travel in the kernel arguments
    big = P.topology_build(0, 300)
    assert _call(fn, n=300, topo=big) == P.DL_ETOPO and "DL_MAX_NODES" in P.last_error()
    dense = _topo(32, [[(j, 1.0 / 32) for j in range(32)] for _ in range(32)])
    assert _call(fn, n=32, topo=dense) == P.DL_OK          # 1024 entries, one weight value: palette encoding
    dense64 = _topo(64, [[(j, 1.0 / 64) for j in range(64)] for _ in range(64)])
    assert _call(fn, n=64, topo=dense64) == P.DL_ETOPO and "DL_MAX_NNZ_ROW_WEIGHTS" in P.last_error()
    dense50 = _topo(50, [[(j, 1.0 / 50) for j in range(50)] for _ in range(50)])
    assert _call(fn, n=50, topo=dense50) == P.DL_OK        # 2500 entries, one weight per row: column indices only
    mixed = [[(j, 1.0 / 50) for j in range(50)] for _ in range(50)]
    mixed[7] = [(j, (1.5 if j == 0 else 0.5 if j == 1 else 1.0) / 50) for j in range(50)]
    assert _call(fn, n=50, topo=_topo(50, mixed)) == P.DL_ETOPO and "mixed weights" in P.last_error()
    exp256 = P.topology_build(P.DL_TOPO_EXP_STATIC, 256)    # 9 x 256 = 2304 entries, all 1/9
    assert _call(fn, n=256, topo=exp256) == P.DL_OK
    # a graph that fits the kernel arguments but not the LDS beside a tile of 16-byte lanes: accepted (it runs
    # with narrower lanes; tests/test_gpu_limits.py launches it)
    wide = _topo(64, [[((i + t) % 64, 1.0 / 40) for t in range(40)] for i in range(64)])   # 2560 entries
    assert _call(fn, n=64, topo=wide) == P.DL_OK            # d == 0: nothing to launch
    rng = np.random.default_rng(0)
    rows = []
    for i in range(30):                                     # 900 entries, all weights different
        wts = rng.uniform(0.5, 1.5, size=30).astype(np.float32).astype(np.float64)
        wts[0] += 1e-3 * i
        wts = (wts / wts.sum()).astype(np.float32)
        rows.append([(j, float(wts[j])) for j in range(30)])
    assert _call(fn, n=30, topo=_topo(30, rows)) == P.DL_ETOPO and "distinct" in P.last_error()
    assert _call(fn, n=16, topo=_topo(16, [r[:16] for r in rows[:16]])) in (P.DL_OK, P.DL_ETOPO)  # row sums decide
    # time-varying W: the phase used is k mod period, and only that phase is inspected
    t = P.topology_build(2, 8)
    t.w[2 * 16 + 3] = -1.0                            # corrupt phase 2 only
    assert _call(fn, n=8, topo=t, k=0) == P.DL_OK
    assert _call(fn, n=8, topo=t, k=1) == P.DL_OK
    assert _call(fn, n=8, topo=t, k=2) == P.DL_ETOPO
    assert _call(fn, n=8, topo=t, k=5) == P.DL_ETOPO
    assert _call(fn, n=8, topo=t, k=6) == P.DL_OK


def test_lsq_argument_validation():
    f = P.raw.local_grad_lsq
    ws = P.local_grad_lsq_workspace(2, 3, 8)
    assert ws > 0 and P.local_grad_lsq_workspace(0, 3, 8) == 0
    ok = dict(A=0x10000, y=0x20000, x=0x30000, g=0x40000, loss=0, n=2, b=3, d=8, ldA=8, ld=8,
              scale=1.0, wsp=0x50000, wsb=ws)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["A"], a["y"], a["x"], a["g"], a["loss"], a["n"], a["b"], a["d"], a["ldA"], a["ld"],
                 a["scale"], a["wsp"], a["wsb"], None)

    assert call(n=0) == P.DL_EINVAL
    assert call(b=0) == P.DL_EINVAL
    assert call(d=-1) == P.DL_EINVAL
    assert call(ldA=4) == P.DL_EINVAL
    assert call(ld=4) == P.DL_EINVAL
    assert call(scale=float("nan")) == P.DL_EINVAL
    assert call(A=0) == P.DL_EINVAL
    assert call(wsb=ws - 1) == P.DL_ECAP and str(ws) in P.last_error()
    assert call(wsp=0) == P.DL_ECAP
    assert call(wsp=0x50008) == P.DL_EINVAL          # workspace not 16-byte aligned
    assert call(g=0x10010) == P.DL_EALIAS            # g inside A
    assert call(g=0x30000) == P.DL_EALIAS            # g == x
    assert call(loss=0x40000) == P.DL_EALIAS         # loss inside g


def test_lsq_workspace_covers_every_smaller_batch():
    """local_grad_lsq_rows runs the kernels on bs <= b rows with a workspace sized for b: the size must not shrink
    when b grows, whichever kernels the shape selects (the row-block count of the single sweep depends on b and d),
    and must hold at least the partial gradients of one row block per node."""
    for d in (4, 1024, 4096, 8192, 8196, 16384, 20480, 32768, 32772, 40000, 65536, 100000, 131072, 131076, 262144, 262148):
        for n in (1, 8, 64):
            sizes = [P.local_grad_lsq_workspace(n, b, d) for b in (1, 2, 7, 8, 9, 16, 100, 1024, 4096)]
            assert all(a <= b for a, b in zip(sizes, sizes[1:])), (n, d, sizes)
            assert sizes[0] >= n * d * 8


def test_lsq_poll_limit_setting():
    old = P.raw.local_grad_lsq_poll_limit(7)
    assert old == 1 << 21
    assert P.raw.local_grad_lsq_poll_limit(-1) == 7      # negative: back to the default
    assert P.raw.local_grad_lsq_poll_limit(-5) == 1 << 21
    assert P.local_grad_lsq_poll_limit(-1) == 1 << 21


def test_lsq_static_refuses_sizes_beyond_its_array():
    """local_grad_lsq_static checks the size first: nothing touches a device, so fake pointers will do."""
    fake = ctypes.c_void_p(0x10000)   # 16-byte aligned: the single-sweep kernels would be chosen
    n, b, d = 64, 4096, 16384         # 64 x 8 row blocks x 16385 doubles = 67 MB of partial sums
    rc = P.raw.local_grad_lsq_static(fake, fake, fake, fake, None, n, b, d, d, d, 1.0, None)
    assert rc == P.DL_ECAP and "DL_STATIC_SCRATCH_BYTES" in P.last_error()
    header = open(os.path.join(ROOT, "include", "decentlam.h")).read()
    assert re.search(r"#define DL_STATIC_SCRATCH_BYTES \(32u << 20\)", header) and P.DL_STATIC_SCRATCH_BYTES == 32 << 20


def test_topology_pack_and_packed_step_validation():
    topo = P.topology_build(P.DL_TOPO_EXP_ONEPEER, 8)
    need = P.topology_pack_bytes(8, topo.period)
    assert need > 0 and P.topology_pack_bytes(0, 1) == 0 and P.topology_pack_bytes(257, 1) == 0 and P.topology_pack_bytes(4, 0) == 0
    buf = np.zeros(need, np.uint8)
    ptr = ctypes.c_void_p(buf.ctypes.data)
    assert P.raw.topology_pack(8, *topo._args(), ptr, need - 1) == P.DL_ECAP and "topology_pack_bytes" in P.last_error()
    assert not buf.any()
    assert P.raw.topology_pack(8, *topo._args(), None, need) == P.DL_EINVAL
    assert P.raw.topology_pack(0, *topo._args(), ptr, need) == P.DL_EINVAL
    rp, ci, w, per = topo._args()
    assert P.raw.topology_pack(8, None, ci, w, per, ptr, need) == P.DL_EINVAL
    assert P.raw.topology_pack(8, rp, ci, w, 0, ptr, need) == P.DL_EINVAL
    bad = P.make_topology(8, topo.row_ptr, topo.col_idx, topo.w * np.float32(0.9), topo.period)   # rows no longer sum to 1
    assert P.raw.topology_pack(8, *bad._args(), ptr, need) == P.DL_ETOPO
    # a failed call leaves no valid buffer behind: the step refuses it
    assert P.raw.decentlam_step_packed(None, None, None, 8, 0, 0, ptr, 0.1, 0.9, 0, None) == P.DL_ETOPO
    assert P.raw.topology_pack(8, *topo._args(), ptr, need) == P.DL_OK
    step = lambda **kw: P.raw.decentlam_step_packed(None, None, None, kw.get("n", 8), kw.get("d", 0), 0, kw.get("packed", ptr),
                                                    kw.get("gamma", 0.1), kw.get("beta", 0.9), kw.get("k", 0), None)
    assert step() == P.DL_OK                                   # d == 0: no device needed
    assert step(n=4) == P.DL_ETOPO and "8 nodes" in P.last_error()
    assert step(packed=None) == P.DL_EINVAL and step(k=-1) == P.DL_EINVAL
    assert step(gamma=0.0) == P.DL_EINVAL and step(beta=1.0) == P.DL_EINVAL
    assert step(packed=ctypes.c_void_p(buf.ctypes.data + 1)) == P.DL_EINVAL      # misaligned
    scribbled = buf.copy()
    scribbled[0] ^= 0xFF
    assert step(packed=ctypes.c_void_p(scribbled.ctypes.data)) == P.DL_ETOPO
    assert P.raw.dmsgd_step_packed(None, None, None, 8, 0, 0, ptr, 0.1, 0.9, 3, None) == P.DL_OK
    assert P.raw.dsgd_step_packed(None, None, 8, 0, 0, ptr, 0.1, 5, None) == P.DL_OK
    # the Python wrapper
    packed = P.topology_pack(topo)
    assert packed.n == 8 and packed.period == topo.period and packed.buffer.size == need
    assert bytes(packed.buffer) == bytes(buf)                  # deterministic encoding


def test_device_topology_argument_validation():
    """What topology_pack_device and the *_step_dev calls refuse before any device work."""
    t = P.topology_build(P.DL_TOPO_EXP_SYM, 512)
    nnz = int(t.col_idx.size)
    need = P.topology_device_bytes(512, 1, nnz)
    assert need == 4 * (4 + 2 + 514 + 2 * nnz)
    assert P.topology_device_bytes(1025, 1, 10) == 0 and P.topology_device_bytes(0, 1, 1) == 0 and P.topology_device_bytes(4, 0, 1) == 0
    desc = P.DeviceTopologyStruct()
    fake = ctypes.c_void_p(0x100000)
    call = lambda topo=t, n=512, buf=fake, nbytes=need, out=ctypes.byref(desc): P.raw.topology_pack_device(
        n, *topo._args(), buf, nbytes, out)
    assert call(nbytes=need - 4) == P.DL_ECAP and "topology_device_bytes" in P.last_error()   # checked before the copy
    assert call(buf=None) == P.DL_EINVAL and call(out=None) == P.DL_EINVAL and call(n=0) == P.DL_EINVAL
    assert call(buf=ctypes.c_void_p(0x100004)) == P.DL_EINVAL
    big = P.make_topology(1025, np.arange(1026), np.arange(1025), np.ones(1025, np.float32))
    assert call(topo=big, n=1025) == P.DL_ETOPO and "1024" in P.last_error()
    bad = P.make_topology(512, t.row_ptr, t.col_idx, t.w * np.float32(1.01))
    assert call(topo=bad) == P.DL_ETOPO and "sums to" in P.last_error()
    assert desc.magic == 0
    step = lambda W=ctypes.byref(desc), n=512, d=0: P.raw.decentlam_step_dev(None, None, None, n, d, 0, W, 0.1, 0.9, 0, None)
    assert step() == P.DL_ETOPO and "topology_pack_device" in P.last_error()     # a descriptor nobody filled in
    assert step(W=None) == P.DL_EINVAL
    filled = P.DeviceTopologyStruct(0x444C4454, 512, 1, 0, 0x100000, need)
    assert step(W=ctypes.byref(filled)) == P.DL_OK                              # d == 0: nothing to launch
    assert step(W=ctypes.byref(filled), n=256) == P.DL_ETOPO and "512 nodes" in P.last_error()
    assert P.raw.dmsgd_step_dev(None, None, None, 512, 0, 0, ctypes.byref(filled), 0.1, 1.5, 0, None) == P.DL_EINVAL
    assert P.raw.dsgd_step_dev(None, None, 512, 0, 0, ctypes.byref(filled), 0.1, -1, None) == P.DL_EINVAL


def test_calibration_stream_argument_validation():
    fake = ctypes.c_void_p(0x10000)
    cols = ctypes.c_int64(-1)
    call = lambda kind=0, split=0, x=fake, n=4, d=1024, ld=1024, out=ctypes.byref(cols): P.raw.dl_calibration_stream(
        kind, split, x, fake, fake, n, d, ld, out, None)
    assert call(kind=3) == P.DL_EINVAL and call(split=2) == P.DL_EINVAL
    assert call(n=0) == P.DL_EINVAL and call(n=33) == P.DL_EINVAL
    assert call(d=-1) == P.DL_EINVAL and call(d=2048) == P.DL_EINVAL        # ld < d
    assert call(x=None) == P.DL_EINVAL and call(out=None) == P.DL_EINVAL
    assert call(x=ctypes.c_void_p(0x10004)) == P.DL_EINVAL and call(ld=1026, d=1024) == P.DL_EINVAL
    assert call(d=200, ld=200) == P.DL_OK and cols.value == 0                 # less than a tile: nothing to launch
    assert call(split=1, d=16000, ld=16000) == P.DL_OK and cols.value == 0


def test_stats_argument_validation():
    f = P.raw.decentlam_stats
    ws = P.decentlam_stats_workspace(4, 100)
    assert ws > 0 and P.decentlam_stats_workspace(0, 100) == 0
    ok = dict(x=0x10000, m=0, ref=0, n=4, d=100, ld=100, out=0x20000, wsp=0x30000, wsb=ws)

    def call(**kw):
        a = dict(ok, **kw)
        return f(a["x"], a["m"], a["ref"], a["n"], a["d"], a["ld"], a["out"], a["wsp"], a["wsb"], None)

    assert call(n=0) == P.DL_EINVAL
    assert call(d=-1) == P.DL_EINVAL
    assert call(ld=99) == P.DL_EINVAL
    assert call(out=0) == P.DL_EINVAL
    assert call(x=0) == P.DL_EINVAL
    assert call(x=0x10002) == P.DL_EINVAL
    assert call(out=0x20004) == P.DL_EINVAL
    assert call(wsb=ws - 1) == P.DL_ECAP
    assert call(wsp=0) == P.DL_ECAP


def test_dsgd_argument_validation():
    t = P.topology_build(0, 4)
    f = lambda **kw: P.raw.dsgd_step(kw.get("x"), kw.get("g"), kw.get("n", 4), kw.get("d", 0), kw.get("ld", 0),
                                     *t._args(), kw.get("gamma", 0.1), kw.get("k", 0), None)
    assert f() == P.DL_OK
    assert f(gamma=0.0) == P.DL_EINVAL
    assert f(k=-1) == P.DL_EINVAL
    assert f(d=8, ld=8) == P.DL_EINVAL
    assert f(d=8, ld=8, x=4096, g=4096 + 32) == P.DL_EALIAS


def test_topology_build_ex_and_metropolis_errors(oracle):
    period, nnz = ctypes.c_int32(), ctypes.c_int64()
    assert P.raw.topology_build(P.DL_TOPO_BIPARTITE_MATCH, 8, None, 0, None, None, 0, ctypes.byref(period),
                                ctypes.byref(nnz), None) == P.DL_EINVAL       # needs seed and phases
    assert P.raw.topology_build_ex(P.DL_TOPO_BIPARTITE_MATCH, 8, 1, 0, None, 0, None, None, 0,
                                   ctypes.byref(period), ctypes.byref(nnz), None) == P.DL_EINVAL
    assert P.raw.topology_build_ex(6, 8, 1, 1, None, 0, None, None, 0, ctypes.byref(period),
                                   ctypes.byref(nnz), None) == P.DL_EINVAL
    # Metropolis weights for a caller's graph: a path 0 - 1 - 2 (degrees 1, 2, 1)
    t = P.topology_metropolis(3, [0, 2, 5, 7], [0, 1, 0, 1, 2, 2, 1])
    np.testing.assert_allclose(t.w, [2 / 3, 1 / 3, 1 / 3, 1 / 3, 1 / 3, 2 / 3, 1 / 3], atol=6e-8)
    assert t.flags == P.DL_FLAG_ROW_STOCHASTIC | P.DL_FLAG_COL_STOCHASTIC | P.DL_FLAG_SYMMETRIC
    # on the mesh it reproduces topology_build, whatever the order inside the rows
    mesh = P.topology_build(P.DL_TOPO_MESH, 12)
    again = P.topology_metropolis(12, mesh.row_ptr, mesh.col_idx)
    np.testing.assert_array_equal(again.w.view(np.uint32), mesh.w.view(np.uint32))
    for bad_rows, needle in (([0, 1, 3, 4], [0, 1, 2, 2]), "reverse"), (([0, 2, 4, 5], [1, 2, 1, 0, 2]), "itself"), \
            (([0, 2, 2, 3], [0, 1, 2]), "empty"), (([0, 3, 5, 6], [0, 1, 1, 1, 0, 2]), "twice"), \
            (([0, 2, 4, 5], [0, 5, 1, 0, 2]), "outside"):
        with pytest.raises(P.DecentLamError) as e:
            P.topology_metropolis(3, *bad_rows)
        assert e.value.status == P.DL_ETOPO and needle in str(e.value), (needle, str(e.value))


def test_lsq_rows_argument_validation():
    f = P.raw.local_grad_lsq_rows
    ws = P.local_grad_lsq_workspace(2, 4, 8)
    base = dict(A=0x10000, y=0x20000, x=0x30000, g=0x40000, loss=0, n=2, b=10, d=8, ldA=8, ld=8,
                rows=0x60000, bs=4, scale=1.0, wsp=0x50000, wsb=ws)

    def call(**kw):
        a = dict(base, **kw)
        return f(a["A"], a["y"], a["x"], a["g"], a["loss"], a["n"], a["b"], a["d"], a["ldA"], a["ld"],
                 a["rows"], a["bs"], a["scale"], a["wsp"], a["wsb"], None)

    assert call(rows=0) == P.DL_EINVAL and "rows" in P.last_error()
    assert call(bs=0) == P.DL_EINVAL
    assert call(wsb=ws - 1) == P.DL_ECAP
    assert call(rows=0x40000) == P.DL_EALIAS
    assert call(rows=0x60002) == P.DL_EINVAL


def test_decentlam_xprev_argument_validation():
    t = P.topology_build(0, 4)
    f = lambda **kw: P.raw.decentlam_step_xprev(kw.get("x"), kw.get("xp"), kw.get("g"), 4, kw.get("d", 0),
                                                kw.get("ld", 0), *t._args(), kw.get("gamma", 0.1),
                                                kw.get("gp", 0.1), kw.get("beta", 0.9), 0, None)
    assert f() == P.DL_OK
    assert f(gp=0.0) == P.DL_EINVAL and "gamma_prev" in P.last_error()
    assert f(gp=float("nan")) == P.DL_EINVAL
    assert f(beta=1.0) == P.DL_EINVAL
    assert f(d=8, ld=8, x=4096, xp=4096, g=8192) == P.DL_EALIAS
    assert f(d=8, ld=8, x=4096, xp=0, g=8192) == P.DL_EINVAL


def test_g16_argument_validation():
    t = P.topology_build(0, 4)
    f = lambda **kw: P.raw.decentlam_step_g16(kw.get("x"), kw.get("m"), kw.get("g"), kw.get("fmt", P.DL_GRAD_BF16),
                                              4, kw.get("d", 0), kw.get("ld", 0), kw.get("ldg", 0), *t._args(),
                                              kw.get("gamma", 0.1), 0.9, 0, None)
    assert f() == P.DL_OK
    assert f(fmt=3) == P.DL_EINVAL and "g_format" in P.last_error()
    assert f(d=8, ld=8, ldg=7) == P.DL_EINVAL and "ldg" in P.last_error()
    assert f(d=8, ld=8, ldg=8, x=0x1000, m=0x2000, g=0) == P.DL_EINVAL
    assert f(d=8, ld=8, ldg=8, x=0x1000, m=0x2000, g=0x3001) == P.DL_EINVAL        # g not 2-byte aligned
    assert f(d=8, ld=8, ldg=8, x=0x1000, m=0x2000, g=0x1000 + 64) == P.DL_EALIAS   # g inside x
    assert f(d=8, ld=8, ldg=8, x=0x1000, m=0x1000 + 16, g=0x3000) == P.DL_EALIAS
    assert P.raw.dmsgd_step_g16(None, None, None, P.DL_GRAD_F16, 4, 0, 0, 0, *t._args(), 0.1, 0.9, 0, None) == P.DL_OK


def test_multi_tensor_argument_validation():
    t = P.topology_build(0, 4)
    I64 = ctypes.c_int64

    def call(offsets, **kw):
        arr = (I64 * len(offsets))(*offsets) if offsets is not None else None
        return P.raw.decentlam_step_multi(kw.get("x", 0x10000), kw.get("m", 0x20000), kw.get("g", 0x30000),
                                          kw.get("fmt", P.DL_GRAD_F32), 4, kw.get("ld", 64), kw.get("ldg", 64),
                                          kw.get("T", len(offsets) - 1 if offsets else 1), arr,
                                          kw.get("norms", 0), kw.get("ws", 0), kw.get("wsb", 0), *t._args(),
                                          0.1, 0.9, 0, None)

    assert call([0, 0, 0]) == P.DL_OK                                   # nothing to do, nothing touched
    assert call(None) == P.DL_EINVAL and "offsets" in P.last_error()
    assert call([0, 10], T=0) == P.DL_EINVAL
    assert call([-1, 10]) == P.DL_EINVAL
    assert call([0, 20, 10]) == P.DL_EINVAL and "decrease" in P.last_error()
    assert call([0, 10, 65]) == P.DL_EINVAL                             # beyond ld
    assert call([0, 10, 64], ldg=63) == P.DL_EINVAL
    need = P.decentlam_step_multi_workspace(4, 64, 2)
    assert need >= (64 // 64 + 3) * 4 * 3 * 8
    assert call([0, 10, 64], norms=0x40000, ws=0, wsb=need) == P.DL_ECAP
    assert call([0, 10, 64], norms=0x40000, ws=0x50000, wsb=need - 1) == P.DL_ECAP
    assert call([0, 10, 64], norms=0x40000, ws=0x50004, wsb=need) == P.DL_EINVAL          # workspace alignment
    assert call([0, 10, 64], norms=0x40004, ws=0x50000, wsb=need) == P.DL_EINVAL          # norms alignment
    assert call([0, 10, 64], norms=0x50000 + 8, ws=0x50000, wsb=need) == P.DL_EALIAS      # norms inside the workspace
    assert call([0, 10, 64], norms=0x10000, ws=0x50000, wsb=need) == P.DL_EALIAS          # norms inside x
    assert P.decentlam_step_multi_workspace(0, 64, 2) == 0


@pytest.mark.parametrize("name", ["awc_dmsgd_step", "da_dmsgd_step"])
def test_sibling_step_argument_validation(name):
    t = P.topology_build(0, 4)
    fn = getattr(P.raw, name)
    f = lambda **kw: fn(kw.get("x"), kw.get("m"), kw.get("g"), 4, kw.get("d", 0), kw.get("ld", 0), *t._args(),
                        kw.get("gamma", 0.1), kw.get("beta", 0.9), kw.get("k", 0), None)
    assert f() == P.DL_OK
    assert f(gamma=-1.0) == P.DL_EINVAL
    assert f(beta=1.0) == P.DL_EINVAL
    assert f(k=-1) == P.DL_EINVAL
    assert f(d=8, ld=4) == P.DL_EINVAL
    assert f(d=8, ld=8) == P.DL_EINVAL and "NULL" in P.last_error()
    assert f(d=8, ld=8, x=4096, m=4096 + 16, g=8192) == P.DL_EALIAS


def test_blocked_argument_validation():
    t = P.topology_build(0, 4)
    f = lambda **kw: P.raw.decentlam_step_blocked(kw.get("x"), kw.get("m"), kw.get("g"), 4, kw.get("d", 0),
                                                  kw.get("bw", 64), *t._args(), kw.get("gamma", 0.1), 0.9,
                                                  kw.get("k", 0), None)
    assert f() == P.DL_OK
    assert f(bw=0) == P.DL_EINVAL and "bw" in P.last_error()
    assert f(d=-1) == P.DL_EINVAL
    assert f(gamma=float("inf")) == P.DL_EINVAL
    assert f(d=100) == P.DL_EINVAL and "NULL" in P.last_error()
    assert f(d=100, x=0x10000, m=0x10000 + 4 * 200, g=0x80000) == P.DL_EALIAS     # m inside x's second block
    assert f(d=100, x=0x10002, m=0x40000, g=0x80000) == P.DL_EINVAL


def test_general_step_argument_validation():
    t = P.topology_build(0, 4)

    def call(fn=P.raw.decentlam_step_ex, lay=None, **kw):
        layout = P.Layout(*(lay or (P.DL_GRAD_F32, 8, 8, 0)))
        return fn(kw.get("x"), kw.get("m"), kw.get("g"), 4, kw.get("d", 0), ctypes.byref(layout), *t._args(),
                  kw.get("gamma", 0.1), 0.9, 0, None)

    assert call() == P.DL_OK
    assert P.raw.decentlam_step_ex(None, None, None, 4, 0, None, *t._args(), 0.1, 0.9, 0, None) == P.DL_EINVAL
    assert "layout" in P.last_error()
    assert call(lay=(P.DL_GRAD_F32, 8, 8, -1)) == P.DL_EINVAL
    assert call(lay=(7, 8, 8, 0)) == P.DL_EINVAL and "g_format" in P.last_error()
    assert call(lay=(7, 8, 8, 64)) == P.DL_EINVAL and "g_format" in P.last_error()
    assert call(d=9) == P.DL_EINVAL                                     # ld < d
    assert call(d=8, lay=(P.DL_GRAD_BF16, 8, 4, 0)) == P.DL_EINVAL      # ldg < d
    assert call(d=8, x=0x1000, m=0x2000, g=0x3001, lay=(P.DL_GRAD_BF16, 8, 8, 0)) == P.DL_EINVAL
    assert call(d=8, x=0x1000, m=0x2000, g=0x1010, lay=(P.DL_GRAD_F16, 8, 8, 64)) == P.DL_EALIAS
    layout = P.Layout(P.DL_GRAD_F32, 8, 8, 0)
    f = lambda gp: P.raw.decentlam_step_xprev_ex(None, None, None, 4, 0, ctypes.byref(layout), *t._args(), 0.1, gp,
                                                 0.9, 0, None)
    assert f(0.1) == P.DL_OK and f(0.0) == P.DL_EINVAL
    layout.bw = 64
    assert f(0.1) == P.DL_OK and f(-1.0) == P.DL_EINVAL and "gamma_prev" in P.last_error()


def test_recommended_row_layout_helpers():
    """recommended_ld / empty_rows: rows on 64 KiB boundaries for large arrays, 256 bytes for small ones."""
    import torch
    import paper_2104_11981_amd as P

    assert P.recommended_ld(25_600_000) == 25_608_192 and P.recommended_ld(25_608_192) == 25_608_192
    assert P.recommended_ld(1 << 20) == (1 << 20) + 16384 and P.recommended_ld((1 << 20) + 1) == (1 << 20) + 16384
    assert P.recommended_ld(1 << 21) == 1 << 21
    assert P.recommended_ld(1000) == 1024 and P.recommended_ld(64) == 64 and P.recommended_ld(1) == 64
    assert P.recommended_ld(65535) == 65536 and P.recommended_ld(65537) == 5 * 16384
    # strides of 127 or 129 times 64 KiB (and their multiples) put the rows of a column on the same channels
    assert P.recommended_ld(127 * 16384) == 128 * 16384 and P.recommended_ld(129 * 16384 - 5) == 130 * 16384
    assert P.recommended_ld(2 * 129 * 16384) == (2 * 129 + 1) * 16384
    v = P.empty_rows(3, (1 << 20) + 5, device="cpu", fill=2.0)
    assert tuple(v.shape) == (3, (1 << 20) + 5) and v.stride() == ((1 << 20) + 16384, 1)
    assert v.data_ptr() % 65536 == 0 and float(v.sum()) == 2.0 * 3 * ((1 << 20) + 5)
    h = P.empty_rows(2, 100, device="cpu", dtype=torch.bfloat16)
    assert h.stride() == (128, 1) and h.data_ptr() % 65536 == 0
