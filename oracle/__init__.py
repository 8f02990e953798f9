"""CPU oracle -- TEST INFRASTRUCTURE, not part of the product.

ctypes front end of `decentlam_oracle.c` (plain fp64 loops that follow the
paper's Algorithm 1, Algorithm 2 and least-squares gradient statement by
statement) plus a trajectory driver.  Only tests, the smoke check and the
benchmark's cpu_baseline leg may import this package; it imports nothing from
the GPU package and the GPU package imports nothing from here.

All step functions take and return float64 arrays.  "fp32 storage" (what the
GPU library keeps in HBM) is emulated by the caller rounding the returned state
to float32 between steps -- see `run`.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "decentlam_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

RING, EXP_STATIC, EXP_ONEPEER, EXP_SYM, MESH, BIPARTITE_MATCH = 0, 1, 2, 3, 4, 5


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fused multiply-add, OpenMP for the timing leg)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fopenmp",
             _SRC, "-o", tmp])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        i32p = ctypes.POINTER(ctypes.c_int32)
        i64p = ctypes.POINTER(ctypes.c_int64)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        _lib.oracle_num_threads.restype = ctypes.c_int
        _lib.oracle_topology.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_uint64, ctypes.c_int, i32p, i64p,
                                         i32p, i32p, f32p]
        _lib.oracle_dsgd_step.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int, i32p, i32p, f32p,
                                          ctypes.c_double, ctypes.c_int64, f64p, f64p, f64p]
        step = [ctypes.c_int, ctypes.c_int64, ctypes.c_int, i32p, i32p, f32p, ctypes.c_double,
                ctypes.c_double, ctypes.c_int64, f64p, f64p, f64p, f64p, f64p]
        _lib.oracle_dmsgd_step.argtypes = step
        _lib.oracle_decentlam_step.argtypes = step
        _lib.oracle_awc_dmsgd_step.argtypes = step
        _lib.oracle_da_dmsgd_step.argtypes = step
        _lib.oracle_decentlam_xprev_step.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int, i32p, i32p, f32p,
                                                     ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                                     ctypes.c_int64, f64p, f64p, f64p, f64p]
        _lib.oracle_lsq_grad_rows.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, f32p, f32p, f64p, i32p,
                                              ctypes.c_int, ctypes.c_double, f64p, f64p]
        _lib.oracle_stats.argtypes = [ctypes.c_int, ctypes.c_int64, f64p, f64p, f64p, f64p]
        _lib.oracle_lsq_grad.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, f32p, f32p, f64p,
                                         ctypes.c_double, f64p, f64p]
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


@dataclass
class Topology:
    """Neighbour lists of a (possibly time-varying) weight matrix, CSR, phase-major."""
    n: int
    period: int
    row_ptr: np.ndarray   # int32 [period*(n+1)], absolute offsets
    col_idx: np.ndarray   # int32 [nnz]
    w: np.ndarray         # float32 [nnz]

    def dense(self, phase: int = 0) -> np.ndarray:
        """W of one phase as a dense float64 matrix (for tests)."""
        W = np.zeros((self.n, self.n))
        rp = self.row_ptr[phase * (self.n + 1):(phase + 1) * (self.n + 1)]
        for i in range(self.n):
            for e in range(rp[i], rp[i + 1]):
                W[i, self.col_idx[e]] += float(self.w[e])
        return W


def topology(kind: int, n: int, seed: int = 0, phases: int = 1) -> Topology:
    """Neighbour lists and weights of one of the paper's topologies (seed, phases: random match only)."""
    lib = _load()
    period = ctypes.c_int32(0)
    nnz = ctypes.c_int64(0)
    rc = lib.oracle_topology(kind, n, seed, phases, ctypes.byref(period), ctypes.byref(nnz), None, None, None)
    if rc:
        raise ValueError(f"oracle_topology({kind}, {n}) -> {rc}")
    row_ptr = np.zeros(period.value * (n + 1), dtype=np.int32)
    col_idx = np.zeros(nnz.value, dtype=np.int32)
    w = np.zeros(nnz.value, dtype=np.float32)
    rc = lib.oracle_topology(kind, n, seed, phases, ctypes.byref(period), ctypes.byref(nnz),
                             _p(row_ptr, ctypes.c_int32), _p(col_idx, ctypes.c_int32),
                             _p(w, ctypes.c_float))
    assert rc == 0
    return Topology(n, period.value, row_ptr, col_idx, w)


def custom_topology(n: int, phases) -> Topology:
    """Topology from explicit neighbour lists: phases[p][i] = [(j, w_ij), ...]."""
    period = len(phases)
    row_ptr, col_idx, w = [], [], []
    for p in range(period):
        assert len(phases[p]) == n
        for i in range(n):
            row_ptr.append(len(col_idx))
            for j, wij in phases[p][i]:
                col_idx.append(j)
                w.append(wij)
        row_ptr.append(len(col_idx))
    return Topology(n, period, np.asarray(row_ptr, np.int32), np.asarray(col_idx, np.int32),
                    np.asarray(w, np.float32))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _topo_args(t: Topology):
    return (t.period, _p(t.row_ptr, ctypes.c_int32), _p(t.col_idx, ctypes.c_int32),
            _p(t.w, ctypes.c_float))


def dsgd_step(x, g, topo: Topology, gamma: float, k: int = 0):
    x, g = _f64(x), _f64(g)
    n, d = x.shape
    assert n == topo.n and g.shape == x.shape
    xo = np.empty_like(x)
    rc = _load().oracle_dsgd_step(n, d, *_topo_args(topo), float(gamma), int(k),
                                  _p(x, ctypes.c_double), _p(g, ctypes.c_double),
                                  _p(xo, ctypes.c_double))
    assert rc == 0
    return xo


def _mom_step(fn, x, m, g, topo, gamma, beta, k):
    x, m, g = _f64(x), _f64(m), _f64(g)
    n, d = x.shape
    assert n == topo.n and m.shape == x.shape and g.shape == x.shape
    xo, mo = np.empty_like(x), np.empty_like(x)
    rc = fn(n, d, *_topo_args(topo), float(gamma), float(beta), int(k),
            _p(x, ctypes.c_double), _p(m, ctypes.c_double), _p(g, ctypes.c_double),
            _p(xo, ctypes.c_double), _p(mo, ctypes.c_double))
    assert rc == 0
    return xo, mo


def dmsgd_step(x, m, g, topo: Topology, gamma: float, beta: float, k: int = 0):
    """One iteration of Algorithm 1 -> (x_next, m_next), float64."""
    return _mom_step(_load().oracle_dmsgd_step, x, m, g, topo, gamma, beta, k)


def decentlam_step(x, m, g, topo: Topology, gamma: float, beta: float, k: int = 0):
    """One iteration of Algorithm 2 -> (x_next, m_next), float64."""
    return _mom_step(_load().oracle_decentlam_step, x, m, g, topo, gamma, beta, k)


def awc_dmsgd_step(x, m, g, topo: Topology, gamma: float, beta: float, k: int = 0):
    """AWC-DmSGD as read here (m <- beta m + g; x <- W x - gamma m) -> (x_next, m_next), float64.
    Parity weakly pinned: the paper prints no recursion for it."""
    return _mom_step(_load().oracle_awc_dmsgd_step, x, m, g, topo, gamma, beta, k)


def da_dmsgd_step(x, m, g, topo: Topology, gamma: float, beta: float, k: int = 0):
    """DA-DmSGD as read here (mh = beta m + g; x <- W (x - gamma mh); m <- W mh) -> (x_next, m_next).
    Parity weakly pinned: the paper prints no recursion for it."""
    return _mom_step(_load().oracle_da_dmsgd_step, x, m, g, topo, gamma, beta, k)


def decentlam_xprev_step(x, x_prev, g, topo: Topology, gamma: float, beta: float, k: int = 0,
                         gamma_prev: float | None = None):
    """Momentum-free DecentLaM: x_next = W(x - gamma g) + beta (gamma/gamma_prev) (x - x_prev), float64."""
    x, x_prev, g = _f64(x), _f64(x_prev), _f64(g)
    n, d = x.shape
    assert n == topo.n and x_prev.shape == x.shape and g.shape == x.shape
    xo = np.empty_like(x)
    rc = _load().oracle_decentlam_xprev_step(n, d, *_topo_args(topo), float(gamma),
                                             float(gamma if gamma_prev is None else gamma_prev), float(beta),
                                             int(k), _p(x, ctypes.c_double), _p(x_prev, ctypes.c_double),
                                             _p(g, ctypes.c_double), _p(xo, ctypes.c_double))
    assert rc == 0
    return xo


def lsq_grad(A, y, x, scale: float = 1.0):
    """g_i = scale * A_i^T (A_i x_i - y_i), loss_i = (scale/2)||A_i x_i - y_i||^2 -> (g, loss)."""
    A = np.ascontiguousarray(A, dtype=np.float32)
    y = np.ascontiguousarray(y, dtype=np.float32)
    x = _f64(x)
    n, b, d = A.shape
    assert y.shape == (n, b) and x.shape == (n, d)
    g = np.empty((n, d), dtype=np.float64)
    loss = np.empty(n, dtype=np.float64)
    rc = _load().oracle_lsq_grad(n, b, d, _p(A, ctypes.c_float), _p(y, ctypes.c_float),
                                 _p(x, ctypes.c_double), float(scale), _p(g, ctypes.c_double),
                                 _p(loss, ctypes.c_double))
    assert rc == 0
    return g, loss


def lsq_grad_rows(A, y, x, rows, scale: float = 1.0):
    """Mini-batch gradient over the sampled rows `rows` (n x bs int32, values in [0, b)) -> (g, loss)."""
    A = np.ascontiguousarray(A, dtype=np.float32)
    y = np.ascontiguousarray(y, dtype=np.float32)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    x = _f64(x)
    n, b, d = A.shape
    assert y.shape == (n, b) and x.shape == (n, d) and rows.ndim == 2 and rows.shape[0] == n
    g = np.empty((n, d), dtype=np.float64)
    loss = np.empty(n, dtype=np.float64)
    rc = _load().oracle_lsq_grad_rows(n, b, d, _p(A, ctypes.c_float), _p(y, ctypes.c_float),
                                      _p(x, ctypes.c_double), _p(rows, ctypes.c_int32), rows.shape[1],
                                      float(scale), _p(g, ctypes.c_double), _p(loss, ctypes.c_double))
    if rc:
        raise ValueError("row index outside [0, b)")
    return g, loss


def stats(x, m=None, ref=None):
    """[sum_i ||x_i - xbar||^2, ||xbar||^2, sum_i ||x_i - ref||^2, ||ref||^2, ||m||_F^2] (float64[5])."""
    x = _f64(x)
    n, d = x.shape
    m = None if m is None else _f64(m)
    ref = None if ref is None else _f64(ref)
    assert m is None or m.shape == x.shape
    assert ref is None or ref.shape == (d,)
    out = np.zeros(5)
    null = ctypes.POINTER(ctypes.c_double)()
    rc = _load().oracle_stats(n, d, _p(x, ctypes.c_double), null if m is None else _p(m, ctypes.c_double),
                              null if ref is None else _p(ref, ctypes.c_double), _p(out, ctypes.c_double))
    assert rc == 0
    return out


def tensor_sumsq(g, m, x, offsets):
    """Layer-wise squared 2-norms: out[t, i] = (||g_i||^2, ||m_i||^2, ||x_i||^2) restricted to the
    columns [offsets[t], offsets[t+1]) of tensor t, for every node i; float64[T, n, 3].
    Plain definition, one element at a time in index order."""
    arrays = [_f64(a) for a in (g, m, x)]
    n = arrays[0].shape[0]
    offsets = [int(o) for o in offsets]
    out = np.zeros((len(offsets) - 1, n, 3))
    for t in range(len(offsets) - 1):
        for i in range(n):
            for q, a in enumerate(arrays):
                acc = 0.0
                for v in a[i, offsets[t]:offsets[t + 1]].tolist():
                    acc += v * v
                out[t, i, q] = acc
    return out


def widen16(bits, fmt: str):
    """Value of each 16-bit pattern (uint16 array) as float64: "bf16" = sign, 8 exponent bits
    (bias 127), 7 fraction bits; "f16" = IEEE binary16: sign, 5 exponent bits (bias 15), 10
    fraction bits.  Evaluated from the field definitions, no reinterpretation of bits."""
    bits = np.asarray(bits, dtype=np.uint16).astype(np.int64)
    ebits, fbits = (8, 7) if fmt == "bf16" else (5, 10)
    bias = (1 << (ebits - 1)) - 1
    sign = np.where(bits >> 15, -1.0, 1.0)
    e = (bits >> fbits) & ((1 << ebits) - 1)
    f = (bits & ((1 << fbits) - 1)).astype(np.float64) / (1 << fbits)
    normal = np.ldexp(1.0 + f, (e - bias).astype(np.int64))
    subnormal = np.ldexp(f, 1 - bias)
    val = np.where(e == 0, subnormal, normal)
    val = np.where(e == (1 << ebits) - 1, np.where(f == 0, np.inf, np.nan), val)
    return sign * val


STEP = {"decentlam": decentlam_step, "dmsgd": dmsgd_step, "awc_dmsgd": awc_dmsgd_step, "da_dmsgd": da_dmsgd_step}


def run(algo: str, x0, grad_fn, topo: Topology, gamma: float, beta: float, steps: int,
        storage: str = "fp32", m0=None, record=None):
    """Iterate `algo` for `steps` iterations from (x0, m0 = 0).

    grad_fn(k, x) returns the n x d gradient handed to iteration k (x is the
    current stacked state).  storage="fp32" rounds x, m (and the gradient) to
    float32 after every iteration, as a library that keeps its state in fp32
    arrays does; storage="fp64" never rounds.  `record(k, x, m)` is called
    after every iteration.
    """
    rnd = (lambda a: a.astype(np.float32).astype(np.float64)) if storage == "fp32" else (lambda a: a)
    x = rnd(_f64(x0))
    m = np.zeros_like(x) if m0 is None else rnd(_f64(m0))
    fn = STEP[algo]
    for k in range(steps):
        g = rnd(_f64(grad_fn(k, x)))
        x, m = fn(x, m, g, topo, gamma, beta, k)
        x, m = rnd(x), rnd(m)
        if record is not None:
            record(k, x, m)
    return x, m
