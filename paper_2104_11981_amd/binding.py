"""ctypes binding of libdecentlam.so: argument marshalling only.

Every function has the name and meaning of its C entry point (see
include/decentlam.h).  Device arrays are torch tensors used purely as handles to
HBM (`data_ptr()`, strides) and the launch stream is torch's current stream.
There is no fallback: if the shared library is missing the import of this
module fails.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np
# torch first: it ships its own HIP runtime (same soname as the system one).  Loading the
# library before torch would pull in a second runtime copy, and a process with two HIP
# runtimes has no usable device in the second.  With torch loaded, the dynamic loader
# resolves libdecentlam.so's dependency to the runtime torch already mapped.
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdecentlam.so")

DL_OK, DL_EINVAL, DL_ETOPO, DL_ECAP, DL_EHIP, DL_EALIAS = 0, -1, -2, -3, -4, -5
DL_TOPO_RING, DL_TOPO_EXP_STATIC, DL_TOPO_EXP_ONEPEER = 0, 1, 2
DL_TOPO_EXP_SYM, DL_TOPO_MESH, DL_TOPO_BIPARTITE_MATCH = 3, 4, 5
DL_FLAG_ROW_STOCHASTIC, DL_FLAG_COL_STOCHASTIC, DL_FLAG_SYMMETRIC = 1, 2, 4
DL_MAX_NODES, DL_MAX_NNZ, DL_MAX_NNZ_PALETTE, DL_MAX_WEIGHT_VALUES = 256, 512, 1536, 64

DL_GRAD_F32, DL_GRAD_BF16, DL_GRAD_F16 = 0, 1, 2
DL_STATIC_SCRATCH_BYTES = 32 << 20
DL_MAX_NODES_DEVICE = 1024

EXPORTS = ("topology_build", "topology_build_ex", "topology_metropolis", "decentlam_step", "decentlam_step_xprev",
           "dmsgd_step", "dsgd_step", "awc_dmsgd_step", "da_dmsgd_step", "decentlam_step_blocked",
           "dmsgd_step_blocked", "decentlam_step_ex", "dmsgd_step_ex", "decentlam_step_xprev_ex", "decentlam_step_multi_ex", "dmsgd_step_multi_ex", "decentlam_step_g16", "dmsgd_step_g16", "decentlam_step_multi",
           "dmsgd_step_multi", "decentlam_step_multi_workspace", "local_grad_lsq", "local_grad_lsq_rows",
           "local_grad_lsq_static", "local_grad_lsq_poll_limit", "dl_calibration_stream", "topology_pack_bytes", "topology_pack",
           "decentlam_step_packed", "dmsgd_step_packed", "dsgd_step_packed", "topology_device_bytes",
           "topology_pack_device", "decentlam_step_dev", "dmsgd_step_dev", "dsgd_step_dev",
           "awc_dmsgd_step_ex", "da_dmsgd_step_ex", "awc_dmsgd_step_multi_ex", "da_dmsgd_step_multi_ex",
           "local_grad_lsq_workspace", "decentlam_stats", "decentlam_stats_workspace", "dl_last_error")


class Layout(ctypes.Structure):
    """dl_layout of include/decentlam.h."""
    _fields_ = [("g_format", ctypes.c_int32), ("ld", ctypes.c_int64), ("ldg", ctypes.c_int64), ("bw", ctypes.c_int64)]


class DeviceTopologyStruct(ctypes.Structure):
    """dl_device_topology of include/decentlam.h."""
    _fields_ = [("magic", ctypes.c_uint32), ("n", ctypes.c_int32), ("period", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("device", ctypes.c_void_p), ("device_bytes", ctypes.c_uint64)]


class DecentLamError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"dl_status {status}: {message}")
        self.status = status


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2104_11981_amd.build). "
            "This package has no CPU or PyTorch fallback.")
    lib = ctypes.CDLL(LIB_PATH)
    i32p, f32p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float)
    vp = ctypes.c_void_p
    lib.topology_build.restype = ctypes.c_int
    lib.topology_build.argtypes = [ctypes.c_int, ctypes.c_int32, i32p, ctypes.c_int64, i32p, f32p,
                                   ctypes.c_int64, i32p, ctypes.POINTER(ctypes.c_int64),
                                   ctypes.POINTER(ctypes.c_uint32)]
    lib.topology_build_ex.restype = ctypes.c_int
    lib.topology_build_ex.argtypes = [ctypes.c_int, ctypes.c_int32, ctypes.c_uint64, ctypes.c_int32, i32p,
                                      ctypes.c_int64, i32p, f32p, ctypes.c_int64, i32p,
                                      ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_uint32)]
    lib.topology_metropolis.restype = ctypes.c_int
    lib.topology_metropolis.argtypes = [ctypes.c_int32, i32p, i32p, f32p, ctypes.POINTER(ctypes.c_uint32)]
    step = [vp, vp, vp, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, i32p, i32p, f32p,
            ctypes.c_int32, ctypes.c_float, ctypes.c_float, ctypes.c_int64, vp]
    for name in ("decentlam_step", "dmsgd_step", "awc_dmsgd_step", "da_dmsgd_step", "decentlam_step_blocked",
                 "dmsgd_step_blocked"):   # the blocked calls take bw where the others take ld
        getattr(lib, name).restype = ctypes.c_int
        getattr(lib, name).argtypes = step
    for name in ("decentlam_step_g16", "dmsgd_step_g16"):
        getattr(lib, name).restype = ctypes.c_int
        getattr(lib, name).argtypes = [vp, vp, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64,
                                       ctypes.c_int64, i32p, i32p, f32p, ctypes.c_int32, ctypes.c_float,
                                       ctypes.c_float, ctypes.c_int64, vp]
    for name in ("decentlam_step_multi", "dmsgd_step_multi"):
        getattr(lib, name).restype = ctypes.c_int
        getattr(lib, name).argtypes = [vp, vp, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64,
                                       ctypes.c_int32, ctypes.POINTER(ctypes.c_int64), vp, vp, ctypes.c_size_t,
                                       i32p, i32p, f32p, ctypes.c_int32, ctypes.c_float, ctypes.c_float,
                                       ctypes.c_int64, vp]
    layp = ctypes.POINTER(Layout)
    for name in ("decentlam_step_ex", "dmsgd_step_ex", "awc_dmsgd_step_ex", "da_dmsgd_step_ex"):
        getattr(lib, name).restype = ctypes.c_int
        getattr(lib, name).argtypes = [vp, vp, vp, ctypes.c_int32, ctypes.c_int64, layp, i32p, i32p, f32p,
                                       ctypes.c_int32, ctypes.c_float, ctypes.c_float, ctypes.c_int64, vp]
    for name in ("decentlam_step_multi_ex", "dmsgd_step_multi_ex", "awc_dmsgd_step_multi_ex", "da_dmsgd_step_multi_ex"):
        getattr(lib, name).restype = ctypes.c_int
        getattr(lib, name).argtypes = [vp, vp, vp, ctypes.c_int32, layp, ctypes.c_int32,
                                       ctypes.POINTER(ctypes.c_int64), vp, vp, ctypes.c_size_t, i32p, i32p, f32p,
                                       ctypes.c_int32, ctypes.c_float, ctypes.c_float, ctypes.c_int64, vp]
    lib.decentlam_step_xprev_ex.restype = ctypes.c_int
    lib.decentlam_step_xprev_ex.argtypes = [vp, vp, vp, ctypes.c_int32, ctypes.c_int64, layp, i32p, i32p, f32p,
                                            ctypes.c_int32, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                            ctypes.c_int64, vp]
    lib.decentlam_step_multi_workspace.restype = ctypes.c_size_t
    lib.decentlam_step_multi_workspace.argtypes = [ctypes.c_int32, ctypes.c_int64, ctypes.c_int32]
    lib.decentlam_step_xprev.restype = ctypes.c_int
    lib.decentlam_step_xprev.argtypes = [vp, vp, vp, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, i32p, i32p,
                                         f32p, ctypes.c_int32, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                         ctypes.c_int64, vp]
    lib.dsgd_step.restype = ctypes.c_int
    lib.dsgd_step.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, i32p, i32p, f32p,
                              ctypes.c_int32, ctypes.c_float, ctypes.c_int64, vp]
    lib.local_grad_lsq_workspace.restype = ctypes.c_size_t
    lib.local_grad_lsq_workspace.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64]
    lib.local_grad_lsq.restype = ctypes.c_int
    lib.local_grad_lsq.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64,
                                   ctypes.c_int64, ctypes.c_int64, ctypes.c_float, vp, ctypes.c_size_t, vp]
    lib.local_grad_lsq_poll_limit.restype = ctypes.c_int
    lib.local_grad_lsq_poll_limit.argtypes = [ctypes.c_int]
    lib.local_grad_lsq_static.restype = ctypes.c_int
    lib.local_grad_lsq_static.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64,
                                          ctypes.c_int64, ctypes.c_int64, ctypes.c_float, vp]
    lib.local_grad_lsq_rows.restype = ctypes.c_int
    lib.local_grad_lsq_rows.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int64,
                                        ctypes.c_int64, ctypes.c_int64, vp, ctypes.c_int32, ctypes.c_float, vp,
                                        ctypes.c_size_t, vp]
    lib.decentlam_stats_workspace.restype = ctypes.c_size_t
    lib.decentlam_stats_workspace.argtypes = [ctypes.c_int32, ctypes.c_int64]
    lib.decentlam_stats.restype = ctypes.c_int
    lib.decentlam_stats.argtypes = [vp, vp, vp, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, vp, vp,
                                    ctypes.c_size_t, vp]
    lib.topology_pack_bytes.restype = ctypes.c_size_t
    lib.topology_pack_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32]
    lib.topology_pack.restype = ctypes.c_int
    lib.topology_pack.argtypes = [ctypes.c_int32, i32p, i32p, f32p, ctypes.c_int32, vp, ctypes.c_size_t]
    for name in ("decentlam_step_packed", "dmsgd_step_packed"):
        getattr(lib, name).restype = ctypes.c_int
        getattr(lib, name).argtypes = [vp, vp, vp, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, vp, ctypes.c_float,
                                       ctypes.c_float, ctypes.c_int64, vp]
    lib.dsgd_step_packed.restype = ctypes.c_int
    lib.dsgd_step_packed.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, vp, ctypes.c_float,
                                     ctypes.c_int64, vp]
    dtp = ctypes.POINTER(DeviceTopologyStruct)
    lib.topology_device_bytes.restype = ctypes.c_size_t
    lib.topology_device_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int64]
    lib.topology_pack_device.restype = ctypes.c_int
    lib.topology_pack_device.argtypes = [ctypes.c_int32, i32p, i32p, f32p, ctypes.c_int32, vp, ctypes.c_size_t, dtp]
    for name in ("decentlam_step_dev", "dmsgd_step_dev"):
        getattr(lib, name).restype = ctypes.c_int
        getattr(lib, name).argtypes = [vp, vp, vp, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, dtp, ctypes.c_float,
                                       ctypes.c_float, ctypes.c_int64, vp]
    lib.dsgd_step_dev.restype = ctypes.c_int
    lib.dsgd_step_dev.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, dtp, ctypes.c_float,
                                  ctypes.c_int64, vp]
    lib.dl_calibration_stream.restype = ctypes.c_int
    lib.dl_calibration_stream.argtypes = [ctypes.c_int, ctypes.c_int, vp, vp, vp, ctypes.c_int32, ctypes.c_int64,
                                          ctypes.c_int64, ctypes.POINTER(ctypes.c_int64), vp]
    lib.dl_last_error.restype = ctypes.c_char_p
    lib.dl_last_error.argtypes = []
    return lib


_lib = _load()


def last_error() -> str:
    return _lib.dl_last_error().decode()


def _check(rc: int):
    if rc != DL_OK:
        raise DecentLamError(rc, last_error())


@dataclass
class Topology:
    """Host-side CSR neighbour lists, exactly the arrays the C ABI takes."""
    n: int
    period: int
    row_ptr: np.ndarray   # int32 [period*(n+1)]
    col_idx: np.ndarray   # int32 [nnz]
    w: np.ndarray         # float32 [nnz]
    flags: int = 0

    def _args(self):
        # the ctypes pointers are built once per (array identity) -- the step functions are called
        # every iteration and the small workloads are launch-latency bound
        key = (id(self.row_ptr), id(self.col_idx), id(self.w), self.period)
        cached = self.__dict__.get("_cached_args")
        if cached is None or cached[0] != key:
            cached = (key, (self.row_ptr.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                            self.col_idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                            self.w.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                            self.period))
            self.__dict__["_cached_args"] = cached
        return cached[1]


def topology_build(kind: int, n: int, seed: int = 0, phases: int = 1) -> Topology:
    """topology_build (or topology_build_ex for the seeded bipartite random match)."""
    period, nnz, flags = ctypes.c_int32(0), ctypes.c_int64(0), ctypes.c_uint32(0)
    if kind == DL_TOPO_BIPARTITE_MATCH:
        call = lambda *a: _lib.topology_build_ex(kind, n, seed, phases, *a)
    else:
        call = lambda *a: _lib.topology_build(kind, n, *a)
    _check(call(None, 0, None, None, 0, ctypes.byref(period), ctypes.byref(nnz), ctypes.byref(flags)))
    row_ptr = np.zeros(period.value * (n + 1), dtype=np.int32)
    col_idx = np.zeros(nnz.value, dtype=np.int32)
    w = np.zeros(nnz.value, dtype=np.float32)
    _check(call(row_ptr.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), row_ptr.size,
                col_idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                w.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), col_idx.size,
                ctypes.byref(period), ctypes.byref(nnz), ctypes.byref(flags)))
    return Topology(n, period.value, row_ptr, col_idx, w, flags.value)


def topology_metropolis(n: int, row_ptr, col_idx) -> Topology:
    """Metropolis-Hastings weights for a caller-supplied undirected one-phase graph."""
    row_ptr = np.ascontiguousarray(row_ptr, np.int32)
    col_idx = np.ascontiguousarray(col_idx, np.int32)
    w = np.zeros(col_idx.size, dtype=np.float32)
    flags = ctypes.c_uint32(0)
    _check(_lib.topology_metropolis(n, row_ptr.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                    col_idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                    w.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), ctypes.byref(flags)))
    return Topology(n, 1, row_ptr, col_idx, w, flags.value)


def make_topology(n: int, row_ptr, col_idx, w, period: int = 1) -> Topology:
    """Wrap caller-supplied CSR arrays (validated by the step functions)."""
    return Topology(n, period, np.ascontiguousarray(row_ptr, np.int32),
                    np.ascontiguousarray(col_idx, np.int32), np.ascontiguousarray(w, np.float32))


_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)
_raw_device = getattr(torch._C, "_cuda_getDevice", None)


def _stream() -> int:
    """Handle of torch's current stream on the current device.  The small workloads are bound by the
    host's call rate, and torch.cuda.current_stream() alone costs about 3 us: the two C accessors
    behind it are used directly where this torch has them."""
    if _raw_stream is not None and _raw_device is not None:
        return _raw_stream(_raw_device())
    return torch.cuda.current_stream().cuda_stream


def _matrix_args(t, name):
    if t.dtype != torch.float32 or not t.is_cuda or t.dim() != 2:
        raise TypeError(f"{name}: need a 2-D float32 device tensor")
    if t.shape[1] > 0 and t.stride(1) != 1:
        raise TypeError(f"{name}: columns must be contiguous")
    return t.data_ptr(), t.shape[0], t.shape[1], (t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1]))


def _step(fn, x, m, g, topo: Topology, gamma: float, beta: float, k: int, stream):
    px, n, d, ld = _matrix_args(x, "x")
    pm, nm, dm, ldm = _matrix_args(m, "m")
    pg, ng, dg, ldg = _matrix_args(g, "g")
    if (nm, dm, ldm) != (n, d, ld) or (ng, dg, ldg) != (n, d, ld):
        raise TypeError("x, m and g must share shape and row stride")
    if topo.n != n:
        raise DecentLamError(DL_ETOPO, f"topology has {topo.n} nodes, arrays have {n} rows")
    _check(fn(px, pm, pg, n, d, ld, *topo._args(), gamma, beta, k,
              _stream() if stream is None else stream))


def decentlam_step(x, m, g, topo: Topology, gamma: float, beta: float, k: int = 0, stream=None):
    """One DecentLaM iteration in place on device tensors x, m (n x d fp32), asynchronous."""
    _step(_lib.decentlam_step, x, m, g, topo, gamma, beta, k, stream)


def dmsgd_step(x, m, g, topo: Topology, gamma: float, beta: float, k: int = 0, stream=None):
    """One DmSGD iteration in place on device tensors x, m (n x d fp32), asynchronous."""
    _step(_lib.dmsgd_step, x, m, g, topo, gamma, beta, k, stream)


ROW_ALIGN_ELEMENTS = 16384   # 64 KiB of fp32: the row alignment the step kernel's large launches want


def recommended_ld(d: int) -> int:
    """Row stride (in elements) the header recommends for an n x d fp32 array: rows on 64 KiB boundaries
    from 65536 columns on (but never a multiple of 127 or 129 times 64 KiB, nor 4 MiB exactly: with such
    strides the rows of a column fall on the same memory channels; measured on 32 nodes x 1 M columns: 0.49
    and 0.64-0.69 of the HBM peak against 0.71-0.80 with one 64 KiB unit more), on 256-byte boundaries below."""
    if d < (1 << 16):
        return (d + 63) // 64 * 64
    units = (d + ROW_ALIGN_ELEMENTS - 1) // ROW_ALIGN_ELEMENTS
    while units % 127 == 0 or units % 129 == 0 or units == 64:
        units += 1
    return units * ROW_ALIGN_ELEMENTS


def empty_rows(n: int, d: int, device="cuda", dtype=None, fill=None):
    """An n x d view (row-major, rows recommended_ld(d) apart, first row on a 64 KiB boundary) of a fresh
    allocation: the layout in which the row-major step calls run fastest.  `fill`: initial value of the
    view (None: uninitialised).  Memory handling only; no arithmetic of the method."""
    dtype = torch.float32 if dtype is None else dtype
    ld = recommended_ld(d)
    item = torch.empty((), dtype=dtype).element_size()
    slack = 65536 // item
    buf = torch.empty(n * ld + slack, dtype=dtype, device=device)
    first = (-(buf.data_ptr() // item)) % slack if buf.data_ptr() % item == 0 else 0
    view = buf[first:first + n * ld].view(n, ld)[:, :d]
    if fill is not None:
        view.fill_(fill)
    return view


def to_blocked(a, bw: int, fill: float = 0.0):
    """Logical n x d tensor -> blocked layout tensor of shape (ceil(d / bw), n, bw) (a copy; padding = fill)."""
    n, d = a.shape
    nb = (d + bw - 1) // bw
    out = torch.full((n, nb * bw), fill, dtype=a.dtype, device=a.device)
    out[:, :d] = a
    return out.view(n, nb, bw).permute(1, 0, 2).contiguous()


def from_blocked(b, d: int):
    """Blocked layout tensor (nb, n, bw) -> logical n x d tensor (a copy)."""
    nb, n, bw = b.shape
    return b.permute(1, 0, 2).reshape(n, nb * bw)[:, :d].contiguous()


def _step_blocked(fn, x, m, g, d, topo, gamma, beta, k, stream):
    for name, t in (("x", x), ("m", m), ("g", g)):
        if t.dtype != torch.float32 or not t.is_cuda or t.dim() != 3 or not t.is_contiguous():
            raise TypeError(f"{name}: need a contiguous 3-D (blocks, n, bw) float32 device tensor")
    if x.shape != m.shape or x.shape != g.shape:
        raise TypeError("x, m and g must share their shape")
    nb, n, bw = x.shape
    if not (0 <= d <= nb * bw) or (nb > 0 and d <= (nb - 1) * bw):
        raise DecentLamError(DL_EINVAL, f"d = {d} does not end in the last of {nb} blocks of {bw} columns")
    if topo.n != n:
        raise DecentLamError(DL_ETOPO, f"topology has {topo.n} nodes, arrays have {n} rows")
    _check(fn(x.data_ptr(), m.data_ptr(), g.data_ptr(), n, d, bw, *topo._args(), gamma, beta, k,
              _stream() if stream is None else stream))


def decentlam_step_blocked(x, m, g, d: int, topo: Topology, gamma: float, beta: float, k: int = 0, stream=None):
    """decentlam_step on arrays in the blocked layout: tensors of shape (ceil(d / bw), n, bw)."""
    _step_blocked(_lib.decentlam_step_blocked, x, m, g, d, topo, gamma, beta, k, stream)


def dmsgd_step_blocked(x, m, g, d: int, topo: Topology, gamma: float, beta: float, k: int = 0, stream=None):
    """dmsgd_step on arrays in the blocked layout: tensors of shape (ceil(d / bw), n, bw)."""
    _step_blocked(_lib.dmsgd_step_blocked, x, m, g, d, topo, gamma, beta, k, stream)


def _step_ex(fn, x, m, g, d, topo, gamma, beta, k, stream, gamma_prev=None):
    """Marshal the general forms: 2-D tensors (n, d) are row-major arrays, 3-D tensors (blocks, n, bw)
    are arrays in the blocked layout (then `d` says where the last block ends); g may be 16-bit."""
    if g.dtype not in _GRAD_FORMAT:
        raise TypeError("g: need a float32, bfloat16 or float16 tensor")
    for name, t in (("x", x), ("m", m)):
        if t.dtype != torch.float32 or not t.is_cuda:
            raise TypeError(f"{name}: need a float32 device tensor")
    if x.dim() == 3:
        if not (x.is_contiguous() and m.is_contiguous() and g.is_contiguous()) or x.shape != m.shape or x.shape != g.shape:
            raise TypeError("blocked layout: x, m and g must be contiguous (blocks, n, bw) tensors of one shape")
        nb, n, bw = x.shape
        if d is None or not ((nb - 1) * bw < d <= nb * bw):
            raise DecentLamError(DL_EINVAL, f"d = {d} does not end in the last of {nb} blocks of {bw} columns")
        lay = Layout(_GRAD_FORMAT[g.dtype], 0, 0, bw)
    else:
        px, n, cols, ld = _matrix_args(x, "x")
        pm, nm, dm, ldm = _matrix_args(m, "m")
        if (nm, dm, ldm) != (n, cols, ld):
            raise TypeError("x and m must share shape and row stride")
        _, fmt, ldg = _grad_args(g, n, cols)
        d = cols
        lay = Layout(fmt, ld, ldg, 0)
    if topo.n != n:
        raise DecentLamError(DL_ETOPO, f"topology has {topo.n} nodes, arrays have {n} rows")
    st = _stream() if stream is None else stream
    if gamma_prev is None:
        _check(fn(x.data_ptr(), m.data_ptr(), g.data_ptr(), n, d, ctypes.byref(lay), *topo._args(), gamma, beta, k, st))
    else:
        _check(fn(x.data_ptr(), m.data_ptr(), g.data_ptr(), n, d, ctypes.byref(lay), *topo._args(), gamma,
                  gamma_prev, beta, k, st))


def decentlam_step_ex(x, m, g, topo: Topology, gamma: float, beta: float, k: int = 0, d=None, stream=None):
    """General DecentLaM step: row-major (2-D tensors) or blocked (3-D tensors, pass d), fp32 or 16-bit g."""
    _step_ex(_lib.decentlam_step_ex, x, m, g, d, topo, gamma, beta, k, stream)


def dmsgd_step_ex(x, m, g, topo: Topology, gamma: float, beta: float, k: int = 0, d=None, stream=None):
    """General DmSGD step, see decentlam_step_ex."""
    _step_ex(_lib.dmsgd_step_ex, x, m, g, d, topo, gamma, beta, k, stream)


def awc_dmsgd_step_ex(x, m, g, topo: Topology, gamma: float, beta: float, k: int = 0, d=None, stream=None):
    """General AWC-DmSGD step, see decentlam_step_ex."""
    _step_ex(_lib.awc_dmsgd_step_ex, x, m, g, d, topo, gamma, beta, k, stream)


def da_dmsgd_step_ex(x, m, g, topo: Topology, gamma: float, beta: float, k: int = 0, d=None, stream=None):
    """General DA-DmSGD step, see decentlam_step_ex."""
    _step_ex(_lib.da_dmsgd_step_ex, x, m, g, d, topo, gamma, beta, k, stream)


def decentlam_step_xprev_ex(x, x_prev, g, topo: Topology, gamma: float, beta: float, k: int = 0,
                            gamma_prev: float | None = None, d=None, stream=None):
    """General momentum-free DecentLaM step (x_prev is overwritten with x^{k+1}), see decentlam_step_ex."""
    _step_ex(_lib.decentlam_step_xprev_ex, x, x_prev, g, d, topo, gamma, beta, k, stream,
             gamma if gamma_prev is None else gamma_prev)


def _step_multi_ex(fn, x, m, g, offsets, topo, gamma, beta, k, norms, workspace, stream):
    if g.dtype not in _GRAD_FORMAT:
        raise TypeError("g: need a float32, bfloat16 or float16 tensor")
    for name, t in (("x", x), ("m", m)):
        if t.dtype != torch.float32 or not t.is_cuda:
            raise TypeError(f"{name}: need a float32 device tensor")
    offsets = np.ascontiguousarray(offsets, np.int64)
    if offsets.ndim != 1 or offsets.size < 2:
        raise TypeError("offsets: need num_tensors + 1 column offsets")
    num = offsets.size - 1
    if x.dim() == 3:
        if not (x.is_contiguous() and m.is_contiguous() and g.is_contiguous()) or x.shape != m.shape or x.shape != g.shape:
            raise TypeError("blocked layout: x, m and g must be contiguous (blocks, n, bw) tensors of one shape")
        nb, n, bw = x.shape
        if offsets[-1] > nb * bw:
            raise DecentLamError(DL_EINVAL, f"offsets end at {offsets[-1]}, arrays hold {nb * bw} columns")
        lay = Layout(_GRAD_FORMAT[g.dtype], 0, 0, bw)
    else:
        px, n, cols, ld = _matrix_args(x, "x")
        pm, nm, dm, ldm = _matrix_args(m, "m")
        if (nm, dm, ldm) != (n, cols, ld):
            raise TypeError("x and m must share shape and row stride")
        _, fmt, ldg = _grad_args(g, n, cols)
        if offsets[-1] > cols:
            raise DecentLamError(DL_EINVAL, f"offsets end at {offsets[-1]}, arrays have {cols} columns")
        lay = Layout(fmt, max(ld, cols), max(ldg, cols), 0)
    if topo.n != n:
        raise DecentLamError(DL_ETOPO, f"topology has {topo.n} nodes, arrays have {n} rows")
    pn = pw = wb = 0
    if norms is not None:
        if norms.dtype != torch.float64 or not norms.is_cuda or not norms.is_contiguous() or norms.numel() != num * n * 3:
            raise TypeError("norms: need a contiguous float64 device tensor of num_tensors x n x 3 elements")
        if workspace is None:
            raise TypeError("workspace: pass a uint8 device tensor (size from decentlam_step_multi_workspace)")
        pn, pw, wb = norms.data_ptr(), workspace.data_ptr(), workspace.numel() * workspace.element_size()
    _check(fn(x.data_ptr(), m.data_ptr(), g.data_ptr(), n, ctypes.byref(lay), num,
              offsets.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), pn, pw, wb, *topo._args(), gamma, beta, k,
              _stream() if stream is None else stream))


def decentlam_step_multi_ex(x, m, g, offsets, topo: Topology, gamma: float, beta: float, k: int = 0,
                            norms=None, workspace=None, stream=None):
    """General multi-tensor DecentLaM step: 2-D tensors are row-major arrays, 3-D (blocks, n, bw) tensors
    the blocked layout (the table then starts at column 0); g may be 16-bit."""
    _step_multi_ex(_lib.decentlam_step_multi_ex, x, m, g, offsets, topo, gamma, beta, k, norms, workspace, stream)


def dmsgd_step_multi_ex(x, m, g, offsets, topo: Topology, gamma: float, beta: float, k: int = 0,
                        norms=None, workspace=None, stream=None):
    """General multi-tensor DmSGD step, see decentlam_step_multi_ex."""
    _step_multi_ex(_lib.dmsgd_step_multi_ex, x, m, g, offsets, topo, gamma, beta, k, norms, workspace, stream)


def topology_pack_bytes(n: int, period: int) -> int:
    return int(_lib.topology_pack_bytes(n, period))


@dataclass
class PackedTopology:
    """A topology validated and encoded once by topology_pack: an opaque host buffer for the *_step_packed calls."""
    n: int
    period: int
    buffer: np.ndarray   # uint8, owned here

    def _ptr(self):
        cached = self.__dict__.get("_cached_ptr")
        if cached is None:
            cached = self.__dict__["_cached_ptr"] = self.buffer.ctypes.data
        return cached


def topology_pack(topo: Topology) -> PackedTopology:
    """topology_pack: check and encode every phase of `topo` once."""
    nbytes = topology_pack_bytes(topo.n, topo.period)
    if nbytes == 0:
        raise DecentLamError(DL_ETOPO, f"topology_pack: n = {topo.n}, period = {topo.period} cannot be packed")
    buf = np.zeros(nbytes, dtype=np.uint8)
    _check(_lib.topology_pack(topo.n, *topo._args(), buf.ctypes.data, nbytes))
    return PackedTopology(topo.n, topo.period, buf)


def _step_packed(fn, x, m, g, packed: PackedTopology, gamma, beta, k, stream):
    px, n, d, ld = _matrix_args(x, "x")
    pm, nm, dm, ldm = _matrix_args(m, "m")
    pg, ng, dg, ldg = _matrix_args(g, "g")
    if (nm, dm, ldm) != (n, d, ld) or (ng, dg, ldg) != (n, d, ld):
        raise TypeError("x, m and g must share shape and row stride")
    _check(fn(px, pm, pg, n, d, ld, packed._ptr(), gamma, beta, k, _stream() if stream is None else stream))


def decentlam_step_packed(x, m, g, packed: PackedTopology, gamma: float, beta: float, k: int = 0, stream=None):
    """decentlam_step with W from topology_pack (no per-call validation of W)."""
    _step_packed(_lib.decentlam_step_packed, x, m, g, packed, gamma, beta, k, stream)


def dmsgd_step_packed(x, m, g, packed: PackedTopology, gamma: float, beta: float, k: int = 0, stream=None):
    """dmsgd_step with W from topology_pack."""
    _step_packed(_lib.dmsgd_step_packed, x, m, g, packed, gamma, beta, k, stream)


def dsgd_step_packed(x, g, packed: PackedTopology, gamma: float, k: int = 0, stream=None):
    """dsgd_step with W from topology_pack."""
    px, n, d, ld = _matrix_args(x, "x")
    pg, ng, dg, ldg = _matrix_args(g, "g")
    if (ng, dg, ldg) != (n, d, ld):
        raise TypeError("x and g must share shape and row stride")
    _check(_lib.dsgd_step_packed(px, pg, n, d, ld, packed._ptr(), gamma, k, _stream() if stream is None else stream))


def topology_device_bytes(n: int, period: int, nnz_total: int) -> int:
    return int(_lib.topology_device_bytes(n, period, nnz_total))


@dataclass
class DeviceTopology:
    """A topology held in device memory by topology_pack_device, for the *_step_dev calls (up to 1024 nodes, lists
    of any length).  `buffer` is the caller-owned device buffer (a uint8 tensor, kept alive here), `desc` the host
    descriptor the C calls take."""
    n: int
    period: int
    buffer: "torch.Tensor"
    desc: DeviceTopologyStruct


def topology_pack_device(topo: Topology, device="cuda") -> DeviceTopology:
    """topology_pack_device: validate every phase and copy the lists into a fresh device buffer (synchronous)."""
    nbytes = topology_device_bytes(topo.n, topo.period, int(topo.col_idx.size))
    if nbytes == 0:
        raise DecentLamError(DL_ETOPO, f"topology_pack_device: n = {topo.n}, period = {topo.period} cannot be packed")
    buf = torch.empty(nbytes, dtype=torch.uint8, device=device)
    desc = DeviceTopologyStruct()
    _check(_lib.topology_pack_device(topo.n, *topo._args(), buf.data_ptr(), nbytes, ctypes.byref(desc)))
    return DeviceTopology(topo.n, topo.period, buf, desc)


def _step_dev(fn, x, m, g, W: DeviceTopology, gamma, beta, k, stream):
    px, n, d, ld = _matrix_args(x, "x")
    pm, nm, dm, ldm = _matrix_args(m, "m")
    pg, ng, dg, ldg = _matrix_args(g, "g")
    if (nm, dm, ldm) != (n, d, ld) or (ng, dg, ldg) != (n, d, ld):
        raise TypeError("x, m and g must share shape and row stride")
    _check(fn(px, pm, pg, n, d, ld, ctypes.byref(W.desc), gamma, beta, k, _stream() if stream is None else stream))


def decentlam_step_dev(x, m, g, W: DeviceTopology, gamma: float, beta: float, k: int = 0, stream=None):
    """decentlam_step with the neighbour lists in device memory (graphs beyond the ordinary calls' limits)."""
    _step_dev(_lib.decentlam_step_dev, x, m, g, W, gamma, beta, k, stream)


def dmsgd_step_dev(x, m, g, W: DeviceTopology, gamma: float, beta: float, k: int = 0, stream=None):
    """dmsgd_step with the neighbour lists in device memory."""
    _step_dev(_lib.dmsgd_step_dev, x, m, g, W, gamma, beta, k, stream)


def dsgd_step_dev(x, g, W: DeviceTopology, gamma: float, k: int = 0, stream=None):
    """dsgd_step with the neighbour lists in device memory."""
    px, n, d, ld = _matrix_args(x, "x")
    pg, ng, dg, ldg = _matrix_args(g, "g")
    if (ng, dg, ldg) != (n, d, ld):
        raise TypeError("x and g must share shape and row stride")
    _check(_lib.dsgd_step_dev(px, pg, n, d, ld, ctypes.byref(W.desc), gamma, k, _stream() if stream is None else stream))


class PreparedCall:
    """A library call whose arguments were marshalled once.  `call(k)` issues it for iteration k on torch's current
    stream (or on the stream fixed at preparation) and checks the status; everything else about the call -- the
    arrays, their shapes and strides, W, gamma, beta -- is as it was when the call was prepared.  The small
    workloads are bound by the host's call rate, and building the argument list is a third of a call's cost.
    Marshalling only: the tensors are kept alive here, nothing is computed."""
    __slots__ = ("_fn", "_head", "_takes_k", "_stream", "_keep")

    def __init__(self, fn, head, takes_k, stream, keep):
        self._fn, self._head, self._takes_k, self._stream, self._keep = fn, head, takes_k, stream, keep

    def __call__(self, k: int = 0):
        st = self._stream if self._stream is not None else _stream()
        rc = self._fn(*self._head, k, st) if self._takes_k else self._fn(*self._head, st)
        if rc != DL_OK:
            raise DecentLamError(rc, last_error())


def prepare_step(algo: str, x, m, g, topo, gamma: float, beta: float, stream=None) -> PreparedCall:
    """decentlam_step / dmsgd_step (`algo` = "decentlam" or "dmsgd") with everything but k fixed; `topo` is a
    Topology or, to skip the per-call validation of W as well, a PackedTopology."""
    if algo not in ("decentlam", "dmsgd"):
        raise ValueError("algo: 'decentlam' or 'dmsgd'")
    px, n, d, ld = _matrix_args(x, "x")
    pm, nm, dm, ldm = _matrix_args(m, "m")
    pg, ng, dg, ldg = _matrix_args(g, "g")
    if (nm, dm, ldm) != (n, d, ld) or (ng, dg, ldg) != (n, d, ld):
        raise TypeError("x, m and g must share shape and row stride")
    if topo.n != n:
        raise DecentLamError(DL_ETOPO, f"topology has {topo.n} nodes, arrays have {n} rows")
    vp = ctypes.c_void_p
    head = [vp(px), vp(pm), vp(pg), ctypes.c_int32(n), ctypes.c_int64(d), ctypes.c_int64(ld)]
    if isinstance(topo, PackedTopology):
        fn = getattr(_lib, algo + "_step_packed")
        head.append(vp(topo._ptr()))
    else:
        fn = getattr(_lib, algo + "_step")
        rp, ci, w, period = topo._args()
        head += [rp, ci, w, ctypes.c_int32(period)]
    head += [ctypes.c_float(gamma), ctypes.c_float(beta)]
    return PreparedCall(fn, tuple(head), True, stream, (x, m, g, topo))


def prepare_local_grad_lsq(A, y, x, g, loss=None, scale: float = 1.0, workspace=None, stream=None) -> PreparedCall:
    """local_grad_lsq with all of its arguments fixed (the iteration number plays no role: call() or call(k))."""
    if A.dtype != torch.float32 or A.dim() != 3 or not A.is_cuda or A.stride(2) != 1:
        raise TypeError("A: need a 3-D float32 device tensor with contiguous last axis")
    n, b, d = A.shape
    if b > 1 and n > 1 and A.stride(0) != b * A.stride(1):
        raise TypeError("A: node stride must be b * row stride")
    ldA = A.stride(1) if b > 1 else max(A.stride(1), d)
    if y.dtype != torch.float32 or tuple(y.shape) != (n, b) or not y.is_contiguous() or not y.is_cuda:
        raise TypeError("y: need a contiguous n x b float32 device tensor")
    px, nx, dx, ld = _matrix_args(x, "x")
    pg, ng, dg, ldg = _matrix_args(g, "g")
    if (nx, dx) != (n, d) or (ng, dg, ldg) != (n, d, ld):
        raise TypeError("x and g must be n x d with the same row stride")
    pl = 0
    if loss is not None:
        if loss.dtype != torch.float32 or tuple(loss.shape) != (n,) or not loss.is_contiguous() or not loss.is_cuda:
            raise TypeError("loss: need a contiguous float32 device tensor of n elements")
        pl = loss.data_ptr()
    if workspace is None:
        raise TypeError("workspace: pass a uint8 device tensor (size from local_grad_lsq_workspace)")
    vp = ctypes.c_void_p
    head = (vp(A.data_ptr()), vp(y.data_ptr()), vp(px), vp(pg), vp(pl), ctypes.c_int32(n), ctypes.c_int32(b),
            ctypes.c_int64(d), ctypes.c_int64(ldA), ctypes.c_int64(ld), ctypes.c_float(scale),
            vp(workspace.data_ptr()), ctypes.c_size_t(workspace.numel() * workspace.element_size()))
    return PreparedCall(_lib.local_grad_lsq, head, False, stream, (A, y, x, g, loss, workspace))


def awc_dmsgd_step_multi_ex(x, m, g, offsets, topo: Topology, gamma: float, beta: float, k: int = 0,
                            norms=None, workspace=None, stream=None):
    """General multi-tensor AWC-DmSGD step, see decentlam_step_multi_ex."""
    _step_multi_ex(_lib.awc_dmsgd_step_multi_ex, x, m, g, offsets, topo, gamma, beta, k, norms, workspace, stream)


def da_dmsgd_step_multi_ex(x, m, g, offsets, topo: Topology, gamma: float, beta: float, k: int = 0,
                           norms=None, workspace=None, stream=None):
    """General multi-tensor DA-DmSGD step, see decentlam_step_multi_ex."""
    _step_multi_ex(_lib.da_dmsgd_step_multi_ex, x, m, g, offsets, topo, gamma, beta, k, norms, workspace, stream)


def awc_dmsgd_step(x, m, g, topo: Topology, gamma: float, beta: float, k: int = 0, stream=None):
    """One AWC-DmSGD iteration (m <- beta m + g; x <- W x - gamma m) in place, asynchronous."""
    _step(_lib.awc_dmsgd_step, x, m, g, topo, gamma, beta, k, stream)


def da_dmsgd_step(x, m, g, topo: Topology, gamma: float, beta: float, k: int = 0, stream=None):
    """One DA-DmSGD iteration (mh = beta m + g; x <- W (x - gamma mh); m <- W mh) in place, asynchronous."""
    _step(_lib.da_dmsgd_step, x, m, g, topo, gamma, beta, k, stream)


_GRAD_FORMAT = {torch.float32: DL_GRAD_F32, torch.bfloat16: DL_GRAD_BF16, torch.float16: DL_GRAD_F16}


def _grad_args(g, n, d):
    if g.dtype not in _GRAD_FORMAT or not g.is_cuda or g.dim() != 2:
        raise TypeError("g: need a 2-D float32, bfloat16 or float16 device tensor")
    if tuple(g.shape) != (n, d):
        raise TypeError("g must have x's shape")
    if d > 0 and g.stride(1) != 1:
        raise TypeError("g: columns must be contiguous")
    return g.data_ptr(), _GRAD_FORMAT[g.dtype], (g.stride(0) if n > 1 else max(g.stride(0), d))


def _step_g16(fn, x, m, g, topo, gamma, beta, k, stream):
    px, n, d, ld = _matrix_args(x, "x")
    pm, nm, dm, ldm = _matrix_args(m, "m")
    if (nm, dm, ldm) != (n, d, ld):
        raise TypeError("x and m must share shape and row stride")
    pg, fmt, ldg = _grad_args(g, n, d)
    if topo.n != n:
        raise DecentLamError(DL_ETOPO, f"topology has {topo.n} nodes, arrays have {n} rows")
    _check(fn(px, pm, pg, fmt, n, d, ld, ldg, *topo._args(), gamma, beta, k,
              _stream() if stream is None else stream))


def decentlam_step_g16(x, m, g, topo: Topology, gamma: float, beta: float, k: int = 0, stream=None):
    """decentlam_step with g stored as bfloat16 / float16 (its dtype selects the format)."""
    _step_g16(_lib.decentlam_step_g16, x, m, g, topo, gamma, beta, k, stream)


def dmsgd_step_g16(x, m, g, topo: Topology, gamma: float, beta: float, k: int = 0, stream=None):
    """dmsgd_step with g stored as bfloat16 / float16 (its dtype selects the format)."""
    _step_g16(_lib.dmsgd_step_g16, x, m, g, topo, gamma, beta, k, stream)


def decentlam_step_multi_workspace(n: int, d: int, num_tensors: int) -> int:
    return int(_lib.decentlam_step_multi_workspace(n, d, num_tensors))


def _step_multi(fn, x, m, g, offsets, topo, gamma, beta, k, norms, workspace, stream):
    px, n, cols, ld = _matrix_args(x, "x")
    pm, nm, dm, ldm = _matrix_args(m, "m")
    if (nm, dm, ldm) != (n, cols, ld):
        raise TypeError("x and m must share shape and row stride")
    pg, fmt, ldg = _grad_args(g, n, cols)
    if topo.n != n:
        raise DecentLamError(DL_ETOPO, f"topology has {topo.n} nodes, arrays have {n} rows")
    offsets = np.ascontiguousarray(offsets, np.int64)
    if offsets.ndim != 1 or offsets.size < 2:
        raise TypeError("offsets: need num_tensors + 1 column offsets")
    num = offsets.size - 1
    if offsets[-1] > cols:
        raise DecentLamError(DL_EINVAL, f"offsets end at {offsets[-1]}, arrays have {cols} columns")
    pn = pw = wb = 0
    if norms is not None:
        if norms.dtype != torch.float64 or not norms.is_cuda or not norms.is_contiguous() or norms.numel() != num * n * 3:
            raise TypeError("norms: need a contiguous float64 device tensor of num_tensors x n x 3 elements")
        if workspace is None:
            raise TypeError("workspace: pass a uint8 device tensor (size from decentlam_step_multi_workspace)")
        pn, pw, wb = norms.data_ptr(), workspace.data_ptr(), workspace.numel() * workspace.element_size()
    _check(fn(px, pm, pg, fmt, n, max(ld, cols), max(ldg, cols), num,
              offsets.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), pn, pw, wb, *topo._args(), gamma, beta, k,
              _stream() if stream is None else stream))


def decentlam_step_multi(x, m, g, offsets, topo: Topology, gamma: float, beta: float, k: int = 0,
                         norms=None, workspace=None, stream=None):
    """decentlam_step over the tensors [offsets[t], offsets[t+1]) of x, m, g (full-width tensors whose
    column 0 is column 0 of the table); `norms` (float64 device tensor, num_tensors x n x 3) receives
    the per-tensor, per-node sums of squares of g, the new m and the new x."""
    _step_multi(_lib.decentlam_step_multi, x, m, g, offsets, topo, gamma, beta, k, norms, workspace, stream)


def dmsgd_step_multi(x, m, g, offsets, topo: Topology, gamma: float, beta: float, k: int = 0,
                     norms=None, workspace=None, stream=None):
    """dmsgd_step over a table of tensors, see decentlam_step_multi."""
    _step_multi(_lib.dmsgd_step_multi, x, m, g, offsets, topo, gamma, beta, k, norms, workspace, stream)


def decentlam_step_xprev(x, x_prev, g, topo: Topology, gamma: float, beta: float, k: int = 0,
                         gamma_prev: float | None = None, stream=None):
    """Momentum-free DecentLaM: x_prev (x^{k-1}) is overwritten with x^{k+1}; x (x^k) is only read."""
    px, n, d, ld = _matrix_args(x, "x")
    pp, n2, d2, ld2 = _matrix_args(x_prev, "x_prev")
    pg, ng, dg, ldg = _matrix_args(g, "g")
    if (n2, d2, ld2) != (n, d, ld) or (ng, dg, ldg) != (n, d, ld):
        raise TypeError("x, x_prev and g must share shape and row stride")
    if topo.n != n:
        raise DecentLamError(DL_ETOPO, f"topology has {topo.n} nodes, arrays have {n} rows")
    _check(_lib.decentlam_step_xprev(px, pp, pg, n, d, ld, *topo._args(), gamma,
                                     gamma if gamma_prev is None else gamma_prev, beta, k,
                                     _stream() if stream is None else stream))


def dsgd_step(x, g, topo: Topology, gamma: float, k: int = 0, stream=None):
    """One DSGD iteration x <- W (x - gamma g) in place on the device tensor x, asynchronous."""
    px, n, d, ld = _matrix_args(x, "x")
    pg, ng, dg, ldg = _matrix_args(g, "g")
    if (ng, dg, ldg) != (n, d, ld):
        raise TypeError("x and g must share shape and row stride")
    if topo.n != n:
        raise DecentLamError(DL_ETOPO, f"topology has {topo.n} nodes, arrays have {n} rows")
    _check(_lib.dsgd_step(px, pg, n, d, ld, *topo._args(), gamma, k, _stream() if stream is None else stream))


def local_grad_lsq_workspace(n: int, b: int, d: int) -> int:
    return int(_lib.local_grad_lsq_workspace(n, b, d))


def local_grad_lsq(A, y, x, g, loss=None, scale: float = 1.0, workspace=None, stream=None, rows=None):
    """g_i = scale * A_i^T (A_i x_i - y_i) on device tensors; `workspace` is a uint8 device tensor
    of at least local_grad_lsq_workspace(n, b, d) bytes.  With `rows` (n x bs int32 device tensor)
    the sums run over the listed rows only (local_grad_lsq_rows)."""
    if A.dtype != torch.float32 or A.dim() != 3 or not A.is_cuda or A.stride(2) != 1:
        raise TypeError("A: need a 3-D float32 device tensor with contiguous last axis")
    n, b, d = A.shape
    if b > 1 and n > 1 and A.stride(0) != b * A.stride(1):
        raise TypeError("A: node stride must be b * row stride")
    ldA = A.stride(1) if b > 1 else max(A.stride(1), d)
    if y.dtype != torch.float32 or tuple(y.shape) != (n, b) or not y.is_contiguous() or not y.is_cuda:
        raise TypeError("y: need a contiguous n x b float32 device tensor")
    px, nx, dx, ld = _matrix_args(x, "x")
    pg, ng, dg, ldg = _matrix_args(g, "g")
    if (nx, dx) != (n, d) or (ng, dg, ldg) != (n, d, ld):
        raise TypeError("x and g must be n x d with the same row stride")
    pl = 0
    if loss is not None:
        if loss.dtype != torch.float32 or tuple(loss.shape) != (n,) or not loss.is_contiguous() or not loss.is_cuda:
            raise TypeError("loss: need a contiguous float32 device tensor of n elements")
        pl = loss.data_ptr()
    if workspace is None:
        raise TypeError("workspace: pass a uint8 device tensor (size from local_grad_lsq_workspace)")
    st = _stream() if stream is None else stream
    ws_bytes = workspace.numel() * workspace.element_size()
    if rows is None:
        _check(_lib.local_grad_lsq(A.data_ptr(), y.data_ptr(), px, pg, pl, n, b, d, ldA, ld, scale,
                                   workspace.data_ptr(), ws_bytes, st))
        return
    if rows.dtype != torch.int32 or rows.dim() != 2 or rows.shape[0] != n or not rows.is_cuda or not rows.is_contiguous():
        raise TypeError("rows: need a contiguous n x bs int32 device tensor")
    _check(_lib.local_grad_lsq_rows(A.data_ptr(), y.data_ptr(), px, pg, pl, n, b, d, ldA, ld, rows.data_ptr(),
                                    rows.shape[1], scale, workspace.data_ptr(), ws_bytes, st))


def local_grad_lsq_poll_limit(polls: int) -> int:
    return int(_lib.local_grad_lsq_poll_limit(int(polls)))


def local_grad_lsq_static(A, y, x, g, loss=None, scale: float = 1.0, stream=None):
    """local_grad_lsq without a workspace argument: the partial sums go to the library's own device array
    (DL_STATIC_SCRATCH_BYTES); no allocation anywhere.  Calls that overlap on one GPU race on that array."""
    if A.dtype != torch.float32 or A.dim() != 3 or not A.is_cuda or A.stride(2) != 1:
        raise TypeError("A: need a 3-D float32 device tensor with contiguous last axis")
    n, b, d = A.shape
    if b > 1 and n > 1 and A.stride(0) != b * A.stride(1):
        raise TypeError("A: node stride must be b * row stride")
    ldA = A.stride(1) if b > 1 else max(A.stride(1), d)
    if y.dtype != torch.float32 or tuple(y.shape) != (n, b) or not y.is_contiguous() or not y.is_cuda:
        raise TypeError("y: need a contiguous n x b float32 device tensor")
    px, nx, dx, ld = _matrix_args(x, "x")
    pg, ng, dg, ldg = _matrix_args(g, "g")
    if (nx, dx) != (n, d) or (ng, dg, ldg) != (n, d, ld):
        raise TypeError("x and g must be n x d with the same row stride")
    pl = 0
    if loss is not None:
        if loss.dtype != torch.float32 or tuple(loss.shape) != (n,) or not loss.is_contiguous() or not loss.is_cuda:
            raise TypeError("loss: need a contiguous float32 device tensor of n elements")
        pl = loss.data_ptr()
    _check(_lib.local_grad_lsq_static(A.data_ptr(), y.data_ptr(), px, pg, pl, n, b, d, ldA, ld, scale,
                                      _stream() if stream is None else stream))


def dl_calibration_stream(kind: int, split: bool, x, m, g, stream=None) -> int:
    """Bare stream with the step kernel's access pattern (kind 0: 3 reads + 2 writes, 1: reads, 2: writes);
    returns the number of columns it covered.  A benchmark aid, no part of the method."""
    px, n, d, ld = _matrix_args(x, "x")
    pm, nm, dm, ldm = _matrix_args(m, "m")
    pg, ng, dg, ldg = _matrix_args(g, "g")
    if (nm, dm, ldm) != (n, d, ld) or (ng, dg, ldg) != (n, d, ld):
        raise TypeError("x, m and g must share shape and row stride")
    cols = ctypes.c_int64(0)
    _check(_lib.dl_calibration_stream(kind, 1 if split else 0, px, pm, pg, n, d, ld, ctypes.byref(cols),
                                      _stream() if stream is None else stream))
    return cols.value


def decentlam_stats_workspace(n: int, d: int) -> int:
    return int(_lib.decentlam_stats_workspace(n, d))


def decentlam_stats(x, m=None, ref=None, out=None, workspace=None, stream=None):
    """Fill `out` (device float64[5]) with [consensus distance, ||xbar||^2, sum_i ||x_i - ref||^2,
    ||ref||^2, ||m||_F^2]; `workspace` is a uint8 device tensor of decentlam_stats_workspace(n, d) bytes."""
    px, n, d, ld = _matrix_args(x, "x")
    pm = 0
    if m is not None:
        pm, nm, dm, ldm = _matrix_args(m, "m")
        if (nm, dm, ldm) != (n, d, ld):
            raise TypeError("m must share x's shape and row stride")
    pr = 0
    if ref is not None:
        if ref.dtype != torch.float32 or tuple(ref.shape) != (d,) or not ref.is_cuda or not ref.is_contiguous():
            raise TypeError("ref: need a contiguous float32 device tensor of d elements")
        pr = ref.data_ptr()
    if out is None or out.dtype != torch.float64 or out.numel() < 5 or not out.is_cuda or not out.is_contiguous():
        raise TypeError("out: need a contiguous float64 device tensor of 5 elements")
    if workspace is None:
        raise TypeError("workspace: pass a uint8 device tensor (size from decentlam_stats_workspace)")
    _check(_lib.decentlam_stats(px, pm, pr, n, d, ld, out.data_ptr(), workspace.data_ptr(),
                                workspace.numel() * workspace.element_size(),
                                _stream() if stream is None else stream))
