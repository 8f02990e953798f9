"""Counter-based input generation (numpy Philox on the host, torch's seeded
generator on the device for the sizes that are only ever built in HBM).

Nothing here is part of the method: these are the random draws the method
*receives* (initial replicas, stochastic gradients, regression data).
"""
from __future__ import annotations

import math

import numpy as np

from .configs import BASE_SEED, Workload

ROLE_X0 = 1
ROLE_GRAD = 2
ROLE_SHIFT = 3
ROLE_A = 4
ROLE_XSTAR_SHARED = 5
ROLE_XSTAR_NODE = 6
ROLE_NOISE = 7
ROLE_LAYOUT = 8
ROLE_SIGMA = 9


def _stream_key(cfg: int, role: int, k: int, i: int) -> int:
    assert 0 <= cfg < 2**8 and 0 <= role < 2**8 and 0 <= k < 2**24 and 0 <= i < 2**24
    return (cfg << 56) | (role << 48) | (k << 24) | i


def _rng(cfg: int, role: int, k: int = 0, i: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[BASE_SEED, _stream_key(cfg, role, k, i)]))


def normal_rows(cfg: int, role: int, k: int, n: int, d: int) -> np.ndarray:
    """n x d fp32, row i drawn from stream (cfg, role, k, i)."""
    out = np.empty((n, d), dtype=np.float32)
    for i in range(n):
        out[i] = _rng(cfg, role, k, i).standard_normal(d, dtype=np.float32)
    return out


def uniform_scalars(cfg: int, role: int, count: int, lo: float, hi: float) -> np.ndarray:
    return _rng(cfg, role).uniform(lo, hi, size=count)


def ragged_layout(w: Workload):
    """Tensor sizes and offsets of the ragged parameter layout.

    Sizes are log-uniform in [64, 2.4e6], rescaled by one common factor towards
    `ragged_total`, clamped back into the range and NOT rounded to multiples of
    4; tensors are packed back to back.  Returns (sizes int64[T], offsets
    int64[T+1], sigma float64[T]) with offsets[-1] == d.
    """
    assert w.n_tensors > 0
    lo, hi = 64.0, 2.4e6
    raw = np.exp(_rng(w.cfg, ROLE_LAYOUT).uniform(math.log(lo), math.log(hi), size=w.n_tensors))
    sizes = np.clip(raw * (w.ragged_total / raw.sum()), lo, hi)
    sizes = np.maximum(np.rint(sizes).astype(np.int64), 1)
    offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    sigma = _rng(w.cfg, ROLE_SIGMA).uniform(0.01, 1.0, size=w.n_tensors)
    return sizes, offsets, sigma


def dim(w: Workload) -> int:
    if w.d:
        return w.d
    return int(ragged_layout(w)[1][-1])


def x0(w: Workload) -> np.ndarray:
    d = dim(w)
    if w.x0_kind == "zero":
        return np.zeros((w.n, d), dtype=np.float32)
    return normal_rows(w.cfg, ROLE_X0, 0, w.n, d)


def node_shift(w: Workload) -> np.ndarray:
    """c_i ~ U(-1, 1), fixed per node (heterogeneity of workload 3)."""
    return uniform_scalars(w.cfg, ROLE_SHIFT, w.n, -1.0, 1.0).astype(np.float32)


def grad(w: Workload, k: int) -> np.ndarray:
    """Stochastic gradient handed to step k (n x d fp32) for the non-LSQ workloads."""
    d = dim(w)
    g = normal_rows(w.cfg, ROLE_GRAD, k, w.n, d)
    if w.grad_kind == "normal":
        return g
    if w.grad_kind == "normal_shift":
        return (g + node_shift(w)[:, None]).astype(np.float32)
    if w.grad_kind == "ragged_sigma":
        _, off, sigma = ragged_layout(w)
        scale = np.repeat(sigma.astype(np.float32), np.diff(off))
        return (g * scale[None, :]).astype(np.float32)
    raise ValueError(f"workload {w.name} takes its gradient from the least-squares data")


def lsq_problem(w: Workload):
    """(A [n,b,d] fp32, y [n,b] fp32, xstar [n,d] fp32): y_i = A_i xstar_i + 0.01 N(0,1),
    xstar_i = shared N(0,1) vector + 0.5 N(0,1) per node."""
    assert w.grad_kind == "lsq" and w.b
    n, b, d = w.n, w.b, w.d
    A = np.empty((n, b, d), dtype=np.float32)
    for i in range(n):
        A[i] = _rng(w.cfg, ROLE_A, 0, i).standard_normal((b, d), dtype=np.float32)
        if w.a_scale != 1.0:
            A[i] *= np.float32(w.a_scale)
    shared = _rng(w.cfg, ROLE_XSTAR_SHARED).standard_normal(d)
    xstar = np.empty((n, d), dtype=np.float32)
    y = np.empty((n, b), dtype=np.float32)
    for i in range(n):
        xs = (shared + 0.5 * _rng(w.cfg, ROLE_XSTAR_NODE, 0, i).standard_normal(d)).astype(np.float32)
        xstar[i] = xs
        noise = 0.01 * _rng(w.cfg, ROLE_NOISE, 0, i).standard_normal(b)
        y[i] = (A[i].astype(np.float64) @ xs.astype(np.float64) + noise).astype(np.float32)
    return A, y, xstar


# --------------------------------------------------------------------------
# Device-side generation for the sizes that are only ever built in HBM
# (workloads 3, 4, 5 at full size).  torch's seeded device generator is the
# random source; the host reads back whatever slices it needs.
# --------------------------------------------------------------------------

def _torch_gen(device, cfg: int, role: int, k: int = 0):
    import torch

    g = torch.Generator(device=device)
    g.manual_seed((BASE_SEED * 1_000_003 + _stream_key(cfg, role, k, 0)) % (2**63 - 1))
    return g


def device_x0(w: Workload, device, ld: int | None = None):
    import torch

    d = dim(w)
    ld = ld or d
    x = torch.zeros((w.n, ld), dtype=torch.float32, device=device)
    if w.x0_kind == "normal":
        x[:, :d].normal_(generator=_torch_gen(device, w.cfg, ROLE_X0))
    return x


def device_grad(w: Workload, k: int, out):
    """Fill `out` (n x ld fp32 device tensor) with the step-k gradient, in place."""
    import torch

    d = dim(w)
    view = out[:, :d]
    view.normal_(generator=_torch_gen(out.device, w.cfg, ROLE_GRAD, k))
    if w.grad_kind == "normal_shift":
        view.add_(torch.from_numpy(node_shift(w)).to(out.device)[:, None])
    elif w.grad_kind == "ragged_sigma":
        _, off, sigma = ragged_layout(w)
        scale = torch.repeat_interleave(
            torch.from_numpy(sigma.astype(np.float32)).to(out.device),
            torch.from_numpy(np.diff(off)).to(out.device))
        view.mul_(scale[None, :])
    elif w.grad_kind != "normal":
        raise ValueError(w.grad_kind)
    return out


def device_lsq_problem(w: Workload, device):
    """Device version of `lsq_problem` (different random stream, same recipe)."""
    import torch

    n, b, d = w.n, w.b, w.d
    A = torch.empty((n, b, d), dtype=torch.float32, device=device)
    A.normal_(generator=_torch_gen(device, w.cfg, ROLE_A))
    if w.a_scale != 1.0:
        A.mul_(w.a_scale)
    shared = torch.empty(d, dtype=torch.float32, device=device)
    shared.normal_(generator=_torch_gen(device, w.cfg, ROLE_XSTAR_SHARED))
    xstar = torch.empty((n, d), dtype=torch.float32, device=device)
    xstar.normal_(generator=_torch_gen(device, w.cfg, ROLE_XSTAR_NODE))
    xstar.mul_(0.5).add_(shared[None, :])
    noise = torch.empty((n, b), dtype=torch.float32, device=device)
    noise.normal_(generator=_torch_gen(device, w.cfg, ROLE_NOISE))
    y = torch.bmm(A, xstar[:, :, None])[:, :, 0] + 0.01 * noise
    return A, y.contiguous(), xstar
