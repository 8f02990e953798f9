"""Seeded synthetic inputs for the decentralized-update workloads.

This package only produces *inputs*: initial replicas, per-step gradients,
least-squares data and the ragged tensor layout.  It contains none of the
method's arithmetic (no mixing, no momentum, no gradient formula), so both the
CPU oracle's tests and the GPU path's tests may draw from it without sharing
any of the code under test.

Every array is a pure function of (BASE_SEED, config id, role, step k, node i):
each (role, k, i) triple owns one Philox stream, so the value of element
(k, i, c) does not depend on the order in which rows are generated.
"""
from .configs import (  # noqa: F401
    BASE_SEED,
    Workload,
    WORKLOADS,
    get,
    scaled,
)
from .generate import (  # noqa: F401
    normal_rows,
    uniform_scalars,
    x0,
    grad,
    lsq_problem,
    ragged_layout,
    device_x0,
    device_grad,
    device_lsq_problem,
)
