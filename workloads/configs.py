"""The five synthetic workloads, as plain data.

Shapes stand in for the paper's deployments: 8-64 nodes (Sec. "Experiments",
implementation paragraph) and ResNet-50-sized flat parameter vectors
(about 25.5 M parameters, image-classification section).  The least-squares
workloads follow the appendix "Experimental setting for linear regression"
(per-node A_i, b_i = A_i x_i^o + 0.01 * noise) at larger sizes.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional

BASE_SEED = 2104_11981

# topology kinds; numeric values are the C-ABI's and the oracle's (an interface
# constant both sides must agree on, like an enum in a file format)
TOPO_RING = 0
TOPO_EXP_STATIC = 1
TOPO_EXP_ONEPEER = 2


@dataclass(frozen=True)
class Workload:
    cfg: int                 # 1..5, enters the seed
    name: str
    n: int                   # nodes
    d: int                   # parameters per node (0 => defined by the ragged layout)
    topo: int
    gamma: float
    beta: float
    steps: int
    x0_kind: str             # "normal": iid N(0,1) per node and element; "zero"
    grad_kind: str           # "normal" | "normal_shift" | "ragged_sigma" | "lsq"
    b: Optional[int] = None  # rows of A_i (least-squares workloads)
    a_scale: float = 1.0     # A_i = a_scale * N(0,1)
    lsq_scale: float = 1.0   # factor in g = lsq_scale * A^T (A x - y)
    n_tensors: int = 0       # ragged layout (workload 4)
    ragged_total: int = 0


WORKLOADS = {
    "c1_ring4": Workload(1, "c1_ring4", n=4, d=4096, topo=TOPO_RING, gamma=0.1, beta=0.9,
                         steps=10, x0_kind="normal", grad_kind="normal"),
    "c2_onepeer8_b32": Workload(2, "c2_onepeer8_b32", n=8, d=1024, topo=TOPO_EXP_ONEPEER,
                                gamma=0.01, beta=0.9, steps=200, x0_kind="zero",
                                grad_kind="lsq", b=32, lsq_scale=1.0 / 32),
    "c2_onepeer8_b1024": Workload(2, "c2_onepeer8_b1024", n=8, d=1024, topo=TOPO_EXP_ONEPEER,
                                  gamma=0.01, beta=0.9, steps=200, x0_kind="zero",
                                  grad_kind="lsq", b=1024, lsq_scale=1.0 / 1024),
    "c3_exp32": Workload(3, "c3_exp32", n=32, d=25_600_000, topo=TOPO_EXP_STATIC, gamma=0.1,
                         beta=0.9, steps=20, x0_kind="normal", grad_kind="normal_shift"),
    "c4_ring16_ragged": Workload(4, "c4_ring16_ragged", n=16, d=0, topo=TOPO_RING, gamma=0.05,
                                 beta=0.9, steps=20, x0_kind="normal", grad_kind="ragged_sigma",
                                 n_tensors=160, ragged_total=25_000_000),
    "c5_onepeer64_lsq": Workload(5, "c5_onepeer64_lsq", n=64, d=4096, topo=TOPO_EXP_ONEPEER,
                                 gamma=0.05, beta=0.9, steps=50, x0_kind="zero", grad_kind="lsq",
                                 b=4096, a_scale=1.0 / 64.0, lsq_scale=1.0),
}


def get(name: str) -> Workload:
    return WORKLOADS[name]


def scaled(w: Workload, **kw) -> Workload:
    """Same recipe at another size (the seed streams stay those of the parent)."""
    return replace(w, **kw)
