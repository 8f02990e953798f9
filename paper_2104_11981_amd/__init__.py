"""MI355X-native decentralized momentum updates (DecentLaM / DmSGD), arXiv 2104.11981.

The product is `libdecentlam.so` (hand-written HIP kernels for gfx950 behind a C
ABI, see include/decentlam.h); this package is its thin ctypes binding.  Importing
it requires the built library -- there is no CPU or PyTorch fallback.
"""
from .binding import (  # noqa: F401
    DL_EALIAS, DL_ECAP, DL_EHIP, DL_EINVAL, DL_ETOPO, DL_OK,
    DL_FLAG_COL_STOCHASTIC, DL_FLAG_ROW_STOCHASTIC, DL_FLAG_SYMMETRIC,
    DL_MAX_NNZ, DL_MAX_NNZ_PALETTE, DL_MAX_NODES, DL_MAX_WEIGHT_VALUES,
    DL_TOPO_BIPARTITE_MATCH, DL_TOPO_EXP_ONEPEER, DL_TOPO_EXP_STATIC, DL_TOPO_EXP_SYM, DL_TOPO_MESH, DL_TOPO_RING,
    EXPORTS, LIB_PATH, DecentLamError, Topology,
    decentlam_stats, decentlam_stats_workspace, decentlam_step, decentlam_step_xprev, dmsgd_step, dsgd_step, last_error, local_grad_lsq, local_grad_lsq_workspace,
    make_topology, topology_build, topology_metropolis,
)
from .binding import _lib as raw  # noqa: F401  (the ctypes handle, for tests of the C ABI itself)
