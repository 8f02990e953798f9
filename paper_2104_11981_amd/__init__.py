"""MI355X-native decentralized momentum updates (DecentLaM / DmSGD), arXiv 2104.11981.

The product is `libdecentlam.so` (hand-written HIP kernels for gfx950 behind a C ABI, see
include/decentlam.h); this package is its thin ctypes binding.  There is no CPU or PyTorch
fallback: the first use of any name below loads the shared library and raises ImportError if it
has not been built (`python -m paper_2104_11981_amd.build`).  The binding is loaded on first use
rather than on import so that `paper_2104_11981_amd.build` itself can be imported in a fresh tree.
"""
_BINDING_NAMES = (
    "DL_EALIAS", "DL_ECAP", "DL_EHIP", "DL_EINVAL", "DL_ETOPO", "DL_OK",
    "DL_FLAG_COL_STOCHASTIC", "DL_FLAG_ROW_STOCHASTIC", "DL_FLAG_SYMMETRIC",
    "DL_MAX_NNZ", "DL_MAX_NNZ_PALETTE", "DL_MAX_NODES", "DL_MAX_WEIGHT_VALUES",
    "DL_TOPO_BIPARTITE_MATCH", "DL_TOPO_EXP_ONEPEER", "DL_TOPO_EXP_STATIC", "DL_TOPO_EXP_SYM",
    "DL_TOPO_MESH", "DL_TOPO_RING", "DL_GRAD_F32", "DL_GRAD_BF16", "DL_GRAD_F16",
    "EXPORTS", "LIB_PATH", "DecentLamError", "Topology",
    "decentlam_stats", "decentlam_stats_workspace", "decentlam_step", "decentlam_step_xprev",
    "dmsgd_step", "dsgd_step", "awc_dmsgd_step", "da_dmsgd_step", "decentlam_step_blocked",
    "dmsgd_step_blocked", "to_blocked", "from_blocked", "recommended_ld", "empty_rows", "decentlam_step_ex", "dmsgd_step_ex",
    "decentlam_step_xprev_ex", "decentlam_step_multi_ex", "dmsgd_step_multi_ex", "Layout", "decentlam_step_g16", "dmsgd_step_g16", "decentlam_step_multi",
    "dmsgd_step_multi", "decentlam_step_multi_workspace", "last_error", "local_grad_lsq", "local_grad_lsq_workspace",
    "local_grad_lsq_static", "local_grad_lsq_poll_limit", "DL_STATIC_SCRATCH_BYTES", "dl_calibration_stream",
    "make_topology", "topology_build", "topology_metropolis", "topology_pack", "topology_pack_bytes", "PackedTopology",
    "decentlam_step_packed", "dmsgd_step_packed", "dsgd_step_packed", "PreparedCall", "prepare_step",
    "prepare_local_grad_lsq", "topology_device_bytes", "topology_pack_device", "DeviceTopology", "DeviceTopologyStruct",
    "decentlam_step_dev", "dmsgd_step_dev", "dsgd_step_dev", "DL_MAX_NODES_DEVICE",
    "awc_dmsgd_step_ex", "da_dmsgd_step_ex", "awc_dmsgd_step_multi_ex", "da_dmsgd_step_multi_ex",
)
__all__ = list(_BINDING_NAMES) + ["raw"]


def __getattr__(name):
    if name in _BINDING_NAMES or name == "raw":
        from . import binding   # raises ImportError if libdecentlam.so is missing

        value = binding._lib if name == "raw" else getattr(binding, name)   # raw: the ctypes handle
        globals()[name] = value
        return value
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")
