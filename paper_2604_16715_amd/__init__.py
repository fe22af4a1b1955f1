"""gta — sparse graph attention (forward + backward) for one MI355X.

Thin ctypes binding over ``libgta.so`` (C ABI declared in ``include/gta.h``); every step of the
path runs in the library's HIP kernels.  PyTorch is used for device memory and streams only.
"""
from .binding import (  # noqa: F401
    GtaError, Plan, gta_attn_bwd, gta_attn_fwd, gta_attn_fwd_noalloc, gta_attn_bwd_halo, gta_attn_fwd_halo, gta_attn_merge, gta_attn_scratch_bytes, gta_plan_create,
    gta_profile_enable, gta_profile_read, gta_stream_probe, gta_version, lib_path, load_library,
    gta_sddmm, gta_edge_softmax, gta_edge_softmax_bwd, gta_spmm, gta_agp_select, gta_head_split, gta_head_merge, gta_linear, gta_linear_dw, gta_linear_dw_group, gta_linear_group, gta_sga_layer_fwd, gta_sga_layer_bwd,
)
