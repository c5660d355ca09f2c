"""dg4: the sparse graph-attention layer of DeepGate4 on MI355X (gfx950).

Thin Python binding over the C ABI in include/dg4.h. Every step of the path
runs in the HIP library; this package only marshals pointers. PyTorch is used
for device memory and streams.
"""
from .binding import (DG4Error, Graph, LayerConfig, dg4_build_levels, dg4_build_levels_device,  # noqa: F401
                      dg4_build_partitioned, dg4_build_partitioned_device, dg4_layer_fwd,
                      dg4_layer_profile, dg4_layer_status, dg4_sweep_elapsed_ms,
                      dg4_layer_workspace_bytes, dg4_proj_workspace_bytes, dg4_qkv_proj,
                      dg4_qkv_proj_static, dg4_static_scratch_bytes,
                      dg4_ffn_fwd, dg4_ffn_workspace_bytes,
                      dg4_sparse_attn_fwd, dg4_struct_encode, lib, library_path)
