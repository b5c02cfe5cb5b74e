"""MI355X-native packed varlen causal attention (forward + backward) for HBP packs.

Thin ctypes binding over ``libhbp.so`` (C ABI declared in ``include/hbp.h``).  Every step of the
hot path runs in the library's HIP kernels; Python only marshals pointers and sizes.
"""
from .binding import (HbpError, AttnDesc, load_library, library_path, hbp_status_string,
                      hbp_pack_plan, hbp_tile_rows, hbp_fwd_tile_rows, hbp_workspace_bytes, hbp_profile_capacity,
                      hbp_varlen_attn_fwd, hbp_varlen_attn_bwd, hbp_varlen_attn_bwd_static, HBP_STATIC_SCRATCH_BYTES, HBP_ERR_STATIC_LIMIT, hbp_set_kernel_events, hbp_mfma_probe, hbp_balance_packing, hbp_auto_select, hbp_packed_ce, hbp_packed_ce_workspace_bytes,
                      HBP_LOSS, HBP_LOSS_TOKEN_MEAN, HBP_LOSS_SAMPLE_MEAN, HBP_LOSS_STABLE, HBP_FWD, HBP_BWD, HBP_BWD_DQ,
                      HBP_TILES_QUERY, HBP_TILES_KEY, PROFILE_DTYPE, EXPORTED_SYMBOLS)

__all__ = ["HbpError", "AttnDesc", "load_library", "library_path", "hbp_status_string",
           "hbp_pack_plan", "hbp_tile_rows", "hbp_fwd_tile_rows", "hbp_workspace_bytes", "hbp_profile_capacity",
           "hbp_varlen_attn_fwd", "hbp_varlen_attn_bwd", "hbp_varlen_attn_bwd_static", "HBP_STATIC_SCRATCH_BYTES", "HBP_ERR_STATIC_LIMIT", "hbp_set_kernel_events", "hbp_mfma_probe", "hbp_balance_packing", "hbp_auto_select", "hbp_packed_ce", "hbp_packed_ce_workspace_bytes",
           "HBP_LOSS", "HBP_LOSS_TOKEN_MEAN", "HBP_LOSS_SAMPLE_MEAN", "HBP_LOSS_STABLE", "HBP_FWD", "HBP_BWD", "HBP_BWD_DQ",
           "HBP_TILES_QUERY", "HBP_TILES_KEY", "PROFILE_DTYPE", "EXPORTED_SYMBOLS"]
