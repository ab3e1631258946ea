"""MI355X-native fused attention forward (hand-written HIP behind a C ABI).

The Python layer only marshals arguments: every step of the path runs in the
HIP kernels of libattn_mi355x.so.  There is no CPU or PyTorch fallback; if the
library is missing, importing `paper_2605_10905_amd.binding` raises.
"""
from .binding import (  # noqa: F401
    ATTN_BF16,
    ATTN_FP8_E4M3,
    AttnError,
    attn_fwd,
    attn_fwd_fp8,
    attn_fwd_variant,
    attn_num_variants,
    attn_num_workgroups,
    attn_status_string,
    attn_tile_coord,
    attn_variant_bm,
    attn_variant_name,
    attn_version,
    lib,
    lib_path,
)
