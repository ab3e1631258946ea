"""MI355X-native fused attention (forward; backward for bf16) and bf16 GEMM: hand-written HIP behind a C ABI.

The Python layer only marshals arguments: every step of the path runs in the
HIP kernels of libattn_mi355x.so.  There is no CPU or PyTorch fallback; if the
library is missing, the first use of any binding name raises.

The binding is imported on first attribute access, so that
`python -m paper_2605_10905_amd.build` can rebuild a missing or broken library.
"""
import importlib

_NAMES = (
    "ATTN_BF16", "ATTN_FP8_E4M3", "AttnError", "attn_bwd", "attn_bwd_noalloc", "attn_bwd_noalloc_max_workspace_bytes", "attn_bwd_workspace_bytes", "attn_default_variant", "attn_fwd", "attn_fwd_fp8", "attn_fwd_fp8_variant", "attn_fwd_persistent", "attn_persistent_queue_bytes", "attn_fwd_variant", "attn_num_variants",
    "attn_num_workgroups", "attn_status_string", "attn_tile_coord", "attn_variant_bm", "attn_variant_name", "attn_version",
    "gemm_bf16_nn", "gemm_bf16_nt", "gemm_bf16_nt_splitk", "gemm_bf16_nt_variant", "gemm_splitk_plan", "gemm_splitk_workspace_bytes", "gemm_num_variants", "gemm_num_workgroups", "gemm_tile_coord", "gemm_variant_kmult", "gemm_variant_name", "gemm_variant_tile",
    "lib", "lib_path",
)


def __getattr__(name):
    if name in _NAMES:
        return getattr(importlib.import_module(".binding", __name__), name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")


def __dir__():
    return sorted(list(globals()) + list(_NAMES))
