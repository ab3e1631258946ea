"""ctypes binding of include/attn.h: same names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
lib_path = os.path.join(HERE, "libattn_mi355x.so")

ATTN_BF16 = 0
ATTN_FP8_E4M3 = 1


class AttnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({attn_status_string(status)})")


def _load():
    if not os.path.exists(lib_path):
        raise ImportError(
            f"{lib_path} is missing: build it first with `python -m paper_2605_10905_amd.build` "
            "(there is no fallback path)")
    return C.CDLL(lib_path)


lib = _load()

_vp, _i, _f = C.c_void_p, C.c_int, C.c_float
lib.attn_fwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _f, _i, _vp]
lib.attn_fwd.restype = _i
lib.attn_fwd_fp8.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _f, _f, _f, _f, _vp]
lib.attn_fwd_fp8.restype = _i
lib.attn_fwd_variant.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _f, _i, _i, _vp]
lib.attn_fwd_variant.restype = _i
lib.attn_fwd_persistent.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _f, _i, _vp, _vp]
lib.attn_fwd_persistent.restype = _i
lib.attn_persistent_queue_bytes.argtypes = []
lib.attn_persistent_queue_bytes.restype = _i
lib.attn_fwd_fp8_variant.argtypes = [_vp] * 5 + [_i] * 6 + [_f, _f, _f, _f, _i, _vp]
lib.attn_fwd_fp8_variant.restype = _i
lib.attn_bwd.argtypes = [_vp] * 10 + [_i, _i, _i, _i, _i, _i, _f, _i, _vp]
lib.attn_bwd.restype = _i
lib.attn_bwd_workspace_bytes.argtypes = [_i, _i, _i]
lib.attn_bwd_workspace_bytes.restype = C.c_longlong
lib.attn_bwd_noalloc.argtypes = [_vp] * 9 + [_i, _i, _i, _i, _i, _i, _f, _i, _vp]
lib.attn_bwd_noalloc.restype = _i
lib.attn_bwd_noalloc_max_workspace_bytes.argtypes = []
lib.attn_bwd_noalloc_max_workspace_bytes.restype = C.c_longlong
lib.gemm_bf16_nt.argtypes = [_vp, _vp, _vp, _i, _i, _i, _vp]
lib.gemm_bf16_nt.restype = _i
lib.gemm_bf16_nn.argtypes = [_vp, _vp, _vp, _i, _i, _i, _vp]
lib.gemm_bf16_nn.restype = _i
lib.gemm_bf16_nt_splitk.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _vp, _vp]
lib.gemm_bf16_nt_splitk.restype = _i
lib.gemm_splitk_workspace_bytes.argtypes = [_i, _i, _i]
lib.gemm_splitk_workspace_bytes.restype = C.c_longlong
lib.gemm_splitk_plan.argtypes = [_i, _i, _i]
lib.gemm_splitk_plan.restype = _i
lib.gemm_bf16_nt_variant.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _vp]
lib.gemm_bf16_nt_variant.restype = _i
lib.gemm_num_variants.argtypes = []
lib.gemm_num_variants.restype = _i
lib.gemm_variant_name.argtypes = [_i]
lib.gemm_variant_name.restype = C.c_char_p
lib.gemm_num_workgroups.argtypes = [_i, _i, _i]
lib.gemm_num_workgroups.restype = _i
lib.gemm_variant_kmult.argtypes = [_i]
lib.gemm_variant_kmult.restype = _i
lib.gemm_variant_tile.argtypes = [_i]
lib.gemm_variant_tile.restype = _i
lib.gemm_tile_coord.argtypes = [_i, _i, _i, _i, C.POINTER(_i), C.POINTER(_i)]
lib.gemm_tile_coord.restype = _i
lib.attn_default_variant.argtypes = [_i, _i, _i, _i, _i]
lib.attn_default_variant.restype = _i
lib.attn_num_variants.argtypes = []
lib.attn_num_variants.restype = _i
lib.attn_variant_name.argtypes = [_i]
lib.attn_variant_name.restype = C.c_char_p
lib.attn_variant_bm.argtypes = [_i]
lib.attn_variant_bm.restype = _i
lib.attn_num_workgroups.argtypes = [_i, _i, _i, _i]
lib.attn_num_workgroups.restype = _i
lib.attn_tile_coord.argtypes = [_i, _i, _i, _i, _i, _i, _i, C.POINTER(_i), C.POINTER(_i), C.POINTER(_i)]
lib.attn_tile_coord.restype = _i
lib.attn_status_string.argtypes = [_i]
lib.attn_status_string.restype = C.c_char_p
lib.attn_version.argtypes = []
lib.attn_version.restype = _i


def attn_status_string(status: int) -> str:
    return lib.attn_status_string(int(status)).decode()


def attn_version() -> int:
    return lib.attn_version()


def attn_num_variants() -> int:
    return lib.attn_num_variants()


def attn_variant_name(variant: int):
    s = lib.attn_variant_name(int(variant))
    return None if s is None else s.decode()


def attn_variant_bm(variant: int) -> int:
    return lib.attn_variant_bm(int(variant))


def attn_num_workgroups(B: int, Hq: int, N: int, BM: int) -> int:
    return lib.attn_num_workgroups(B, Hq, N, BM)


def attn_tile_coord(wg, B, Hq, Hkv, N, BM, causal):
    b, h, t = _i(), _i(), _i()
    st = lib.attn_tile_coord(wg, B, Hq, Hkv, N, BM, int(bool(causal)), C.byref(b), C.byref(h), C.byref(t))
    if st != 0:
        raise AttnError(st, "attn_tile_coord")
    return b.value, h.value, t.value


def _ptr(t):
    """Device pointer of a torch tensor (or a raw integer address / None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("attention tensors must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch

        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def attn_fwd(q, k, v, o, lse, B, Hq, Hkv, N, d, causal, scale, dtype, stream=None, check=True):
    st = lib.attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, Hq, Hkv, N, d, int(bool(causal)),
                      float(scale), int(dtype), _stream(stream))
    if check and st != 0:
        raise AttnError(st, "attn_fwd")
    return st


def attn_fwd_fp8(q, k, v, o, lse, B, Hq, Hkv, N, d, causal, scale, q_descale, k_descale, v_descale,
                 stream=None, check=True):
    st = lib.attn_fwd_fp8(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, Hq, Hkv, N, d, int(bool(causal)),
                          float(scale), float(q_descale), float(k_descale), float(v_descale), _stream(stream))
    if check and st != 0:
        raise AttnError(st, "attn_fwd_fp8")
    return st


def attn_fwd_variant(q, k, v, o, lse, B, Hq, Hkv, N, d, causal, scale, dtype, variant, stream=None, check=True):
    st = lib.attn_fwd_variant(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, Hq, Hkv, N, d, int(bool(causal)),
                              float(scale), int(dtype), int(variant), _stream(stream))
    if check and st != 0:
        raise AttnError(st, "attn_fwd_variant")
    return st


def attn_fwd_fp8_variant(q, k, v, o, lse, B, Hq, Hkv, N, d, causal, scale, q_descale, k_descale, v_descale, variant, stream=None,
                         check=True):
    st = lib.attn_fwd_fp8_variant(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, Hq, Hkv, N, d, int(bool(causal)),
                                  float(scale), float(q_descale), float(k_descale), float(v_descale), int(variant), _stream(stream))
    if check and st != 0:
        raise AttnError(st, "attn_fwd_fp8_variant")
    return st


def attn_bwd_workspace_bytes(B: int, Hq: int, N: int) -> int:
    return lib.attn_bwd_workspace_bytes(B, Hq, N)


def attn_bwd(q, k, v, o, dout, lse, dq, dk, dv, workspace, B, Hq, Hkv, N, d, causal, scale, dtype, stream=None,
             check=True):
    st = lib.attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(dout), _ptr(lse), _ptr(dq), _ptr(dk), _ptr(dv),
                      _ptr(workspace), B, Hq, Hkv, N, d, int(bool(causal)), float(scale), int(dtype), _stream(stream))
    if check and st != 0:
        raise AttnError(st, "attn_bwd")
    return st


def attn_bwd_noalloc_max_workspace_bytes() -> int:
    return lib.attn_bwd_noalloc_max_workspace_bytes()


def attn_bwd_noalloc(q, k, v, o, dout, lse, dq, dk, dv, B, Hq, Hkv, N, d, causal, scale, dtype, stream=None, check=True):
    st = lib.attn_bwd_noalloc(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(dout), _ptr(lse), _ptr(dq), _ptr(dk), _ptr(dv),
                              B, Hq, Hkv, N, d, int(bool(causal)), float(scale), int(dtype), _stream(stream))
    if check and st != 0:
        raise AttnError(st, "attn_bwd_noalloc")
    return st


def gemm_bf16_nt(a, b, c, M, N, K, stream=None, check=True):
    st = lib.gemm_bf16_nt(_ptr(a), _ptr(b), _ptr(c), M, N, K, _stream(stream))
    if check and st != 0:
        raise AttnError(st, "gemm_bf16_nt")
    return st


def gemm_bf16_nt_variant(a, b, c, M, N, K, variant, stream=None, check=True):
    st = lib.gemm_bf16_nt_variant(_ptr(a), _ptr(b), _ptr(c), M, N, K, int(variant), _stream(stream))
    if check and st != 0:
        raise AttnError(st, "gemm_bf16_nt_variant")
    return st


def gemm_num_variants() -> int:
    return lib.gemm_num_variants()


def gemm_variant_name(variant: int):
    s = lib.gemm_variant_name(int(variant))
    return None if s is None else s.decode()


def gemm_num_workgroups(M: int, N: int, tile: int) -> int:
    return lib.gemm_num_workgroups(M, N, tile)


def gemm_variant_tile(variant: int) -> int:
    return lib.gemm_variant_tile(int(variant))


def gemm_tile_coord(wg, M, N, tile):
    tm, tn = _i(), _i()
    st = lib.gemm_tile_coord(wg, M, N, tile, C.byref(tm), C.byref(tn))
    if st != 0:
        raise AttnError(st, "gemm_tile_coord")
    return tm.value, tn.value


def attn_persistent_queue_bytes() -> int:
    return lib.attn_persistent_queue_bytes()


def attn_fwd_persistent(q, k, v, o, lse, B, Hq, Hkv, N, d, causal, scale, dtype, queue, stream=None, check=True):
    st = lib.attn_fwd_persistent(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, Hq, Hkv, N, d, int(bool(causal)),
                                 float(scale), int(dtype), _ptr(queue), _stream(stream))
    if check and st != 0:
        raise AttnError(st, "attn_fwd_persistent")
    return st


def attn_default_variant(dtype: int, B: int, Hq: int, N: int, d: int) -> int:
    return lib.attn_default_variant(int(dtype), B, Hq, N, d)


def gemm_variant_kmult(variant: int) -> int:
    return lib.gemm_variant_kmult(int(variant))


def gemm_bf16_nn(a, b, c, M, N, K, stream=None, check=True):
    st = lib.gemm_bf16_nn(_ptr(a), _ptr(b), _ptr(c), M, N, K, _stream(stream))
    if check and st != 0:
        raise AttnError(st, "gemm_bf16_nn")
    return st


def gemm_bf16_nt_splitk(a, b, c, M, N, K, splits, workspace, stream=None, check=True):
    st = lib.gemm_bf16_nt_splitk(_ptr(a), _ptr(b), _ptr(c), M, N, K, int(splits), _ptr(workspace), _stream(stream))
    if check and st != 0:
        raise AttnError(st, "gemm_bf16_nt_splitk")
    return st


def gemm_splitk_workspace_bytes(M: int, N: int, splits: int) -> int:
    return lib.gemm_splitk_workspace_bytes(M, N, splits)


def gemm_splitk_plan(M: int, N: int, K: int) -> int:
    return lib.gemm_splitk_plan(M, N, K)


