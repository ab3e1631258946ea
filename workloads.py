"""Seeded synthetic inputs for the attention forward path.

This module only draws random numbers and stores them in the formats the GPU
reads (bf16 bit patterns, fp8 e4m3 codes with one fp32 scale per tensor).  It
holds none of the method's arithmetic and is the one piece of code that both
the CPU oracle's tests and the HIP path's tests / bench use.

The paper measures attention on synthetic shapes (appendix A, attention-shape
table: batch 4, 48 heads, sequence 1024..16384, head dim 128); the configs
below are the five this build is graded on plus that grid.
"""
from __future__ import annotations

import math

import numpy as np

# (name, B, Hq, Hkv, N, d, dtype, sigma, causal)
CONFIGS = [
    dict(name="tiny_noncausal", B=1, Hq=2, Hkv=2, N=256, d=64, dtype="bf16", sigma=1.0, causal=False),
    dict(name="causal_2k", B=4, Hq=16, Hkv=16, N=2048, d=128, dtype="bf16", sigma=1.0, causal=True),
    dict(name="long_noncausal_8k", B=2, Hq=32, Hkv=32, N=8192, d=128, dtype="bf16", sigma=0.5, causal=False),
    dict(name="gqa_causal_4k", B=4, Hq=64, Hkv=8, N=4096, d=128, dtype="bf16", sigma=1.0, causal=True),
    dict(name="fp8_causal_16k", B=4, Hq=16, Hkv=16, N=16384, d=128, dtype="fp8_e4m3", sigma=1.0, causal=True),
]
for _i, _c in enumerate(CONFIGS):
    _c["index"] = _i
    _c["scale"] = 1.0 / math.sqrt(_c["d"])
    _c["seed"] = 1000 + _i


def paper_grid():
    """The paper's attention benchmark grid (forward rows of its shape table)."""
    out = []
    for causal in (True, False):
        for n in (1024, 2048, 4096, 8192, 16384):
            out.append(dict(name=f"paper_{'causal' if causal else 'noncausal'}_{n}", B=4, Hq=48, Hkv=48,
                            N=n, d=128, dtype="bf16", sigma=1.0, causal=causal,
                            scale=1.0 / math.sqrt(128), seed=2000 + n + int(causal)))
    return out


def extra_shapes():
    """Shapes beside the graded configs and the paper's grid: head dimension 64 and ragged lengths
    (not multiples of the 64-key tile or the 256-query tile) at the headline size."""
    out = []
    for name, n, d, causal in (("d64_noncausal_8192", 8192, 64, False), ("d64_causal_8192", 8192, 64, True),
                               ("ragged_noncausal_8191", 8191, 128, False), ("ragged_causal_8191", 8191, 128, True),
                               ("ragged_noncausal_8000", 8000, 128, False), ("ragged_noncausal_1000", 1000, 128, False)):
        out.append(dict(name=name, B=2, Hq=32, Hkv=32, N=n, d=d, dtype="bf16", sigma=1.0, causal=causal,
                        scale=1.0 / math.sqrt(d), seed=2500 + n + d + int(causal)))
    return out


def algorithmic_flops(cfg) -> float:
    """4*B*Hq*N^2*d, halved for causal (the figure usually quoted for attention)."""
    f = 4.0 * cfg["B"] * cfg["Hq"] * cfg["N"] * cfg["N"] * cfg["d"]
    return f / 2 if cfg["causal"] else f


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even.
    Inputs here are finite, so no NaN handling is needed."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def normal_f32(seed: int, stream: int, shape, sigma: float) -> np.ndarray:
    rng = np.random.default_rng([int(seed), int(stream)])
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        x *= np.float32(sigma)
    return x


def make_bf16(seed: int, stream: int, shape, sigma: float) -> np.ndarray:
    return f32_to_bf16_bits(normal_f32(seed, stream, shape, sigma))


def quantise_e4m3(x: np.ndarray):
    """Per-tensor fp8 quantisation as the fp8 config states it: one fp32 scale
    s = amax/448, codes = round-to-nearest-even e4m3 of x/s.  Returns (uint8
    codes, float32 scale).  The cast itself is torch's float8_e4m3fn."""
    import torch

    amax = float(np.max(np.abs(x)))
    s = np.float32(amax / 448.0) if amax > 0 else np.float32(1.0)
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)) / float(s)
    t = t.clamp_(-448.0, 448.0).to(torch.float8_e4m3fn)
    return t.view(torch.uint8).numpy().copy(), s


def make_inputs(cfg, B=None, Hq=None, Hkv=None, N=None):
    """Draw q, k, v for a config (optionally with some sizes overridden, for
    reduced-size parity cases).  Returns a dict with numpy arrays:
      bf16:  q,k,v uint16 bit patterns;  descale = (1,1,1)
      fp8 :  q,k,v uint8 e4m3 codes;     descale = per-tensor fp32 scales
    """
    B = cfg["B"] if B is None else B
    Hq = cfg["Hq"] if Hq is None else Hq
    Hkv = cfg["Hkv"] if Hkv is None else Hkv
    N = cfg["N"] if N is None else N
    d = cfg["d"]
    shapes = [(B, Hq, N, d), (B, Hkv, N, d), (B, Hkv, N, d)]
    out = dict(B=B, Hq=Hq, Hkv=Hkv, N=N, d=d, causal=cfg["causal"], scale=cfg["scale"], dtype=cfg["dtype"])
    names = ("q", "k", "v")
    if cfg["dtype"] == "bf16":
        for i, nm in enumerate(names):
            out[nm] = make_bf16(cfg["seed"], i, shapes[i], cfg["sigma"])
        out["descale"] = (1.0, 1.0, 1.0)
    elif cfg["dtype"] == "fp8_e4m3":
        ds = []
        for i, nm in enumerate(names):
            codes, s = quantise_e4m3(normal_f32(cfg["seed"], i, shapes[i], cfg["sigma"]))
            out[nm] = codes
            ds.append(float(s))
        out["descale"] = tuple(ds)
    else:
        raise ValueError(cfg["dtype"])
    return out


def to_device(inp):
    """The numpy bit patterns of make_inputs as device tensors the library reads (format
    plumbing only: bf16 bit patterns are viewed as torch.bfloat16, fp8 codes stay bytes)."""
    import torch

    dev = {}
    for nm in "qkv":
        a = inp[nm]
        if a.dtype == np.uint16:
            dev[nm] = torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
        else:
            dev[nm] = torch.from_numpy(a).cuda()
    return dev


def make_dout(cfg, B=None, Hq=None, N=None, sigma=1.0):
    """Output gradient for the backward pass: bf16 bit patterns [B,Hq,N,d], i.i.d. normal,
    drawn from a stream of its own of the config's seed."""
    B = cfg["B"] if B is None else B
    Hq = cfg["Hq"] if Hq is None else Hq
    N = cfg["N"] if N is None else N
    return make_bf16(cfg["seed"], 3, (B, Hq, N, cfg["d"]), sigma)


def algorithmic_flops_bwd(cfg) -> float:
    """Backward: five N x N x d products (S, dP, dV, dQ, dK) = 10*B*Hq*N^2*d, halved for causal."""
    return 2.5 * algorithmic_flops(cfg)


# ---- GEMM (paper appendix A: GEMM shape tables) -----------------------------------------------
# (name, M, N, K): the MI350 progression, the canonical 8192 x 8192 x K family, and the skewed
# production shapes of the B200 table whose operands fit comfortably on one GPU
GEMM_SHAPES = (
    [dict(name=f"mi350_{n}", M=n, N=n, K=n) for n in (256, 512, 1024, 2048)]
    + [dict(name=f"canonical_k{k}", M=8192, N=8192, K=k) for k in (1024, 2048, 4096, 8192, 16384)]
    + [dict(name="large_m_442368x448x192", M=442368, N=448, K=192),
       dict(name="large_m_589824x256x128", M=589824, N=256, K=128),
       dict(name="large_m_589824x512x2048", M=589824, N=512, K=2048),
       dict(name="large_n_1152x32768x9216", M=1152, N=32768, K=9216),
       dict(name="large_n_2048x64512x256", M=2048, N=64512, K=256),
       dict(name="large_k_512x4096x64512", M=512, N=4096, K=64512),
       dict(name="large_k_2304x1024x65536", M=2304, N=1024, K=65536)]
)
for _i, _g in enumerate(GEMM_SHAPES):
    _g["seed"] = 3000 + _i


def make_gemm_inputs(seed: int, M: int, N: int, K: int, sigma: float = 1.0):
    """A [M,K] and B [N,K] as bf16 bit patterns, i.i.d. normal."""
    return make_bf16(seed, 0, (M, K), sigma), make_bf16(seed, 1, (N, K), sigma)


def gemm_flops(M: int, N: int, K: int) -> float:
    return 2.0 * M * N * K
