"""Helpers for the GPU parity tests: run the C-ABI library on seeded inputs and
compare with the CPU oracle.  Torch is used for device memory only."""
from __future__ import annotations

import numpy as np
import torch

import workloads as wl
from oracle import attn_ref as orc

# tolerances fixed by the target statement: bf16 and fp8 inputs
TOL = {
    "bf16": dict(max_abs=2e-2, rel_fro=5e-3, lse=1e-3),
    "fp8_e4m3": dict(max_abs=6e-2, rel_fro=2e-2, lse=1e-3),
}


def to_device(inp):
    """numpy bit patterns -> device tensors the library reads."""
    dev = {}
    for nm in "qkv":
        a = inp[nm]
        if a.dtype == np.uint16:
            dev[nm] = torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
        else:
            dev[nm] = torch.from_numpy(a).cuda()
    return dev


def decode(inp):
    """numpy bit patterns -> the float64 values they stand for (oracle input)."""
    out = {}
    for i, nm in enumerate("qkv"):
        a = inp[nm]
        if a.dtype == np.uint16:
            out[nm] = orc.bf16_bits_to_f64(a)
        else:
            out[nm] = orc.e4m3_bits_to_f64(a) * float(inp["descale"][i])
    return out


def run_gpu(inp, dev=None, variant=None):
    """One call through the C ABI.  Returns (O bf16 tensor on device, lse fp32 tensor)."""
    import paper_2605_10905_amd as A

    dev = dev or to_device(inp)
    B, Hq, Hkv, N, d = inp["B"], inp["Hq"], inp["Hkv"], inp["N"], inp["d"]
    o = torch.full((B, Hq, N, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((B, Hq, N), float("nan"), dtype=torch.float32, device="cuda")
    if inp["dtype"] == "bf16":
        if variant is None:
            A.attn_fwd(dev["q"], dev["k"], dev["v"], o, lse, B, Hq, Hkv, N, d, inp["causal"], inp["scale"], A.ATTN_BF16)
        else:
            A.attn_fwd_variant(dev["q"], dev["k"], dev["v"], o, lse, B, Hq, Hkv, N, d, inp["causal"], inp["scale"],
                               A.ATTN_BF16, variant)
    else:
        ds = inp["descale"]
        A.attn_fwd_fp8(dev["q"], dev["k"], dev["v"], o, lse, B, Hq, Hkv, N, d, inp["causal"], inp["scale"],
                       ds[0], ds[1], ds[2])
    torch.cuda.synchronize()
    return o, lse


def o_to_f64(o):
    return o.float().cpu().numpy().astype(np.float64)


def check_full(inp, o, lse, label=""):
    """Element-by-element comparison of the whole tensor with the oracle."""
    x = decode(inp)
    o_ref, lse_ref = orc.attn_ref(x["q"], x["k"], x["v"], inp["causal"], inp["scale"])
    og = o_to_f64(o)
    lg = lse.cpu().numpy().astype(np.float64)
    assert np.isfinite(og).all(), f"{label}: non-finite O"
    assert np.isfinite(lg).all(), f"{label}: non-finite lse"
    m = orc.error_metrics(og, o_ref, lg, lse_ref)
    tol = TOL[inp["dtype"]]
    assert m["max_abs"] <= tol["max_abs"], f"{label}: {m}"
    assert m["rel_fro"] <= tol["rel_fro"], f"{label}: {m}"
    assert m["lse_max_abs"] <= tol["lse"], f"{label}: {m}"
    return m


def sample_rows(N, BM, rng, n_random=24):
    """Rows at tile edges plus random ones."""
    rows = {0, 1, N - 1, N // 2}
    for t in (1, 2, N // BM - 1):
        for r in (t * BM - 1, t * BM, t * BM + 31, t * BM + 32):
            if 0 <= r < N:
                rows.add(r)
    rows.update(int(r) for r in rng.integers(0, N, n_random))
    return np.array(sorted(rows))


def check_sampled(inp, o, lse, heads, rows_per_head, label=""):
    """Full-size check: the oracle evaluates sampled (b, h, row) outputs one by one."""
    x = decode(inp)
    tol = TOL[inp["dtype"]]
    num = den = 0.0
    worst = dict(max_abs=0.0, lse_max_abs=0.0)
    for (b, h), rows in zip(heads, rows_per_head):
        o_ref, lse_ref = orc.attn_ref_rows(x["q"], x["k"], x["v"], inp["causal"], inp["scale"], b, h, rows)
        idx = torch.from_numpy(rows).cuda()
        og = o_to_f64(o[b, h].index_select(0, idx))
        lg = lse[b, h].index_select(0, idx).cpu().numpy().astype(np.float64)
        assert np.isfinite(og).all() and np.isfinite(lg).all(), f"{label}: non-finite output at b={b} h={h}"
        worst["max_abs"] = max(worst["max_abs"], float(np.abs(og - o_ref).max()))
        worst["lse_max_abs"] = max(worst["lse_max_abs"], float(np.abs(lg - lse_ref).max()))
        num += float(((og - o_ref) ** 2).sum())
        den += float((o_ref ** 2).sum())
    worst["rel_fro"] = (num / den) ** 0.5
    assert worst["max_abs"] <= tol["max_abs"], f"{label}: {worst}"
    assert worst["rel_fro"] <= tol["rel_fro"], f"{label}: {worst}"
    assert worst["lse_max_abs"] <= tol["lse"], f"{label}: {worst}"
    return worst


def check_whole_head(inp, o, lse, b, h, label=""):
    """Full-size check of ONE whole (b, h) slice: every row of that head against the oracle."""
    x = decode(inp)
    g = h // (inp["Hq"] // inp["Hkv"])
    o_ref, lse_ref = orc.attn_head(x["q"][b, h], x["k"][b, g], x["v"][b, g], inp["causal"], inp["scale"])
    m = orc.error_metrics(o_to_f64(o[b, h]), o_ref, lse[b, h].cpu().numpy().astype(np.float64), lse_ref)
    tol = TOL[inp["dtype"]]
    assert m["max_abs"] <= tol["max_abs"], f"{label}: {m}"
    assert m["rel_fro"] <= tol["rel_fro"], f"{label}: {m}"
    assert m["lse_max_abs"] <= tol["lse"], f"{label}: {m}"
    return m
