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


to_device = wl.to_device  # numpy bit patterns -> device tensors the library reads


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


# ---- backward --------------------------------------------------------------------------------
# The target statement gives tolerances for the forward outputs only; the gradient bounds are
# derived from the kernels' arithmetic.  Every rounding on the path is bf16 round-to-nearest with
# relative RMS error 2^-9 / sqrt(3) = 1.1e-3: P (or dS) as a matrix operand, the stored forward O
# inside delta = rowsum(dO * O), and the written gradient.  They add incoherently to about 2.3e-3
# relative Frobenius error, which is what every well-conditioned case measures (2.3e-3 .. 2.5e-3
# on the reduced and full-size configs).  Bounds: relative Frobenius error 5e-3 per tensor, and
# every element within 2e-2 * max(1, max|reference|) (the gradients' scale varies with the mask
# and the length, so the element-wise bound scales with the tensor's largest entry).
# Where one key dominates a softmax row (rows of fewer than 64 keys, or inputs built that way),
# dS = P * (dP - delta) cancels by the factor 1 - max(P): the 2^-9 rounding of the stored O that
# enters delta is amplified by its inverse.  With max(P) = 0.9 the 2.3e-3 becomes about 6e-3
# (measured: at most 5.8e-3 on the adversarial rows and the lengths below 64).  For those cases,
# and only those, the Frobenius bound is 1e-2; the element-wise bound is the same everywhere.
TOL_BWD = dict(rel_fro=5e-3, rel_fro_short=1e-2, short_n=64, max_abs_rel=2e-2)


def bf16_to_device(bits):
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()


def run_gpu_bwd(inp, dout_bits, dev=None, poison=float("nan")):
    """Forward then backward through the C ABI.  Returns (dq, dk, dv, o, lse) on the device."""
    import paper_2605_10905_amd as A

    dev = dev or to_device(inp)
    B, Hq, Hkv, N, d = inp["B"], inp["Hq"], inp["Hkv"], inp["N"], inp["d"]
    o, lse = run_gpu(inp, dev)
    do = bf16_to_device(dout_bits)
    dq = torch.full((B, Hq, N, d), poison, dtype=torch.bfloat16, device="cuda")
    dk = torch.full((B, Hkv, N, d), poison, dtype=torch.bfloat16, device="cuda")
    dv = torch.full((B, Hkv, N, d), poison, dtype=torch.bfloat16, device="cuda")
    ws = torch.full((A.attn_bwd_workspace_bytes(B, Hq, N) // 4,), poison, dtype=torch.float32, device="cuda")
    A.attn_bwd(dev["q"], dev["k"], dev["v"], o, do, lse, dq, dk, dv, ws, B, Hq, Hkv, N, d, inp["causal"], inp["scale"],
               A.ATTN_BF16)
    torch.cuda.synchronize()
    return dq, dk, dv, o, lse


def check_grads(got, ref, label="", peaked=False):
    """got, ref: dicts name -> array; every tensor against TOL_BWD (`peaked`: the few-key
    Frobenius bound, for inputs built so that single keys dominate their rows)."""
    from oracle import attn_bwd_ref as ob

    out = {}
    for nm in ref:
        g = got[nm].float().cpu().numpy().astype(np.float64) if torch.is_tensor(got[nm]) else got[nm]
        assert np.isfinite(g).all(), f"{label}: non-finite {nm}"
        m = ob.grad_error_metrics(g, ref[nm])
        bound = TOL_BWD["max_abs_rel"] * max(1.0, float(np.abs(ref[nm]).max()))
        assert m["max_abs"] <= bound, f"{label}: {nm} {m} bound {bound}"
        n_keys = ref[nm].shape[-2]
        fro = TOL_BWD["rel_fro_short"] if (peaked or n_keys < TOL_BWD["short_n"]) else TOL_BWD["rel_fro"]
        assert m["rel_fro"] <= fro, f"{label}: {nm} {m}"
        out[nm] = m
    return out


def check_bwd_full(inp, dout_bits, dq, dk, dv, label="", peaked=False):
    from oracle import attn_bwd_ref as ob

    x = decode(inp)
    rq, rk, rv = ob.attn_bwd_ref(x["q"], x["k"], x["v"], orc.bf16_bits_to_f64(dout_bits), inp["causal"], inp["scale"])
    return check_grads(dict(dq=dq, dk=dk, dv=dv), dict(dq=rq, dk=rk, dv=rv), label, peaked)


def check_bwd_group(inp, dout_bits, dq, dk, dv, b, g, label=""):
    """Full-size check of one whole (batch, kv head) group: dK, dV of that kv head and dQ of
    every query head that reads it."""
    from oracle import attn_bwd_ref as ob

    G = inp["Hq"] // inp["Hkv"]
    hs = slice(g * G, (g + 1) * G)
    x = decode(inp)
    rq, rk, rv = ob.attn_bwd_ref(x["q"][b:b + 1, hs], x["k"][b:b + 1, g:g + 1], x["v"][b:b + 1, g:g + 1],
                                 orc.bf16_bits_to_f64(dout_bits[b:b + 1, hs]), inp["causal"], inp["scale"])
    return check_grads(dict(dq=dq[b:b + 1, hs], dk=dk[b:b + 1, g:g + 1], dv=dv[b:b + 1, g:g + 1]),
                       dict(dq=rq, dk=rk, dv=rv), label)
