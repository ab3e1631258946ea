"""CPU oracle for the fused attention forward pass.  TEST INFRASTRUCTURE ONLY.

This module is the slow, obviously-correct statement of what the hot path
computes.  It is imported only by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  The product (the HIP library and its Python
binding) never imports it and shares no code, table or constant with it.

What is computed (paper section 6.1, "Major Operators": score computation,
masking, normalisation, output accumulation; appendix C.3 for the two outputs,
the normalised accumulator and the per-row statistic  m + log(l)):

    for every batch b and query head h, with kv head g = h // (Hq // Hkv):
        S      = scale * Q[b,h] @ K[b,g]^T            (N x N, float64)
        S[i,j] = -inf  for j > i                      (causal only)
        m_i    = max_j S[i,j]
        E[i,j] = exp(S[i,j] - m_i)
        l_i    = sum_j E[i,j]
        P      = E / l                                (N x N, rows sum to one)
        O[b,h] = P @ V[b,g]                           (N x d)
        lse_i  = m_i + ln(l_i)                        (natural log)

The streaming ("online") softmax used on the GPU is an exact algebraic
rearrangement of the above, so the oracle is the plain definition: the full S
and P are materialised, nothing is tiled, fused or reordered.  All arithmetic
is float64.  Inputs are the exact values of the bf16 / fp8 bit patterns the GPU
reads (decoders below, written from the formats' definitions).

Readings taken where the paper is silent (all listed in the design notes):
natural log for the statistic; scale applied to the product, not to Q before
rounding; contiguous GQA groups (h // G); causal means key j visible to query
i iff j <= i with equal query and key lengths; for fp8 the oracle consumes the
de-quantised inputs and keeps P in float64.

Every function here is pinned by tests/test_oracle_pins.py against closed forms,
brute-force loops, invariances and library routines; nothing is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------
# exact decoders of the storage formats (bit pattern -> float64)
# --------------------------------------------------------------------------
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float64, exactly.

    bfloat16 is the upper half of an IEEE-754 binary32: 1 sign, 8 exponent,
    7 mantissa bits.  Widening the pattern with 16 zero bits gives the same
    real number as a binary32.
    """
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    with np.errstate(invalid="ignore"):  # signalling-NaN patterns widen to NaN, silently
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def e4m3_bits_to_f64(codes: np.ndarray) -> np.ndarray:
    """OCP 8-bit float E4M3 ("e4m3fn") codes (uint8) -> float64, exactly.

    Layout: 1 sign, 4 exponent (bias 7), 3 mantissa bits.  Exponent field 0 is
    subnormal: value = mant/8 * 2^-6.  Otherwise value = (1 + mant/8) *
    2^(exp-7).  There is no infinity; the single NaN is exponent 15 with
    mantissa 7, so the largest finite magnitude is 1.75 * 2^8 = 448.
    """
    c = np.ascontiguousarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where((c >> 7) & 1, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = c & 0x7
    sub = (m / 8.0) * 2.0 ** -6
    nor = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    val = np.where(e == 0, sub, nor)
    val = np.where((e == 15) & (m == 7), np.nan, val)
    return sign * val


# --------------------------------------------------------------------------
# the definition
# --------------------------------------------------------------------------
def _scores(qh: np.ndarray, kh: np.ndarray, scale: float, causal: bool,
            rows: np.ndarray | None) -> np.ndarray:
    """S = scale * Q K^T for one head (optionally only some query rows), masked."""
    n = kh.shape[0]
    qsel = qh if rows is None else qh[rows]
    s = (qsel @ kh.T) * float(scale)
    if causal:
        i = (np.arange(qh.shape[0]) if rows is None else np.asarray(rows))[:, None]
        j = np.arange(n)[None, :]
        s = np.where(j > i, -np.inf, s)
    return s


def softmax_rows(s: np.ndarray):
    """Row softmax of a score matrix.  Returns (P, m, l): P rows sum to one,
    m the row maxima, l the row sums of exp(s - m)."""
    m = np.max(s, axis=1)
    e = np.exp(s - m[:, None])
    l = np.sum(e, axis=1)
    return e / l[:, None], m, l


def attn_head(qh: np.ndarray, kh: np.ndarray, vh: np.ndarray, causal: bool,
              scale: float, rows: np.ndarray | None = None):
    """One (batch, head): qh [N,d], kh [N,d], vh [N,d] float64.
    Returns O [N or len(rows), d] and lse [N or len(rows)]."""
    s = _scores(qh, kh, scale, causal, rows)
    p, m, l = softmax_rows(s)
    return p @ vh, m + np.log(l)


def attn_ref(q: np.ndarray, k: np.ndarray, v: np.ndarray, causal: bool, scale: float):
    """Whole tensor.  q [B,Hq,N,d], k and v [B,Hkv,N,d], float64.
    Query head h reads kv head h // (Hq // Hkv).
    Returns O [B,Hq,N,d] float64 (never rounded) and lse [B,Hq,N] float64."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, Hq, N, d = q.shape
    Bk, Hkv, Nk, dk = k.shape
    if (Bk, Nk, dk) != (B, N, d) or v.shape != k.shape or Hq % Hkv != 0:
        raise ValueError("inconsistent attention shapes")
    G = Hq // Hkv
    o = np.empty((B, Hq, N, d), dtype=np.float64)
    lse = np.empty((B, Hq, N), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            o[b, h], lse[b, h] = attn_head(q[b, h], k[b, h // G], v[b, h // G], causal, scale)
    return o, lse


def attn_ref_rows(q: np.ndarray, k: np.ndarray, v: np.ndarray, causal: bool, scale: float,
                  b: int, h: int, rows):
    """The same definition for a sample of query rows of one (b, h): used where
    the whole tensor is too large to evaluate.  q,k,v as in attn_ref (or any
    arrays indexable as [b, head] giving float64 [N,d])."""
    Hq, Hkv = q.shape[1], k.shape[1]
    g = h // (Hq // Hkv)
    rows = np.asarray(rows, dtype=np.int64)
    return attn_head(np.asarray(q[b, h], dtype=np.float64),
                     np.asarray(k[b, g], dtype=np.float64),
                     np.asarray(v[b, g], dtype=np.float64), causal, scale, rows)


# --------------------------------------------------------------------------
# error metrics used by every parity check
# --------------------------------------------------------------------------
def error_metrics(o_test: np.ndarray, o_ref: np.ndarray, lse_test: np.ndarray, lse_ref: np.ndarray):
    """max-abs and relative Frobenius error of O, max-abs error of lse."""
    o_test = np.asarray(o_test, dtype=np.float64)
    o_ref = np.asarray(o_ref, dtype=np.float64)
    diff = o_test - o_ref
    denom = float(np.sqrt(np.sum(o_ref * o_ref)))
    return {
        "max_abs": float(np.max(np.abs(diff))) if diff.size else 0.0,
        "rel_fro": float(np.sqrt(np.sum(diff * diff)) / denom) if denom > 0 else 0.0,
        "lse_max_abs": float(np.max(np.abs(np.asarray(lse_test, np.float64) - lse_ref))) if lse_ref.size else 0.0,
    }
