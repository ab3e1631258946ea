"""CPU oracle for the attention BACKWARD pass.  TEST INFRASTRUCTURE ONLY.

Imported only by tests/, by __graft_entry__.smoke() and by the cpu_baseline leg of
bench.py; the product never imports it and shares no code, table or constant with it.

What is computed (paper section 6.1 lists the backward pass beside the forward among the
attention kernels; appendix A, attention shape table, backward rows): the gradients of the
forward operation of oracle/attn_ref.py with respect to Q, K and V, given the gradient dO of
the output.  With S, P, O as in the forward definition and the scalar L = sum(O * dO):

    dV[b,g] = sum over the query heads h of group g of   P^T dO[b,h]
    dP      = dO[b,h] V[b,g]^T
    dS      = P * (dP - rowsum(P * dP))          (Jacobian of the row softmax; masked
                                                  entries have P = 0, hence dS = 0)
    dQ[b,h] = scale * dS K[b,g]
    dK[b,g] = sum over the heads of the group of   scale * dS^T Q[b,h]

This is the textbook derivation written out on the full N x N matrices in float64:
nothing is tiled, recomputed from a stored statistic or reordered.  (The GPU path uses
the stored logsumexp to rebuild P and the identity rowsum(P * dP) = rowsum(dO * O); the
oracle uses neither.)

Every function here is pinned by tests/test_oracle_bwd_pins.py against central finite
differences of the FORWARD oracle, a scalar-loop Jacobian, closed forms, invariances and
torch autograd in float64; nothing is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

from oracle import attn_ref as fwd


def attn_bwd_head(qh, kh, vh, doh, causal: bool, scale: float):
    """One (batch, query head): qh, kh, vh, doh float64 [N,d].
    Returns dQ [N,d] and this head's contributions dK, dV [N,d]."""
    s = fwd._scores(qh, kh, scale, causal, None)
    p, _, _ = fwd.softmax_rows(s)
    dv = p.T @ doh
    dp = doh @ vh.T
    ds = p * (dp - np.sum(p * dp, axis=1, keepdims=True))
    dq = (ds @ kh) * float(scale)
    dk = (ds.T @ qh) * float(scale)
    return dq, dk, dv


def attn_bwd_ref(q, k, v, do, causal: bool, scale: float):
    """Whole tensor.  q, do [B,Hq,N,d]; k, v [B,Hkv,N,d]; float64.
    Query head h reads kv head h // (Hq // Hkv); dK and dV sum over the heads of a group.
    Returns dQ [B,Hq,N,d], dK, dV [B,Hkv,N,d] float64."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    do = np.asarray(do, dtype=np.float64)
    B, Hq, N, d = q.shape
    Hkv = k.shape[1]
    if k.shape != (B, Hkv, N, d) or v.shape != k.shape or do.shape != q.shape or Hq % Hkv != 0:
        raise ValueError("inconsistent attention shapes")
    G = Hq // Hkv
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            a, bk, bv = attn_bwd_head(q[b, h], k[b, g], v[b, g], do[b, h], causal, scale)
            dq[b, h] = a
            dk[b, g] += bk
            dv[b, g] += bv
    return dq, dk, dv


def grad_error_metrics(test, ref):
    """max-abs and relative Frobenius error of one gradient tensor."""
    test = np.asarray(test, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    diff = test - ref
    den = float(np.sqrt(np.sum(ref * ref)))
    return {"max_abs": float(np.max(np.abs(diff))) if diff.size else 0.0,
            "rel_fro": float(np.sqrt(np.sum(diff * diff)) / den) if den > 0 else 0.0}
