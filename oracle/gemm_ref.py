"""CPU oracle for the bf16 GEMM.  TEST INFRASTRUCTURE ONLY.

Imported only by tests/, by __graft_entry__.smoke() and by the cpu_baseline leg of bench.py;
the product never imports it and shares no code, table or constant with it.

What is computed (paper section 6.1, GEMM paragraph; section 6.3 and appendix A, the GEMM
shape tables, of which the MI350 one lists 256^3 ... 2048^3): the dense matrix product with
the second operand stored row-major as [N, K], the layout of a linear layer's weight:

    C[m, n] = sum_k A[m, k] * B[n, k]          A [M,K],  B [N,K],  C [M,N]

or, with `b_is_kn`, the second operand stored as [K, N]:  C[m, n] = sum_k A[m, k] * B[k, n].
The oracle is that definition in float64 on the exact values of the bf16 inputs; numpy's
matmul is the one library step.  It also returns sum_k |A[m,k]| |B[n,k]|, the quantity that
bounds the rounding error of any summation order.

Pinned by tests/test_oracle_gemm_pins.py (scalar triple loop, closed forms, identities that
catch a transposed or swapped operand); nothing is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> the float64 values they stand for."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def gemm_ref(a, b, b_is_kn: bool = False):
    """a float64 [M,K]; b float64 [N,K] (or [K,N] with b_is_kn).  Returns C [M,N] float64."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    if a.ndim != 2 or b.ndim != 2:
        raise ValueError("gemm_ref takes matrices")
    bt = b if b_is_kn else b.T
    if a.shape[1] != bt.shape[0]:
        raise ValueError("inner dimensions differ")
    return a @ bt


def gemm_abs_ref(a, b, b_is_kn: bool = False):
    """sum_k |A[m,k]| |B[n,k]|: the scale of the rounding-error bound of a length-K dot product."""
    return gemm_ref(np.abs(np.asarray(a, dtype=np.float64)), np.abs(np.asarray(b, dtype=np.float64)), b_is_kn)


def gemm_rows(a, b, rows, b_is_kn: bool = False):
    """Selected rows of C only (full-size checks): C[rows, :]."""
    a = np.asarray(a, dtype=np.float64)
    return gemm_ref(a[np.asarray(rows)], b, b_is_kn)


def error_metrics(test, ref):
    test = np.asarray(test, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    diff = test - ref
    den = float(np.sqrt(np.sum(ref * ref)))
    return {"max_abs": float(np.max(np.abs(diff))) if diff.size else 0.0,
            "rel_fro": float(np.sqrt(np.sum(diff * diff)) / den) if den > 0 else 0.0}
