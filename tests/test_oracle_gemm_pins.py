"""Pins of the GEMM oracle against things other than itself: a scalar triple loop, closed
forms, and identities chosen so that a transposed operand, a swapped index or a wrong layout
flag fails at least one of them."""
import numpy as np
import pytest

from oracle import gemm_ref as og


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


@pytest.mark.parametrize("M,N,K", [(3, 5, 7), (1, 1, 1), (4, 2, 9), (6, 6, 2)])
def test_scalar_triple_loop(M, N, K):
    a, b = _rand((M, K), 1), _rand((N, K), 2)
    c = og.gemm_ref(a, b)
    assert c.shape == (M, N)
    for m in range(M):
        for n in range(N):
            s = 0.0
            for k in range(K):
                s += a[m, k] * b[n, k]
            assert abs(c[m, n] - s) <= 1e-12 * (1 + abs(s))


def test_closed_form_index_ramps():
    # A[m,k] = m + 1, B[n,k] = (n + 1) * (k + 1):  C[m,n] = (m+1)(n+1) K(K+1)/2
    M, N, K = 5, 4, 11
    a = np.repeat(np.arange(1, M + 1, dtype=np.float64)[:, None], K, axis=1)
    b = np.outer(np.arange(1, N + 1), np.arange(1, K + 1)).astype(np.float64)
    c = og.gemm_ref(a, b)
    want = np.outer(np.arange(1, M + 1), np.arange(1, N + 1)) * (K * (K + 1) / 2)
    assert np.array_equal(c, want)
    # and the asymmetric one: A[m,k] = k^2 delta(m, 2): only row 2 is non-zero
    a2 = np.zeros((M, K)); a2[2] = np.arange(K) ** 2
    c2 = og.gemm_ref(a2, b)
    assert np.all(c2[[0, 1, 3, 4]] == 0)
    assert np.array_equal(c2[2], np.arange(1, N + 1) * np.sum(np.arange(K) ** 2 * np.arange(1, K + 1)))


def test_identity_and_selection():
    K = 6
    a = _rand((4, K), 3)
    assert np.array_equal(og.gemm_ref(a, np.eye(K)), a)            # B = I ([N=K, K])
    sel = np.zeros((2, K)); sel[0, 4] = 1; sel[1, 1] = 1             # B rows pick columns 4 and 1 of A
    assert np.array_equal(og.gemm_ref(a, sel), a[:, [4, 1]])


def test_layout_flag_and_transpose_identity():
    a, b = _rand((5, 8), 4), _rand((3, 8), 5)
    c = og.gemm_ref(a, b)
    assert np.allclose(og.gemm_ref(a, b.T.copy(), b_is_kn=True), c, rtol=0, atol=1e-13)
    assert np.allclose(og.gemm_ref(b, a).T, c, rtol=0, atol=1e-13)     # (A B^T)^T = B A^T
    with pytest.raises(ValueError):
        og.gemm_ref(a, b, b_is_kn=True)                                  # [3,8] is not [K=8, N]


def test_linearity_and_rows():
    a, a2, b = _rand((6, 9), 6), _rand((6, 9), 7), _rand((4, 9), 8)
    assert np.allclose(og.gemm_ref(2 * a - 3 * a2, b), 2 * og.gemm_ref(a, b) - 3 * og.gemm_ref(a2, b), atol=1e-12)
    assert np.array_equal(og.gemm_rows(a, b, [5, 0]), og.gemm_ref(a, b)[[5, 0]])


def test_abs_bound_and_bf16_decode():
    a, b = _rand((4, 16), 9), _rand((5, 16), 10)
    assert np.all(np.abs(og.gemm_ref(a, b)) <= og.gemm_abs_ref(a, b) + 1e-12)
    # bf16 bit patterns: 0x3F80 = 1.0, 0xC000 = -2.0, 0x3DCC = 0.099609375, 0x0000 = 0
    bits = np.array([0x3F80, 0xC000, 0x3DCC, 0x0000], dtype=np.uint16)
    assert np.array_equal(og.bf16_bits_to_f64(bits), np.array([1.0, -2.0, 0.099609375, 0.0]))


def test_against_torch_matmul_float64():
    import torch

    a, b = _rand((17, 33), 11), _rand((9, 33), 12)
    want = (torch.from_numpy(a) @ torch.from_numpy(b).T).numpy()
    assert np.allclose(og.gemm_ref(a, b), want, rtol=0, atol=1e-12)
    m = og.error_metrics(want, og.gemm_ref(a, b))
    assert m["rel_fro"] < 1e-14
