"""Pins for the backward CPU oracle.  None of the expected values comes from the backward
oracle itself or from the HIP path: finite differences of the forward oracle, a scalar-loop
softmax Jacobian, closed forms, invariances and torch autograd."""
import math

import numpy as np
import pytest

from oracle import attn_bwd_ref as bwd
from oracle import attn_ref as fwd

RNG = np.random.default_rng(11)


def rand(*shape):
    return RNG.standard_normal(shape)


def loss(q, k, v, do, causal, scale):
    o, _ = fwd.attn_ref(q, k, v, causal, scale)
    return float(np.sum(o * do))


def finite_diff(fun, x, h=1e-6):
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        old = x[i]
        x[i] = old + h
        fp = fun()
        x[i] = old - h
        fm = fun()
        x[i] = old
        g[i] = (fp - fm) / (2 * h)
    return g


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2)])
def test_against_finite_differences_of_the_forward_oracle(causal, Hq, Hkv):
    q, k, v, do = rand(1, Hq, 6, 3), rand(1, Hkv, 6, 3), rand(1, Hkv, 6, 3), rand(1, Hq, 6, 3)
    scale = 0.41
    dq, dk, dv = bwd.attn_bwd_ref(q, k, v, do, causal, scale)
    f = lambda: loss(q, k, v, do, causal, scale)
    np.testing.assert_allclose(dq, finite_diff(f, q), rtol=0, atol=2e-8)
    np.testing.assert_allclose(dk, finite_diff(f, k), rtol=0, atol=2e-8)
    np.testing.assert_allclose(dv, finite_diff(f, v), rtol=0, atol=2e-8)


def test_scalar_loop_jacobian_single_head():
    """dL/ds_ij = p_ij (dp_ij - sum_t p_it dp_it), then the chain rule through s = scale q.k,
    all with Python loops and math.exp."""
    N, d, scale = 5, 2, 0.7
    q, k, v, do = rand(N, d), rand(N, d), rand(N, d), rand(N, d)
    for causal in (False, True):
        dq = np.zeros((N, d)); dk = np.zeros((N, d)); dv = np.zeros((N, d))
        for i in range(N):
            vis = [j for j in range(N) if (not causal) or j <= i]
            s = [scale * sum(q[i, c] * k[j, c] for c in range(d)) for j in vis]
            mx = max(s)
            e = [math.exp(x - mx) for x in s]
            p = [x / sum(e) for x in e]
            dp = [sum(do[i, c] * v[j, c] for c in range(d)) for j in vis]
            dot = sum(pt * dpt for pt, dpt in zip(p, dp))
            for t, j in enumerate(vis):
                ds = p[t] * (dp[t] - dot)
                for c in range(d):
                    dq[i, c] += scale * ds * k[j, c]
                    dk[j, c] += scale * ds * q[i, c]
                    dv[j, c] += p[t] * do[i, c]
        a, b, c_ = bwd.attn_bwd_head(q, k, v, do, causal, scale)
        np.testing.assert_allclose(a, dq, rtol=0, atol=1e-13)
        np.testing.assert_allclose(b, dk, rtol=0, atol=1e-13)
        np.testing.assert_allclose(c_, dv, rtol=0, atol=1e-13)


@pytest.mark.parametrize("causal", [False, True])
def test_constant_V_gives_zero_dQ_dK(causal):
    """O does not depend on the scores when all value rows are equal."""
    q, k, do = rand(1, 2, 9, 4), rand(1, 2, 9, 4), rand(1, 2, 9, 4)
    v = np.broadcast_to(rand(1, 2, 1, 4), (1, 2, 9, 4)).copy()
    dq, dk, dv = bwd.attn_bwd_ref(q, k, v, do, causal, 0.5)
    assert np.abs(dq).max() < 1e-14 and np.abs(dk).max() < 1e-14
    # and dV is P^T dO: its column sums equal those of dO (rows of P sum to one)
    np.testing.assert_allclose(dv.sum(axis=2), do.sum(axis=2), rtol=0, atol=1e-12)


def test_zero_K_gives_uniform_weights():
    """K = 0: P = 1/N everywhere (non-causal), so dV_j = mean_i dO_i for every j and
    dQ = 0 (dS K = 0)."""
    N = 8
    q, v, do = rand(1, 1, N, 3), rand(1, 1, N, 3), rand(1, 1, N, 3)
    k = np.zeros((1, 1, N, 3))
    dq, dk, dv = bwd.attn_bwd_ref(q, k, v, do, False, 1.3)
    assert np.abs(dq).max() == 0.0
    np.testing.assert_allclose(dv[0, 0], np.broadcast_to(do[0, 0].mean(axis=0), (N, 3)), rtol=0, atol=1e-14)


def test_key_shift_invariance_means_dK_sums_to_zero():
    """Adding one vector to every key leaves O unchanged (non-causal), so the gradient has no
    component along that direction: sum_j dK_j = 0."""
    q, k, v, do = rand(2, 2, 10, 4), rand(2, 2, 10, 4), rand(2, 2, 10, 4), rand(2, 2, 10, 4)
    _, dk, _ = bwd.attn_bwd_ref(q, k, v, do, False, 0.6)
    assert np.abs(dk.sum(axis=2)).max() < 1e-13


def test_causal_last_key_only_sees_last_query():
    N = 7
    q, k, v, do = rand(1, 1, N, 3), rand(1, 1, N, 3), rand(1, 1, N, 3), rand(1, 1, N, 3)
    _, dk, dv = bwd.attn_bwd_ref(q, k, v, do, True, 0.9)
    # weight of the last key in the last row
    s = 0.9 * (k[0, 0] @ q[0, 0, N - 1])
    p = np.exp(s - s.max()); p /= p.sum()
    np.testing.assert_allclose(dv[0, 0, N - 1], p[N - 1] * do[0, 0, N - 1], rtol=0, atol=1e-14)
    # causal row 0 sees only key 0 with weight one: O_0 = V_0, no dependence on q_0
    dq, _, _ = bwd.attn_bwd_ref(q, k, v, do, True, 0.9)
    assert np.abs(dq[0, 0, 0]).max() < 1e-15


def test_scale_trades_against_Q():
    """Doubling scale and halving Q gives the same O, hence dK, dV equal and dQ doubled."""
    q, k, v, do = rand(1, 2, 9, 4), rand(1, 2, 9, 4), rand(1, 2, 9, 4), rand(1, 2, 9, 4)
    a = bwd.attn_bwd_ref(q, k, v, do, True, 0.3)
    b = bwd.attn_bwd_ref(q / 2, k, v, do, True, 0.6)
    np.testing.assert_allclose(b[0], 2 * a[0], rtol=0, atol=1e-13)
    np.testing.assert_allclose(b[1], a[1], rtol=0, atol=1e-13)
    np.testing.assert_allclose(b[2], a[2], rtol=0, atol=1e-13)


def test_gqa_sums_the_group():
    q, do = rand(1, 4, 8, 3), rand(1, 4, 8, 3)
    k, v = rand(1, 2, 8, 3), rand(1, 2, 8, 3)
    dq, dk, dv = bwd.attn_bwd_ref(q, k, v, do, False, 0.5)
    kr, vr = np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1)
    dq2, dk2, dv2 = bwd.attn_bwd_ref(q, kr, vr, do, False, 0.5)
    np.testing.assert_allclose(dq, dq2, rtol=0, atol=1e-14)
    np.testing.assert_allclose(dk, dk2.reshape(1, 2, 2, 8, 3).sum(axis=2), rtol=0, atol=1e-13)
    np.testing.assert_allclose(dv, dv2.reshape(1, 2, 2, 8, 3).sum(axis=2), rtol=0, atol=1e-13)


@pytest.mark.parametrize("causal", [False, True])
def test_against_torch_autograd_float64(causal):
    import torch

    q, k, v, do = rand(2, 4, 17, 8), rand(2, 2, 17, 8), rand(2, 2, 17, 8), rand(2, 4, 17, 8)
    scale = 0.29
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    kr, vr = tk.repeat_interleave(2, dim=1), tv.repeat_interleave(2, dim=1)
    o = torch.nn.functional.scaled_dot_product_attention(tq, kr, vr, is_causal=causal, scale=scale)
    (o * torch.tensor(do)).sum().backward()
    dq, dk, dv = bwd.attn_bwd_ref(q, k, v, do, causal, scale)
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=0, atol=1e-12)


def test_error_metrics_definition():
    a = np.array([1.0, 2.0, 2.0]); b = np.array([1.0, 2.0, 0.0])
    m = bwd.grad_error_metrics(a, b)
    assert m["max_abs"] == 2.0 and abs(m["rel_fro"] - 2.0 / math.sqrt(5.0)) < 1e-15
