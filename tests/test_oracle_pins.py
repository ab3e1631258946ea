"""Pins for the CPU oracle: closed forms, brute force, invariances, library routines.

Each test is chosen so that a plausible mistake in oracle/attn_ref.py (dropped
scale, wrong sign, transposed operand, wrong GQA mapping, off-by-one in the
causal mask, wrong log base) fails at least one of them.  None of the expected
values comes from the oracle or from the HIP path.
"""
import math
import os

import numpy as np
import pytest

from oracle import attn_ref as orc

RNG = np.random.default_rng(7)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand(*shape):
    return RNG.standard_normal(shape)


def brute_force(q, k, v, causal, scale):
    """Scalar triple loop with math.exp: the definition with nothing vectorised."""
    B, Hq, N, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    o = np.zeros((B, Hq, N, d))
    lse = np.zeros((B, Hq, N))
    for b in range(B):
        for h in range(Hq):
            g = h // G
            for i in range(N):
                vis = [j for j in range(N) if (not causal) or j <= i]
                s = []
                for j in vis:
                    acc = 0.0
                    for c in range(d):
                        acc += q[b, h, i, c] * k[b, g, j, c]
                    s.append(acc * scale)
                mx = max(s)
                e = [math.exp(x - mx) for x in s]
                tot = sum(e)
                for c in range(d):
                    o[b, h, i, c] = sum(e[t] * v[b, g, j, c] for t, j in enumerate(vis)) / tot
                lse[b, h, i] = mx + math.log(tot)
    return o, lse


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 2), (6, 1)])
def test_brute_force(causal, Hq, Hkv):
    q, k, v = rand(2, Hq, 11, 5), rand(2, Hkv, 11, 5), rand(2, Hkv, 11, 5)
    o, lse = orc.attn_ref(q, k, v, causal, 0.37)
    bo, bl = brute_force(q, k, v, causal, 0.37)
    np.testing.assert_allclose(o, bo, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, bl, rtol=0, atol=1e-13)


def test_golden_rational_example():
    q = np.array([1.0, 2.0, 0.0]).reshape(1, 1, 3, 1)
    k = np.array([0.0, math.log(2.0), math.log(4.0)]).reshape(1, 1, 3, 1)
    v = np.array([3.0, 6.0, 12.0]).reshape(1, 1, 3, 1)
    res = {False: orc.attn_ref(q, k, v, False, 1.0), True: orc.attn_ref(q, k, v, True, 1.0)}
    n = 0
    with open(os.path.join(GOLDEN, "softmax_rational.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            mode, row, o_exp, lse_arg = line.split()
            o, lse = res[mode == "causal"]
            assert abs(o[0, 0, int(row), 0] - float(o_exp)) < 1e-12
            assert abs(lse[0, 0, int(row)] - math.log(float(lse_arg))) < 1e-12
            n += 1
    assert n == 6


def test_rows_of_P_sum_to_one_and_match_scipy():
    from scipy.special import logsumexp, softmax

    s = rand(9, 13) * 3
    p, m, l = orc.softmax_rows(s)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, atol=1e-15)
    np.testing.assert_allclose(p, softmax(s, axis=1), atol=1e-15)
    np.testing.assert_allclose(m + np.log(l), logsumexp(s, axis=1), atol=1e-14)
    assert (p >= 0).all()


@pytest.mark.parametrize("causal", [False, True])
def test_constant_V_gives_that_row(causal):
    q, k = rand(1, 3, 8, 4), rand(1, 3, 8, 4)
    row = rand(4)
    v = np.broadcast_to(row, (1, 3, 8, 4)).copy()
    o, _ = orc.attn_ref(q, k, v, causal, 0.5)
    np.testing.assert_allclose(o, v, atol=1e-14)


def test_zero_K_gives_mean_of_V_and_log_count():
    q, v = rand(2, 2, 10, 3), rand(2, 2, 10, 3)
    k = np.zeros_like(v)
    o, lse = orc.attn_ref(q, k, v, False, 0.7)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(axis=2, keepdims=True), o.shape), atol=1e-14)
    np.testing.assert_allclose(lse, math.log(10), atol=1e-14)
    o, lse = orc.attn_ref(q, k, v, True, 0.7)
    prefix = np.cumsum(v, axis=2) / np.arange(1, 11)[None, None, :, None]
    np.testing.assert_allclose(o, prefix, atol=1e-14)
    np.testing.assert_allclose(lse, np.broadcast_to(np.log(np.arange(1, 11)), lse.shape), atol=1e-14)


def test_causal_row0_is_V0_and_lse_is_its_score():
    q, k, v = rand(2, 2, 6, 4), rand(2, 2, 6, 4), rand(2, 2, 6, 4)
    o, lse = orc.attn_ref(q, k, v, True, 0.25)
    np.testing.assert_allclose(o[:, :, 0], v[:, :, 0], atol=1e-15)
    np.testing.assert_allclose(lse[:, :, 0], 0.25 * np.sum(q[:, :, 0] * k[:, :, 0], axis=-1), atol=1e-14)


def test_causal_row_equals_noncausal_on_prefix():
    # catches an off-by-one or flipped mask: row i of causal attention is plain
    # attention over keys 0..i only.
    q, k, v = rand(1, 2, 9, 4), rand(1, 2, 9, 4), rand(1, 2, 9, 4)
    oc, lc = orc.attn_ref(q, k, v, True, 0.4)
    for i in range(9):
        on, ln = _prefix(q, k, v, i, 0.4)
        np.testing.assert_allclose(oc[:, :, i], on, atol=1e-14)
        np.testing.assert_allclose(lc[:, :, i], ln, atol=1e-14)


def _prefix(q, k, v, i, scale):
    # query row i against keys 0..i, via scipy's softmax (not the oracle's)
    from scipy.special import logsumexp, softmax

    s = np.einsum("bhd,bhjd->bhj", q[:, :, i], k[:, :, :i + 1]) * scale
    return np.einsum("bhj,bhjd->bhd", softmax(s, axis=-1), v[:, :, :i + 1]), logsumexp(s, axis=-1)


def test_dominant_key_selects_its_value_row():
    N, d = 7, 4
    q = np.zeros((1, 1, N, d)); q[..., 0] = 1.0
    k = np.zeros((1, 1, N, d)); k[0, 0, 3, 0] = 60.0
    v = rand(1, 1, N, d)
    o, lse = orc.attn_ref(q, k, v, False, 1.0)
    np.testing.assert_allclose(o, np.broadcast_to(v[:, :, 3:4], o.shape), atol=1e-13)
    np.testing.assert_allclose(lse, 60.0, atol=1e-13)


def test_single_key():
    q, k, v = rand(1, 2, 1, 4), rand(1, 2, 1, 4), rand(1, 2, 1, 4)
    for causal in (False, True):
        o, lse = orc.attn_ref(q, k, v, causal, 0.3)
        np.testing.assert_allclose(o, v, atol=1e-15)
        np.testing.assert_allclose(lse[..., 0], 0.3 * np.sum(q * k, axis=-1)[..., 0], atol=1e-15)


def test_key_permutation_invariance_noncausal():
    q, k, v = rand(1, 2, 12, 4), rand(1, 2, 12, 4), rand(1, 2, 12, 4)
    perm = RNG.permutation(12)
    o1, l1 = orc.attn_ref(q, k, v, False, 0.5)
    o2, l2 = orc.attn_ref(q, k[:, :, perm], v[:, :, perm], False, 0.5)
    np.testing.assert_allclose(o1, o2, atol=1e-14)
    np.testing.assert_allclose(l1, l2, atol=1e-14)


def test_key_shift_moves_lse_only():
    q, k, v = rand(1, 2, 8, 4), rand(1, 2, 8, 4), rand(1, 2, 8, 4)
    c = rand(4)
    o1, l1 = orc.attn_ref(q, k, v, True, 0.5)
    o2, l2 = orc.attn_ref(q, k + c, v, True, 0.5)
    np.testing.assert_allclose(o1, o2, atol=1e-13)
    np.testing.assert_allclose(l2 - l1, 0.5 * (q @ c), atol=1e-13)


def test_scale_trades_against_Q():
    q, k, v = rand(1, 2, 8, 4), rand(1, 2, 8, 4), rand(1, 2, 8, 4)
    o1, l1 = orc.attn_ref(q, k, v, False, 0.5)
    o2, l2 = orc.attn_ref(q * 0.5, k, v, False, 1.0)
    np.testing.assert_allclose(o1, o2, atol=1e-14)
    np.testing.assert_allclose(l1, l2, atol=1e-14)
    # and scale really is applied: a different scale changes the answer
    o3, _ = orc.attn_ref(q, k, v, False, 1.0)
    assert np.max(np.abs(o3 - o1)) > 1e-3


def test_gqa_is_mha_with_repeated_kv_contiguous_groups():
    q, k, v = rand(2, 6, 7, 4), rand(2, 2, 7, 4), rand(2, 2, 7, 4)
    o1, l1 = orc.attn_ref(q, k, v, True, 0.5)
    o2, l2 = orc.attn_ref(q, np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1), True, 0.5)
    np.testing.assert_allclose(o1, o2, atol=0)
    np.testing.assert_allclose(l1, l2, atol=0)
    # heads 0..2 use kv head 0, heads 3..5 kv head 1 (contiguous, not interleaved)
    o3, _ = orc.attn_ref(q[:, 3:4], k[:, 1:2], v[:, 1:2], True, 0.5)
    np.testing.assert_allclose(o1[:, 3:4], o3, atol=0)


@pytest.mark.parametrize("causal", [False, True])
def test_against_torch_sdpa_float64(causal):
    import torch
    import torch.nn.functional as F

    q, k, v = rand(2, 4, 33, 16), rand(2, 2, 33, 16), rand(2, 2, 33, 16)
    o, lse = orc.attn_ref(q, k, v, causal, 0.21)
    tq = torch.from_numpy(q)
    tk = torch.from_numpy(np.repeat(k, 2, axis=1))
    tv = torch.from_numpy(np.repeat(v, 2, axis=1))
    to = F.scaled_dot_product_attention(tq, tk, tv, is_causal=causal, scale=0.21)
    np.testing.assert_allclose(o, to.numpy(), atol=1e-12)
    s = torch.einsum("bhid,bhjd->bhij", tq, tk) * 0.21
    if causal:
        s = s.masked_fill(torch.triu(torch.ones(33, 33, dtype=torch.bool), 1), float("-inf"))
    np.testing.assert_allclose(lse, torch.logsumexp(s, dim=-1).numpy(), atol=1e-12)


def test_split_key_merge_identity():
    # the algebra the streaming softmax relies on: two key halves merge through lse
    q, k, v = rand(1, 1, 6, 4), rand(1, 1, 10, 4), rand(1, 1, 10, 4)
    # (rectangular on purpose: use attn_head directly)
    o, lse = orc.attn_head(q[0, 0], k[0, 0], v[0, 0], False, 0.6)
    oa, la = orc.attn_head(q[0, 0], k[0, 0, :4], v[0, 0, :4], False, 0.6)
    ob, lb = orc.attn_head(q[0, 0], k[0, 0, 4:], v[0, 0, 4:], False, 0.6)
    lm = np.logaddexp(la, lb)
    np.testing.assert_allclose(lse, lm, atol=1e-14)
    np.testing.assert_allclose(o, np.exp(la - lm)[:, None] * oa + np.exp(lb - lm)[:, None] * ob, atol=1e-14)


def test_rows_variant_matches_full():
    q, k, v = rand(2, 4, 20, 8), rand(2, 2, 20, 8), rand(2, 2, 20, 8)
    for causal in (False, True):
        o, lse = orc.attn_ref(q, k, v, causal, 0.3)
        rows = [0, 3, 19]
        orow, lrow = orc.attn_ref_rows(q, k, v, causal, 0.3, 1, 3, rows)
        np.testing.assert_allclose(orow, o[1, 3, rows], atol=1e-15)
        np.testing.assert_allclose(lrow, lse[1, 3, rows], atol=1e-15)


def test_large_scores_do_not_overflow():
    q = np.full((1, 1, 4, 2), 40.0)
    k = np.full((1, 1, 4, 2), 40.0)
    v = rand(1, 1, 4, 2)
    o, lse = orc.attn_ref(q, k, v, False, 1.0)
    assert np.isfinite(o).all() and np.isfinite(lse).all()
    np.testing.assert_allclose(lse, 3200.0 + math.log(4), atol=1e-9)


# ---- storage-format decoders -------------------------------------------------
def test_bf16_decoder_against_torch_and_definition():
    import torch

    bits = np.arange(0, 65536, dtype=np.uint32).astype(np.uint16)
    ours = orc.bf16_bits_to_f64(bits)
    t = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    both = np.isfinite(t)
    assert (np.isfinite(ours) == both).all()
    assert (ours[both] == t[both]).all()
    # definition spot checks: 0x3F80 = 1.0, 0xC000 = -2.0, 0x3DCD ~ 0.1 rounded up
    assert orc.bf16_bits_to_f64(np.array([0x3F80, 0xC000], np.uint16)).tolist() == [1.0, -2.0]
    assert orc.bf16_bits_to_f64(np.array([0x0001], np.uint16))[0] == 2.0 ** -133


def test_e4m3_decoder_against_torch_and_definition():
    import torch

    codes = np.arange(256, dtype=np.uint8)
    ours = orc.e4m3_bits_to_f64(codes)
    t = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.isnan(ours[[0x7F, 0xFF]]).all() and np.isnan(t[[0x7F, 0xFF]]).all()
    fin = ~np.isnan(t)
    assert fin.sum() == 254 and (ours[fin] == t[fin]).all()
    assert ours[0x7E] == 448.0 and ours[0xFE] == -448.0
    assert ours[0x01] == 2.0 ** -9 and ours[0x08] == 2.0 ** -6 and ours[0x38] == 1.0
    # strictly increasing over the positive finite codes
    assert (np.diff(ours[0:0x7F]) > 0).all()


def test_error_metrics_definition():
    o_ref = np.array([[3.0, 4.0]])
    o = np.array([[3.0, 4.5]])
    m = orc.error_metrics(o, o_ref, np.array([1.0]), np.array([1.25]))
    assert m["max_abs"] == 0.5 and abs(m["rel_fro"] - 0.1) < 1e-15 and m["lse_max_abs"] == 0.25
