"""GPU parity of the attention backward pass (bf16, head dimension 128 or 64): the HIP path, called
through the C ABI on the forward's own outputs, against the float64 CPU oracle of the
gradients on the same seeded inputs."""
import numpy as np
import pytest
import torch

import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _case(ci, B, Hq, Hkv, N, causal=None, seed=None, d=None):
    cfg = dict(wl.CONFIGS[ci])
    if causal is not None:
        cfg["causal"] = causal
    if seed is not None:
        cfg["seed"] = seed
    if d is not None:
        cfg["d"] = d
        cfg["scale"] = 1.0 / float(np.sqrt(d))
    inp = wl.make_inputs(cfg, B=B, Hq=Hq, Hkv=Hkv, N=N)
    return cfg, inp, wl.make_dout(cfg, B=B, Hq=Hq, N=N)


# several tiles, ragged tails, both masks, grouped heads
REDUCED = [
    # (config index, B, Hq, Hkv, N)
    (1, 1, 2, 2, 2048),
    (1, 2, 2, 2, 1000),
    (1, 1, 2, 2, 257),
    (2, 1, 2, 2, 2048),
    (2, 1, 2, 2, 1531),
    (3, 1, 8, 2, 1024),
    (3, 2, 8, 1, 777),
    (3, 1, 16, 2, 320),
]


@pytest.mark.parametrize("ci,B,Hq,Hkv,N", REDUCED)
def test_bwd_reduced_configs(ci, B, Hq, Hkv, N):
    cfg, inp, dob = _case(ci, B, Hq, Hkv, N)
    print(f"bwd config{ci + 1} reduced B={B} Hq={Hq} Hkv={Hkv} N={N} causal={cfg['causal']}", flush=True)
    dq, dk, dv, _, _ = gu.run_gpu_bwd(inp, dob)
    print(gu.check_bwd_full(inp, dob, dq, dk, dv, f"bwd cfg{ci + 1} N={N}"), flush=True)


@pytest.mark.parametrize("N", [1, 2, 31, 32, 33, 63, 64, 65, 127, 129, 255, 256, 257, 511, 513])
@pytest.mark.parametrize("causal", [False, True])
def test_bwd_edge_lengths(N, causal):
    cfg, inp, dob = _case(1, 1, 2, 1, N, causal=causal, seed=177 + N)
    print(f"bwd edge N={N} causal={causal}", flush=True)
    dq, dk, dv, _, _ = gu.run_gpu_bwd(inp, dob)
    gu.check_bwd_full(inp, dob, dq, dk, dv, f"bwd edge N={N} causal={causal}")


# head dimension 64: the same kernels with half the k-steps and column blocks and the 128-byte-row
# swizzle of the streamed tiles
@pytest.mark.parametrize("N", [1, 33, 64, 65, 127, 128, 129, 255, 257, 513])
@pytest.mark.parametrize("causal", [False, True])
def test_bwd_d64_edge_lengths(N, causal):
    cfg, inp, dob = _case(1, 1, 2, 1, N, causal=causal, seed=911 + N, d=64)
    print(f"bwd d64 edge N={N} causal={causal}", flush=True)
    dq, dk, dv, _, _ = gu.run_gpu_bwd(inp, dob)
    gu.check_bwd_full(inp, dob, dq, dk, dv, f"bwd d64 edge N={N} causal={causal}")


@pytest.mark.parametrize("ci,B,Hq,Hkv,N", [(1, 1, 2, 2, 2048), (2, 2, 2, 2, 1531), (3, 1, 8, 2, 1024), (3, 2, 8, 1, 777)])
def test_bwd_d64_reduced_configs(ci, B, Hq, Hkv, N):
    cfg, inp, dob = _case(ci, B, Hq, Hkv, N, d=64)
    print(f"bwd d64 config{ci + 1} reduced B={B} Hq={Hq} Hkv={Hkv} N={N} causal={cfg['causal']}", flush=True)
    dq, dk, dv, _, _ = gu.run_gpu_bwd(inp, dob)
    print(gu.check_bwd_full(inp, dob, dq, dk, dv, f"bwd d64 cfg{ci + 1} N={N}"), flush=True)


def _bits(x):
    return wl.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


@pytest.mark.parametrize("causal", [False, True])
def test_bwd_adversarial_rows(causal):
    """Degenerate score patterns: all-equal scores (uniform P), one dominant key per row
    (P close to one-hot, dS close to zero), large magnitudes."""
    rng = np.random.default_rng(6)
    N, d = 640, 128
    scale = 1.0 / d ** 0.5
    q = rng.standard_normal((1, 2, N, d)).astype(np.float32)
    k = rng.standard_normal((1, 1, N, d)).astype(np.float32)
    v = rng.standard_normal((1, 1, N, d)).astype(np.float32)
    do = rng.standard_normal((1, 2, N, d)).astype(np.float32)
    k_dom = k.copy()
    k_dom[0, 0, 5] = 8.0 * q[0, 0, 300] / np.linalg.norm(q[0, 0, 300]) * 4
    cases = dict(all_equal_scores=(q, np.zeros_like(k)), dominant_key=(q, k_dom), large_magnitude=(q * 4, k * 4))
    for name, (qq, kk) in cases.items():
        inp = dict(B=1, Hq=2, Hkv=1, N=N, d=d, causal=causal, scale=scale, dtype="bf16", q=_bits(qq), k=_bits(kk), v=_bits(v),
                   descale=(1.0, 1.0, 1.0))
        print(f"bwd adversarial {name} causal={causal}", flush=True)
        dob = _bits(do)
        dq, dk, dv, _, _ = gu.run_gpu_bwd(inp, dob)
        # softmax rows close to one-hot: same cancellation in dP - delta as in few-key rows
        gu.check_bwd_full(inp, dob, dq, dk, dv, f"bwd {name} causal={causal}", peaked=name != "all_equal_scores")


def test_bwd_zero_dout_gives_zero_gradients():
    cfg, inp, dob = _case(1, 1, 2, 2, 300)
    dq, dk, dv, _, _ = gu.run_gpu_bwd(inp, np.zeros_like(dob))
    for g in (dq, dk, dv):
        assert bool((g.float() == 0).all())


def test_bwd_determinism_and_workspace_contents_do_not_matter():
    cfg, inp, dob = _case(3, 1, 8, 2, 1024)
    a = gu.run_gpu_bwd(inp, dob, poison=float("nan"))
    b = gu.run_gpu_bwd(inp, dob, poison=1.0e30)
    for x, y in zip(a[:3], b[:3]):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16))


def test_bwd_rejects_what_it_does_not_cover():
    import paper_2605_10905_amd as A

    t = torch.zeros(1 * 2 * 64 * 128, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(2 * 64, dtype=torch.float32, device="cuda")
    ws = torch.zeros(A.attn_bwd_workspace_bytes(1, 2, 64) // 4, dtype=torch.float32, device="cuda")
    common = dict(stream=None, check=False)
    # other head dimensions than 128 and 64, and fp8, have no backward kernel
    assert A.attn_bwd(t, t, t, t, t, lse, t, t, t, ws, 1, 2, 2, 64, 32, 0, 0.125, A.ATTN_BF16, **common) != 0
    assert A.attn_bwd(t, t, t, t, t, lse, t, t, t, ws, 1, 2, 2, 64, 128, 0, 0.125, A.ATTN_FP8_E4M3, **common) != 0
    assert A.attn_bwd(t, t, t, t, t, lse, t, t, t, None, 1, 2, 2, 64, 128, 0, 0.125, A.ATTN_BF16, **common) != 0


# ---- full-size configs in the launch configuration bench.py --backward times -------------------
@pytest.mark.parametrize("ci", [1, 2, 3])
def test_bwd_full_size(ci):
    cfg = wl.CONFIGS[ci]
    print(f"bwd full-size config{ci + 1}: generating inputs", flush=True)
    inp = wl.make_inputs(cfg)
    dob = wl.make_dout(cfg)
    print(f"bwd full-size config{ci + 1}: launching", flush=True)
    dq, dk, dv, _, _ = gu.run_gpu_bwd(inp, dob)
    for g in (dq, dk, dv):
        assert bool(torch.isfinite(g.float()).all())
    B, Hq, Hkv, N = cfg["B"], cfg["Hq"], cfg["Hkv"], cfg["N"]
    G = Hq // Hkv
    # properties that hold at any size, over every head:
    #  * rows of P sum to one, so the column sums of dV equal those of dO summed over the group
    #  * tr(Q^T dQ) summed over the group equals tr(K^T dK) (both are scale * sum(dS * Q K^T))
    do = gu.bf16_to_device(dob).float()
    dev = gu.to_device(inp)
    lhs = dv.float().sum(dim=2)
    rhs = do.sum(dim=2).view(B, Hkv, G, -1).sum(dim=2)
    tol = 2e-2 * float(N) ** 0.5 * G ** 0.5
    assert float((lhs - rhs).abs().max()) <= tol, float((lhs - rhs).abs().max())
    tq = (dev["q"].float() * dq.float()).sum(dim=(2, 3)).view(B, Hkv, G).sum(dim=2)
    tk = (dev["k"].float() * dk.float()).sum(dim=(2, 3))
    norm = ((dev["q"].float() * dq.float()).abs().sum(dim=(2, 3)).view(B, Hkv, G).sum(dim=2)) + 1e-6
    assert float(((tq - tk).abs() / norm).max()) <= 5e-3, float(((tq - tk).abs() / norm).max())
    # the oracle on whole (batch, kv head) groups
    rng = np.random.default_rng(200 + ci)
    groups = [(0, 0), (B - 1, Hkv - 1)] if N <= 4096 else [(int(rng.integers(0, B)), int(rng.integers(0, Hkv)))]
    for b, g in groups:
        print(f"bwd full-size config{ci + 1}: oracle on group b={b} g={g} ({G} query heads)", flush=True)
        m = gu.check_bwd_group(inp, dob, dq, dk, dv, b, g, f"bwd config{ci + 1} full size group {(b, g)}")
        print(f"bwd full-size config{ci + 1}: {m}", flush=True)


def _random_bwd_shapes(seed, count, max_n):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        hkv = int(rng.integers(1, 4))
        g = int(rng.choice([1, 2, 4]))
        out.append((int(rng.integers(1, 3)), hkv * g, hkv, int(rng.integers(1, max_n + 1)), bool(rng.integers(0, 2)), int(rng.integers(1, 1 << 30))))
    return out


@pytest.mark.parametrize("B,Hq,Hkv,N,causal,seed", _random_bwd_shapes(20260512, 16, 700))
def test_bwd_random_shapes(B, Hq, Hkv, N, causal, seed):
    """Seeded random batch / head / group / length / mask combinations."""
    cfg, inp, dob = _case(1, B, Hq, Hkv, N, causal=causal, seed=seed)
    print(f"bwd random B={B} Hq={Hq} Hkv={Hkv} N={N} causal={causal}", flush=True)
    dq, dk, dv, _, _ = gu.run_gpu_bwd(inp, dob)
    gu.check_bwd_full(inp, dob, dq, dk, dv, f"bwd random B={B} Hq={Hq} Hkv={Hkv} N={N} causal={causal}")
