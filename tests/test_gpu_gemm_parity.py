"""GPU parity of the bf16 GEMM: the HIP path, called through the C ABI, against the float64
CPU oracle on the same seeded inputs.

Tolerance (derived from the arithmetic): products of bf16 values are exact in fp32, the fp32
accumulation of K terms errs by at most K * 2^-24 * sum_k |a||b| whatever the order, and the
result is rounded once to bf16 (relative 2^-9).  Element-wise bound:
    |c - ref| <= 2^-8 |ref| + K * 2^-23 * sum_k |a_k||b_k|
(twice each term), and relative Frobenius error <= 3e-3 (bf16 rounding alone gives 1.1e-3 RMS)."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import gemm_ref as og
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _variants(K):
    """The library's own choice plus every variant whose K-slice divides K."""
    import paper_2605_10905_amd as A

    out = [None]
    for i in range(A.gemm_num_variants()):
        if K % A.gemm_variant_kmult(i) == 0:
            out.append(i)
    return out


def run_gemm(a_bits, b_bits, variant=None, poison=float("nan")):
    import paper_2605_10905_amd as A

    M, K = a_bits.shape
    N = b_bits.shape[0]
    a, b = gu.bf16_to_device(a_bits), gu.bf16_to_device(b_bits)
    c = torch.full((M, N), poison, dtype=torch.bfloat16, device="cuda")
    if variant is None:
        A.gemm_bf16_nt(a, b, c, M, N, K)
    else:
        A.gemm_bf16_nt_variant(a, b, c, M, N, K, variant)
    torch.cuda.synchronize()
    return c


def check(c, a_bits, b_bits, label, rows=None):
    a, b = og.bf16_bits_to_f64(a_bits), og.bf16_bits_to_f64(b_bits)
    K = a.shape[1]
    if rows is None:
        ref, mag = og.gemm_ref(a, b), og.gemm_abs_ref(a, b)
        got = c.float().cpu().numpy().astype(np.float64)
    else:
        ref, mag = og.gemm_rows(a, b, rows), og.gemm_rows(np.abs(a), np.abs(b), rows)
        got = c[torch.from_numpy(np.asarray(rows)).cuda()].float().cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all(), f"{label}: non-finite C"
    bound = 2.0 ** -8 * np.abs(ref) + K * 2.0 ** -23 * mag + 1e-30
    worst = float(np.max(np.abs(got - ref) / bound))
    assert worst <= 1.0, f"{label}: element-wise error {worst:.3f} x bound"
    m = og.error_metrics(got, ref)
    assert m["rel_fro"] <= 3e-3, f"{label}: {m}"
    return m


# several tiles, ragged M and N, one to many k-steps
SMALL = [(256, 256, 256), (512, 512, 512), (300, 520, 96), (1, 8, 32), (257, 264, 1024), (1000, 72, 64), (33, 1000, 2048),
         (777, 513, 160), (64, 7, 32), (5, 3, 64), (1024, 1024, 32)]


@pytest.mark.parametrize("M,N,K", SMALL)
def test_gemm_small_shapes_all_variants(M, N, K):
    a, b = wl.make_gemm_inputs(500 + M + N + K, M, N, K)
    for var in _variants(K):
        print(f"gemm {M}x{N}x{K} variant {var}", flush=True)
        c = run_gemm(a, b, var)
        check(c, a, b, f"gemm {M}x{N}x{K} variant {var}")


def test_gemm_structured_inputs():
    """Operands that expose a wrong row/column or k mapping: one-hot rows select single entries."""
    M, N, K = 384, 320, 128
    rng = np.random.default_rng(3)
    a = rng.standard_normal((M, K)).astype(np.float32)
    b = np.zeros((N, K), dtype=np.float32)
    cols = rng.integers(0, K, N)
    b[np.arange(N), cols] = 1.0
    ab, bb = wl.f32_to_bf16_bits(a), wl.f32_to_bf16_bits(b)
    for var in _variants(K):
        c = run_gemm(ab, bb, var)
        want = torch.from_numpy(ab.view(np.int16)).view(torch.bfloat16)[:, torch.from_numpy(cols)]
        assert torch.equal(c.cpu().view(torch.int16), want.contiguous().view(torch.int16)), f"variant {var}"


def test_gemm_determinism_and_unsupported():
    import paper_2605_10905_amd as A

    a, b = wl.make_gemm_inputs(9, 512, 384, 256)
    c1, c2 = run_gemm(a, b), run_gemm(a, b, poison=1.0e30)
    assert torch.equal(c1.view(torch.int16), c2.view(torch.int16))
    t = torch.zeros(64 * 64, dtype=torch.bfloat16, device="cuda")
    assert A.gemm_bf16_nt(t, t, t, 64, 64, 24, check=False) != 0       # K not a multiple of 32
    assert A.gemm_bf16_nt(t, t, None, 64, 64, 32, check=False) != 0
    assert A.gemm_bf16_nt(t, t, t, 0, 64, 32, check=False) != 0


@pytest.mark.parametrize("name", ["mi350_2048", "canonical_k8192", "large_k_512x4096x64512", "large_n_2048x64512x256"])
def test_gemm_full_size_sampled(name):
    """Paper shapes at full size, in the launch configuration bench.py times: the oracle on sampled
    rows of C (tile edges and random rows), every column."""
    g = next(s for s in wl.GEMM_SHAPES if s["name"] == name)
    M, N, K = g["M"], g["N"], g["K"]
    print(f"gemm full size {name}: generating inputs", flush=True)
    a, b = wl.make_gemm_inputs(g["seed"], M, N, K)
    print(f"gemm full size {name}: launching", flush=True)
    c = run_gemm(a, b)
    assert bool(torch.isfinite(c.float()).all())
    rng = np.random.default_rng(g["seed"])
    rows = sorted({0, 1, 255, 256, 127, 128, M - 1, M // 2, *(int(r) for r in rng.integers(0, M, 24))} & set(range(M)))
    print(f"gemm full size {name}: oracle on {len(rows)} rows", flush=True)
    print(check(c, a, b, f"gemm {name}", rows=rows), flush=True)


# ---- split-K ------------------------------------------------------------------------------------------
def run_gemm_splitk(a_bits, b_bits, splits, poison=float("nan")):
    import paper_2605_10905_amd as A

    M, K = a_bits.shape
    N = b_bits.shape[0]
    a, b = gu.bf16_to_device(a_bits), gu.bf16_to_device(b_bits)
    c = torch.full((M, N), poison, dtype=torch.bfloat16, device="cuda")
    ws = torch.full((A.gemm_splitk_workspace_bytes(M, N, splits) // 4,), poison, dtype=torch.float32, device="cuda")
    A.gemm_bf16_nt_splitk(a, b, c, M, N, K, splits, ws)
    torch.cuda.synchronize()
    return c


# one and several tiles, ragged M and N (vector and scalar stores of the partial tiles and of C),
# slices that divide K evenly, a shorter last slice, more slices asked for than k-steps exist
SPLITK = [(256, 256, 512, 2), (300, 520, 4032, 4), (513, 257, 1024, 8), (64, 7, 640, 3), (5, 3, 128, 64), (1000, 72, 2048, 1),
          (512, 384, 8192, 16), (33, 1001, 4096, 5)]


@pytest.mark.parametrize("M,N,K,splits", SPLITK)
def test_gemm_splitk_shapes(M, N, K, splits):
    a, b = wl.make_gemm_inputs(700 + M + N + K, M, N, K)
    print(f"gemm split-K {M}x{N}x{K} splits {splits}", flush=True)
    c = run_gemm_splitk(a, b, splits)
    check(c, a, b, f"gemm split-K {M}x{N}x{K} / {splits}")
    c2 = run_gemm_splitk(a, b, splits, poison=1.0e30)  # deterministic, and no stale workspace value is read
    assert torch.equal(c.view(torch.int16), c2.view(torch.int16))


def test_gemm_splitk_structured_and_unsupported():
    import paper_2605_10905_amd as A

    M, N, K = 384, 320, 1024
    rng = np.random.default_rng(5)
    a = rng.standard_normal((M, K)).astype(np.float32)
    b = np.zeros((N, K), dtype=np.float32)
    cols = rng.integers(0, K, N)
    b[np.arange(N), cols] = 1.0  # one-hot rows: C[m, n] = A[m, cols[n]] exactly, whichever slice holds the column
    ab, bb = wl.f32_to_bf16_bits(a), wl.f32_to_bf16_bits(b)
    c = run_gemm_splitk(ab, bb, 4)
    want = torch.from_numpy(ab.view(np.int16)).view(torch.bfloat16)[:, torch.from_numpy(cols)]
    assert torch.equal(c.cpu().view(torch.int16), want.contiguous().view(torch.int16))
    t = torch.zeros(64 * 64, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(64 * 64 * 4, dtype=torch.float32, device="cuda")
    assert A.gemm_bf16_nt_splitk(t, t, t, 64, 64, 96, 2, w, check=False) != 0    # K not a multiple of 64
    assert A.gemm_bf16_nt_splitk(t, t, t, 64, 64, 64, 0, w, check=False) != 0    # no slices
    assert A.gemm_bf16_nt_splitk(t, t, t, 64, 64, 64, 65, w, check=False) != 0
    assert A.gemm_bf16_nt_splitk(t, t, t, 64, 64, 64, 2, None, check=False) != 0


@pytest.mark.parametrize("name", ["large_k_512x4096x64512", "large_k_2304x1024x65536"])
def test_gemm_splitk_full_size_sampled(name):
    """The paper's large-K shapes with the slice count the library recommends, as bench.py times them."""
    import paper_2605_10905_amd as A

    g = next(s for s in wl.GEMM_SHAPES if s["name"] == name)
    M, N, K = g["M"], g["N"], g["K"]
    splits = A.gemm_splitk_plan(M, N, K)
    assert splits > 1
    print(f"gemm split-K full size {name}: {splits} slices, generating inputs", flush=True)
    a, b = wl.make_gemm_inputs(g["seed"], M, N, K)
    c = run_gemm_splitk(a, b, splits)
    assert bool(torch.isfinite(c.float()).all())
    rng = np.random.default_rng(g["seed"])
    rows = sorted({0, 1, 255, 256, M - 1, M // 2, *(int(r) for r in rng.integers(0, M, 16))} & set(range(M)))
    print(f"gemm split-K full size {name}: oracle on {len(rows)} rows", flush=True)
    print(check(c, a, b, f"gemm split-K {name}", rows=rows), flush=True)


# ---- second operand stored [K, N] ---------------------------------------------------------------------
def run_gemm_nn(a_bits, bkn_bits, poison=float("nan")):
    import paper_2605_10905_amd as A

    M, K = a_bits.shape
    N = bkn_bits.shape[1]
    a, b = gu.bf16_to_device(a_bits), gu.bf16_to_device(bkn_bits)
    c = torch.full((M, N), poison, dtype=torch.bfloat16, device="cuda")
    A.gemm_bf16_nn(a, b, c, M, N, K)
    torch.cuda.synchronize()
    return c


@pytest.mark.parametrize("M,N,K", [(256, 256, 256), (300, 520, 96), (1, 8, 32), (257, 264, 1024), (1000, 72, 64), (33, 1000, 2048),
                                   (777, 512, 160), (5, 8, 64), (2048, 2048, 512), (4096, 4352, 128)])
def test_gemm_nn_shapes(M, N, K):
    a, b = wl.make_gemm_inputs(700 + M + N + K, M, N, K)
    bkn = np.ascontiguousarray(b.T)           # the same matrix stored [K, N]
    print(f"gemm nn {M}x{N}x{K}", flush=True)
    c = run_gemm_nn(a, bkn)
    check(c, a, b, f"gemm nn {M}x{N}x{K}")   # the oracle on the [N, K] copy: same product
    # and the oracle's own [K, N] path agrees with it
    ref = og.gemm_ref(og.bf16_bits_to_f64(a), og.bf16_bits_to_f64(bkn), b_is_kn=True)
    assert og.error_metrics(c.float().cpu().numpy().astype(np.float64), ref)["rel_fro"] <= 3e-3


def test_gemm_nn_structured_and_unsupported():
    import paper_2605_10905_amd as A

    M, N, K = 384, 320, 128
    rng = np.random.default_rng(4)
    a = rng.standard_normal((M, K)).astype(np.float32)
    bkn = np.zeros((K, N), dtype=np.float32)
    rows = rng.integers(0, K, N)
    bkn[rows, np.arange(N)] = 1.0              # column n of B selects column rows[n] of A
    ab = wl.f32_to_bf16_bits(a)
    c = run_gemm_nn(ab, wl.f32_to_bf16_bits(bkn))
    want = torch.from_numpy(ab.view(np.int16)).view(torch.bfloat16)[:, torch.from_numpy(rows)]
    assert torch.equal(c.cpu().view(torch.int16), want.contiguous().view(torch.int16))
    t = torch.zeros(64 * 64, dtype=torch.bfloat16, device="cuda")
    assert A.gemm_bf16_nn(t, t, t, 64, 60, 32, check=False) != 0   # N not a multiple of 8
    assert A.gemm_bf16_nn(t, t, t, 64, 64, 24, check=False) != 0   # K not a multiple of 32


def test_gemm_calls_can_be_captured_in_a_graph_and_replayed():
    """gemm_bf16_nt, gemm_bf16_nn and gemm_bf16_nt_splitk (two kernels) captured into one graph; every
    replay, with eager work in between, must reproduce the eager results bit for bit."""
    import paper_2605_10905_amd as A

    M, N, K = 520, 392, 4096
    ab, bb = wl.make_gemm_inputs(77, M, N, K)
    a, b = gu.bf16_to_device(ab), gu.bf16_to_device(bb)
    bkn = b.t().contiguous()
    splits = 5

    def buffers():
        return dict(c=torch.zeros((M, N), dtype=torch.bfloat16, device="cuda"),
                    cn=torch.zeros((M, N), dtype=torch.bfloat16, device="cuda"),
                    cs=torch.zeros((M, N), dtype=torch.bfloat16, device="cuda"),
                    ws=torch.zeros(A.gemm_splitk_workspace_bytes(M, N, splits) // 4, dtype=torch.float32, device="cuda"))

    def run(t):
        A.gemm_bf16_nt(a, b, t["c"], M, N, K)
        A.gemm_bf16_nn(a, bkn, t["cn"], M, N, K)
        A.gemm_bf16_nt_splitk(a, b, t["cs"], M, N, K, splits, t["ws"])

    eager = buffers()
    run(eager)
    torch.cuda.synchronize()
    check(eager["c"], ab, bb, "eager nt")
    check(eager["cn"], ab, bb, "eager nn")
    check(eager["cs"], ab, bb, "eager split-K")

    cap = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(cap)  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run(cap)
    for rep in range(3):
        for name in ("c", "cn", "cs", "ws"):
            cap[name].fill_(7.0)  # eager work between the replays; also proves the replay rewrites everything
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in ("c", "cn", "cs"):
            assert torch.equal(cap[name].view(torch.uint8), eager[name].view(torch.uint8)), f"replay {rep}: {name} differs"


def _random_gemm_shapes(seed, count):
    rng = np.random.default_rng(seed)
    return [(int(rng.integers(1, 900)), int(rng.integers(1, 900)), 32 * int(rng.integers(1, 40))) for _ in range(count)]


@pytest.mark.parametrize("M,N,K", _random_gemm_shapes(20260513, 12))
def test_gemm_random_shapes(M, N, K):
    """Seeded random shapes: the library's choice, the [K, N] layout where it applies, split-K where K allows."""
    a, b = wl.make_gemm_inputs(900 + M + N + K, M, N, K)
    print(f"gemm random {M}x{N}x{K}", flush=True)
    check(run_gemm(a, b), a, b, f"gemm random {M}x{N}x{K}")
    if N % 8 == 0:
        bkn = np.ascontiguousarray(b.T)
        c = run_gemm_nn(a, bkn)
        check(c, a, b, f"gemm nn random {M}x{N}x{K}")
    if K % 64 == 0:
        check(run_gemm_splitk(a, b, 3), a, b, f"gemm split-K random {M}x{N}x{K}")
