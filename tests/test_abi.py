"""CPU-side checks of the boundary: the library loads, exports every symbol the
header declares, rejects bad arguments before touching a device, and its work
decomposition is a bijection that keeps K/V sharers on one XCD."""
import ctypes
import os

import numpy as np
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def A():
    import paper_2605_10905_amd as A

    return A


def header_functions():
    names = set()
    for h in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names.update(re.findall(r"\b((?:attn|gemm)_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(A):
    names = header_functions()
    assert "attn_fwd" in names and "attn_fwd_fp8" in names and len(names) >= 9
    for n in names:
        assert hasattr(A.lib, n), f"{n} declared in include/attn.h but not exported"


def test_header_compiles_as_c():
    import subprocess
    import tempfile

    with tempfile.TemporaryDirectory() as td:
        src = os.path.join(td, "t.c")
        open(src, "w").write('#include "attn.h"\n#include "gemm.h"\nint main(void){return attn_version() == 0;}\n')
        subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), "-c", src,
                        "-o", os.path.join(td, "t.o")], check=True)


def test_status_strings_and_version(A):
    assert A.attn_version() >= 1
    assert A.attn_status_string(0) == "ok"
    assert len({A.attn_status_string(i) for i in range(6)}) == 6
    assert A.attn_num_variants() >= 1
    assert A.attn_variant_name(-1) is None and A.attn_variant_name(10 ** 6) is None
    assert all(A.attn_variant_bm(i) % 32 == 0 for i in range(A.attn_num_variants()))


def test_argument_validation_without_a_device(A):
    # (fake, never dereferenced) aligned addresses; every call must fail before any launch
    p = 0x1000
    ok = dict(B=1, Hq=2, Hkv=1, N=8, d=64)

    def call(q=p, k=p, v=p, o=p, lse=p, causal=0, scale=0.5, dtype=0, **kw):
        a = dict(ok, **kw)
        return A.attn_fwd(q, k, v, o, lse, a["B"], a["Hq"], a["Hkv"], a["N"], a["d"], causal, scale, dtype, stream=0,
                          check=False)

    assert call(q=None) == 1 and call(lse=None) == 1 and call(o=None) == 1
    assert call(B=0) == 2 and call(N=-1) == 2 and call(Hq=3, Hkv=2) == 2
    assert call(q=p + 8) == 2 and call(lse=p + 2) == 2
    assert call(dtype=7) == 3
    assert call(d=96) == 4 and call(d=256) == 4
    assert call(scale=0.0) == 4 and call(scale=-1.0) == 4
    with pytest.raises(A.AttnError):
        A.attn_fwd(None, p, p, p, p, 1, 1, 1, 8, 64, 0, 1.0, 0, stream=0)
    assert A.attn_fwd_variant(p, p, p, p, p, 1, 1, 1, 8, 64, 0, 1.0, 0, 10 ** 6, stream=0, check=False) == 4
    assert A.attn_fwd_fp8(p, p, p, p, p, 1, 1, 1, 8, 128, 0, 1.0, -1.0, 1.0, 1.0, stream=0, check=False) == 4
    # what include/attn.h states: scale must be positive; fp8 inputs exist for head dimension 128 only
    assert A.attn_fwd(p, p, p, p, p, 1, 1, 1, 8, 64, 0, 0.0, 0, stream=0, check=False) == 4
    assert A.attn_fwd(p, p, p, p, p, 1, 1, 1, 8, 64, 0, -1.0, 0, stream=0, check=False) == 4
    assert A.attn_fwd(p, p, p, p, p, 1, 1, 1, 8, 64, 0, 1.0, 1, stream=0, check=False) == 4
    assert A.attn_fwd_fp8(p, p, p, p, p, 1, 1, 1, 8, 64, 0, 1.0, 1.0, 1.0, 1.0, stream=0, check=False) == 4
    assert A.attn_fwd(p, p, p, p, p, 1, 1, 1, 8, 96, 0, 1.0, 0, stream=0, check=False) == 4


@pytest.mark.parametrize("B,Hq,Hkv,N,BM,causal", [
    (2, 32, 32, 8192, 256, 0), (4, 64, 8, 4096, 256, 1), (4, 16, 16, 2048, 256, 1), (1, 2, 2, 256, 128, 0),
    (3, 6, 2, 1000, 128, 1), (1, 1, 1, 1, 256, 0), (4, 48, 48, 1024, 256, 1), (4, 48, 48, 2048, 256, 1), (4, 48, 48, 16384, 256, 1),
    (5, 7, 7, 700, 256, 1), (2, 24, 4, 1300, 256, 1),
])
def test_tile_map_is_a_bijection_and_xcd_local(A, B, Hq, Hkv, N, BM, causal):
    n = A.attn_num_workgroups(B, Hq, N, BM)
    T = (N + BM - 1) // BM
    assert n == B * Hq * T
    seen = set()
    xcd_of_kv = {}
    G = Hq // Hkv
    first_t_of_head = {}
    for wg in range(n):
        b, h, t = A.attn_tile_coord(wg, B, Hq, Hkv, N, BM, causal)
        assert 0 <= b < B and 0 <= h < Hq and 0 <= t < T
        seen.add((b, h, t))
        if (B * Hkv) % 8 == 0:
            xcd_of_kv.setdefault((b, h // G), set()).add(wg % 8)
        first_t_of_head.setdefault((b, h), t)
    assert len(seen) == n
    for s in xcd_of_kv.values():
        assert len(s) == 1  # all workgroups that share a K/V head run on one XCD
    if causal:
        assert all(t == T - 1 for t in first_t_of_head.values())  # heaviest tile first
    with pytest.raises(A.AttnError):
        A.attn_tile_coord(n, B, Hq, Hkv, N, BM, causal)


def _tile_coord_by_plain_division(wg, B, Hq, Hkv, T, causal, batch_wgs=64):
    """The tile order written with Python's integer division (the library divides by the launch's
    constants with a multiply-high and one correction)."""
    G, groups, W = Hq // Hkv, B * Hkv, (Hq // Hkv) * T
    lists = 8 if groups % 8 == 0 else 1
    xcd, s = (wg % 8, wg // 8) if lists == 8 else (0, wg)
    if causal:
        gx = groups // lists
        pb = min((batch_wgs * (8 // lists) + W - 1) // W, gx)
        batch, r = divmod(s, pb * W)
        nb = min(gx - batch * pb, pb)
        tt, rem = divmod(r, nb * G)
        gl, hg = batch * pb + rem // G, rem % G
    else:
        gl, inner = divmod(s, W)
        tt, hg = divmod(inner, G)
    group = gl * lists + xcd
    return group // Hkv, (group % Hkv) * G + hg, (T - 1 - tt) if causal else tt


def test_tile_map_equals_its_definition_by_plain_division(A):
    rng = np.random.default_rng(77)
    shapes = [(1, 1, 1, 1), (2, 32, 32, 8192), (4, 64, 8, 4096), (3, 5, 5, 13100), (1, 12, 4, 16450), (7, 3, 1, 300), (8, 9, 3, 2000),
              (5, 16, 2, 70000), (16, 1, 1, 257)]
    shapes += [(int(rng.integers(1, 9)), int(g * k), int(k), int(rng.integers(1, 40000)))
               for g, k in zip(rng.integers(1, 9, 12), rng.integers(1, 9, 12))]
    for B, Hq, Hkv, N in shapes:
        T = (N + 255) // 256
        n = A.attn_num_workgroups(B, Hq, N, 256)
        ids = set(range(min(n, 300))) | set(range(max(0, n - 300), n)) | {int(x) for x in rng.integers(0, n, 400)}
        for causal in (False, True):
            for wg in ids:
                assert tuple(A.attn_tile_coord(wg, B, Hq, Hkv, N, 256, causal)) == _tile_coord_by_plain_division(wg, B, Hq, Hkv, T, causal), \
                    (wg, B, Hq, Hkv, N, causal)


def test_no_product_code_imports_the_oracle():
    for dirpath, _, files in os.walk(os.path.join(ROOT, "paper_2605_10905_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "from oracle" not in text and "import oracle" not in text


@pytest.mark.parametrize("M,N,tile", [(8192, 8192, 256), (2048, 2048, 128), (300, 5000, 64), (256, 256, 256), (1000, 777, 128),
                                      (2304, 1024, 256)])
def test_gemm_tile_map_is_a_bijection(A, M, N, tile):
    n = A.gemm_num_workgroups(M, N, tile)
    tm_n, tn_n = -(-M // tile), -(-N // tile)
    assert n == tm_n * tn_n
    seen = {A.gemm_tile_coord(wg, M, N, tile) for wg in range(n)}
    assert seen == {(i, j) for i in range(tm_n) for j in range(tn_n)}
    with pytest.raises(A.AttnError):
        A.gemm_tile_coord(n, M, N, tile)


def test_gemm_tile_map_keeps_an_xcd_on_few_rows(A):
    """The 128 tiles an XCD owns of an 8192 x 8192 output (256-wide tiles) lie in one band of 4 tile rows."""
    rows = {}
    for wg in range(A.gemm_num_workgroups(8192, 8192, 256)):
        tm, _ = A.gemm_tile_coord(wg, 8192, 8192, 256)
        rows.setdefault(wg % 8, set()).add(tm)
    assert all(len(r) == 4 for r in rows.values())


def test_gemm_argument_validation_without_a_device(A):
    p = 0x1000
    assert A.gemm_bf16_nt(p, p, p, 64, 64, 48, stream=0, check=False) == 4
    assert A.gemm_bf16_nt(None, p, p, 64, 64, 64, stream=0, check=False) == 1
    assert A.gemm_bf16_nt(p, p, p, 64, -1, 64, stream=0, check=False) == 2
    assert A.gemm_bf16_nt(p + 2, p, p, 64, 64, 64, stream=0, check=False) == 2
    assert A.gemm_bf16_nt_variant(p, p, p, 64, 64, 64, 10 ** 6, stream=0, check=False) == 4
    assert A.gemm_variant_tile(0) == 256 and A.gemm_variant_tile(-1) == 0


def test_gemm_splitk_plan_and_validation_without_a_device(A):
    p = 0x1000
    assert A.gemm_bf16_nt_splitk(p, p, p, 64, 64, 96, 2, p, stream=0, check=False) == 4   # K % 64
    assert A.gemm_bf16_nt_splitk(p, p, p, 64, 64, 64, 0, p, stream=0, check=False) == 2
    assert A.gemm_bf16_nt_splitk(p, p, p, 64, 64, 64, 65, p, stream=0, check=False) == 2
    assert A.gemm_bf16_nt_splitk(p, p, p, 64, 64, 64, 2, None, stream=0, check=False) == 1
    assert A.gemm_bf16_nt_splitk(p, p, p, 64, 64, 64, 2, p + 4, stream=0, check=False) == 2
    assert A.gemm_splitk_workspace_bytes(512, 4096, 8) == 8 * 512 * 4096 * 4
    assert A.gemm_splitk_workspace_bytes(0, 4096, 8) == 0
    # the paper's large-K shapes get slices that fill the 256 CUs, the others none
    assert A.gemm_splitk_plan(512, 4096, 64512) == 8
    assert A.gemm_splitk_plan(2304, 1024, 65536) == 7
    assert A.gemm_splitk_plan(8192, 8192, 8192) == 1
    assert A.gemm_splitk_plan(2048, 2048, 2048) == 1      # too little k per slice
    assert A.gemm_splitk_plan(512, 512, 8200) == 1        # K not a multiple of 64
    for M, N, K in [(512, 4096, 64512), (256, 256, 1 << 20), (1, 1, 4096), (2304, 1024, 65536)]:
        s = A.gemm_splitk_plan(M, N, K)
        tiles = -(-M // 256) * -(-N // 256)
        assert 1 <= s <= 64 and (s == 1 or (tiles * s <= 256 and K // s >= 2048))


def test_backward_and_persistent_validation_without_a_device(A):
    p = 0x1000

    def bwd(q=p, ws=p, d=128, dtype=0, N=8, Hq=2, Hkv=1):
        return A.attn_bwd(q, p, p, p, p, p, p, p, p, ws, 1, Hq, Hkv, N, d, 0, 0.5, dtype, stream=0, check=False)

    assert bwd(q=None) == 1 and bwd(ws=None) == 1
    assert bwd(N=0) == 2 and bwd(Hq=3, Hkv=2) == 2 and bwd(ws=p + 4) == 2
    assert bwd(d=96) == 4 and bwd(d=256) == 4  # the backward covers head dimensions 128 and 64
    assert bwd(dtype=1) in (3, 4)              # and bf16 only
    assert A.attn_bwd_workspace_bytes(2, 32, 8192) == 2 * 32 * 2 * 8192 * 4
    assert A.attn_bwd_workspace_bytes(1, 1, 1) == 2 * 64 * 4 and A.attn_bwd_workspace_bytes(0, 1, 1) == 0

    # the entry point without a workspace argument: same checks, and sizes beyond its built-in
    # scratch memory are refused before anything touches a device
    def bwd_na(q=p, d=128, dtype=0, N=8, Hq=2, Hkv=1, B=1):
        return A.attn_bwd_noalloc(q, p, p, p, p, p, p, p, p, B, Hq, Hkv, N, d, 0, 0.5, dtype, stream=0, check=False)

    assert bwd_na(q=None) == 1 and bwd_na(N=0) == 2 and bwd_na(Hq=3, Hkv=2) == 2 and bwd_na(d=96) == 4
    cap = A.attn_bwd_noalloc_max_workspace_bytes()
    assert cap == 32 << 20
    assert A.attn_bwd_workspace_bytes(4, 64, 16384) == cap and A.attn_bwd_workspace_bytes(4, 64, 16385) > cap
    assert bwd_na(B=4, Hq=64, Hkv=64, N=16385) == 6
    assert "scratch" in A.attn_status_string(6)

    def pers(queue=p, dtype=0, d=128):
        return A.attn_fwd_persistent(p, p, p, p, p, 1, 2, 1, 8, d, 0, 0.5, dtype, queue, stream=0, check=False)

    assert pers(queue=None) == 1 and pers(queue=p + 64) == 2
    assert pers(dtype=1) == 4 and pers(d=96) == 4
    assert A.attn_persistent_queue_bytes() == 1024


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys

    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "--gpus" in r.stderr and r.stdout.strip() == ""
