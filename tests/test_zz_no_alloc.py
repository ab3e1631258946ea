"""The backward entry point that allocates nothing (attn_bwd_noalloc: workspace in the library's
own device array) against attn_bwd with a caller-owned workspace: same bytes, on two calls in a
row of which the second is smaller, and within the gradient tolerances of the float64 oracle."""
import numpy as np
import pytest
import torch

import workloads as wl
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _run_both(ci, B, Hq, Hkv, N):
    import paper_2605_10905_amd as A

    cfg = dict(wl.CONFIGS[ci])
    inp = wl.make_inputs(cfg, B=B, Hq=Hq, Hkv=Hkv, N=N)
    dob = wl.make_dout(cfg, B=B, Hq=Hq, N=N)
    dev = gu.to_device(inp)
    d = inp["d"]
    print(f"no-alloc backward: config{ci + 1} B={B} Hq={Hq} Hkv={Hkv} N={N} causal={cfg['causal']}", flush=True)
    dq, dk, dv, o, lse = gu.run_gpu_bwd(inp, dob, dev)  # attn_fwd, then attn_bwd with a torch-owned workspace
    do = gu.bf16_to_device(dob)
    nan = float("nan")
    dq2 = torch.full((B, Hq, N, d), nan, dtype=torch.bfloat16, device="cuda")
    dk2 = torch.full((B, Hkv, N, d), nan, dtype=torch.bfloat16, device="cuda")
    dv2 = torch.full((B, Hkv, N, d), nan, dtype=torch.bfloat16, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    A.attn_bwd_noalloc(dev["q"], dev["k"], dev["v"], o, do, lse, dq2, dk2, dv2, B, Hq, Hkv, N, d, inp["causal"], inp["scale"],
                       A.ATTN_BF16)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for nm, x, y in (("dq", dq, dq2), ("dk", dk, dk2), ("dv", dv, dv2)):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16)), f"{nm} differs from attn_bwd"
    return inp, dob, dq2, dk2, dv2


def test_noalloc_backward_matches_attn_bwd_on_two_calls_in_a_row():
    # the first call fills a large part of the scratch array, the second (smaller, other mask,
    # ragged length, grouped heads) runs on top of what the first one left there
    big = _run_both(2, 1, 4, 4, 2048)
    small = _run_both(3, 2, 8, 2, 777)
    for inp, dob, dq, dk, dv in (big, small):
        print(gu.check_bwd_full(inp, dob, dq, dk, dv, "no-alloc backward"), flush=True)


def test_noalloc_backward_refuses_sizes_beyond_its_scratch():
    import paper_2605_10905_amd as A

    t = torch.zeros(16, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(16, dtype=torch.float32, device="cuda")
    # 4 * 64 * 16448 padded rows need more than the 32 MiB array; refused before any launch
    st = A.attn_bwd_noalloc(t, t, t, t, t, lse, t, t, t, 4, 64, 64, 16385, 128, 0, 0.1, A.ATTN_BF16, check=False)
    assert st == 6 and "scratch" in A.attn_status_string(st)
