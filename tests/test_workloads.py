"""The seeded input generators: formats and determinism (no method arithmetic here)."""
import numpy as np
import torch

import workloads as wl
from oracle import attn_ref as orc


def test_bf16_rounding_matches_torch_rne():
    x = np.random.default_rng(3).standard_normal(100000).astype(np.float32) * 3
    # include exact ties: values halfway between two bf16 neighbours
    ties = (np.arange(1, 2001, dtype=np.uint32) << np.uint32(16) | np.uint32(0x8000)) + np.uint32(0x3F000000)
    x = np.concatenate([x, ties.view(np.float32)])
    ours = wl.f32_to_bf16_bits(x)
    t = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (ours == t).all()


def test_generators_are_seeded_and_shaped():
    cfg = wl.CONFIGS[0]
    a = wl.make_inputs(cfg)
    b = wl.make_inputs(cfg)
    for nm in "qkv":
        assert a[nm].dtype == np.uint16 and (a[nm] == b[nm]).all()
    assert a["q"].shape == (1, 2, 256, 64) and a["k"].shape == (1, 2, 256, 64)
    assert not (a["q"] == a["k"]).all()
    x = orc.bf16_bits_to_f64(a["q"])
    assert abs(x.std() - 1.0) < 0.02 and abs(x.mean()) < 0.02
    c3 = wl.make_inputs(wl.CONFIGS[2], B=1, Hq=2, Hkv=2, N=128)
    assert abs(orc.bf16_bits_to_f64(c3["v"]).std() - 0.5) < 0.02


def test_fp8_quantiser_roundtrip_and_scale():
    # every finite e4m3 value, scaled, must come back as its own code
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF, 0x80)], dtype=np.uint8)
    vals = orc.e4m3_bits_to_f64(codes)
    s = 0.0123
    q, scale = wl.quantise_e4m3((vals * s).astype(np.float32))
    assert abs(float(scale) - s) < 1e-8
    assert (q == codes).all()
    cfg = wl.CONFIGS[4]
    inp = wl.make_inputs(cfg, B=1, Hq=1, Hkv=1, N=512)
    assert inp["q"].dtype == np.uint8
    deq = orc.e4m3_bits_to_f64(inp["q"])
    assert np.isfinite(deq).all() and np.abs(deq).max() == 448.0
    assert abs(inp["descale"][0] * 448.0 - np.abs(wl.normal_f32(cfg["seed"], 0, (1, 1, 512, 128), 1.0)).max()) < 1e-4


def test_flop_counts_match_published_table():
    f = [wl.algorithmic_flops(c) for c in wl.CONFIGS]
    expect = [3.355e7, 6.872e10, 2.199e12, 1.0995e12, 4.398e12]
    for a, b in zip(f, expect):
        assert abs(a - b) / b < 1e-3
