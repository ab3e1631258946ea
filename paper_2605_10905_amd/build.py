"""Builds the HIP library in-tree (hipcc, gfx950 only).  `python -m paper_2605_10905_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libattn_mi355x.so")
SOURCES = ["attn_api.hip", "attn_fwd_bf16.hip", "attn_fwd_bf16_pp.hip", "attn_fwd_bf16_sp.hip", "attn_fwd_bf16_w16.hip", "attn_fwd_bf16_q64.hip", "attn_fwd_fp8.hip", "attn_fwd_fp8_sp.hip", "attn_fwd_fp8_cv.hip", "attn_fwd_fp8_hy.hip", "attn_bwd_bf16.hip", "gemm_api.hip", "gemm_bf16.hip", "mfma_probe.hip"]
# sources with MFMAs written as inline assembly: their generated assembly is checked for the wait
# states the compiler cannot know about (mfma_lint.py)
LINTED = ["attn_fwd_bf16_q64.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed fp32 VALU forms are switched off on purpose (they have misbehaved on the test machines)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Wno-inline-asm"]


def build(verbose: bool = True, extra_flags=()) -> str:
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [HIPCC, *FLAGS, *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    lint_procs = []
    for src in LINTED:
        asm = os.path.join(CSRC, src.replace(".hip", ".lint.s"))
        cmd = [HIPCC, *FLAGS, *extra_flags, "-S", "--cuda-device-only", os.path.join(CSRC, src), "-o", asm]
        lint_procs.append((asm, cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for cmd, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + out)
        if verbose and out.strip():
            print(out)
    from . import mfma_lint

    for asm, cmd, pr in lint_procs:
        out, _ = pr.communicate()
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + out)
        with open(asm) as f:
            bad = mfma_lint.lint(f.read())
        os.remove(asm)
        if bad:
            raise RuntimeError(f"{asm}: {len(bad)} instructions touch the result of an inline-assembly MFMA too early, first: "
                               f"line {bad[0][0]}: {bad[0][1].strip()}")
        if verbose:
            print(f"mfma_lint: {os.path.basename(asm)} clean", flush=True)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(extra_flags=sys.argv[1:])
