"""Builds the HIP library in-tree: paper_2306_09782_amd/lib/liblomo.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
LIB_PATH = os.path.join(LIB_DIR, "liblomo.so")
SOURCES = ["lomo_api.hip", "lomo_gemm.hip", "lomo_gemm_fast.hip", "lomo_gemm_dma.hip", "lomo_gram.hip", "lomo_chain.hip", "lomo_attention.hip", "lomo_attention_fwd.hip", "lomo_forward.hip", "lomo_rowops.hip", "lomo_timing.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
    # packed fp32 VALU ops are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
]


def build(verbose: bool = True, extra_flags=(), out_path: str = LIB_PATH) -> str:
    os.makedirs(os.path.dirname(out_path), exist_ok=True)
    cmd = [HIPCC, *FLAGS, *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", out_path]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        sys.stdout.write(res.stdout)
        sys.stderr.write("\n".join(ln for ln in res.stderr.splitlines()
                                   if "packed-fp32-ops" not in ln and "is not a recognized feature" not in ln) + "\n")
    if res.returncode != 0:
        raise RuntimeError("hipcc failed")
    return out_path


def build_synth(verbose: bool = True) -> str:
    """The input-generator kernel of lomo_synth (not part of the product library)."""
    src = os.path.join(ROOT, "lomo_synth", "csrc", "synth_gen.hip")
    out = os.path.join(ROOT, "lomo_synth", "lib", "libsynthgen.so")
    os.makedirs(os.path.dirname(out), exist_ok=True)
    cmd = [HIPCC, *FLAGS, src, "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stderr)
        raise RuntimeError("hipcc failed (synth generator)")
    return out


if __name__ == "__main__":
    build()
    build_synth()
