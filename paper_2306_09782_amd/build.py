"""Builds the HIP library in-tree: paper_2306_09782_amd/lib/liblomo.so (gfx950 only).

Every source is compiled to an object of its own (in parallel, device assembly kept next to it under
_build/), then linked.  The compiler's output is passed through unfiltered.  After compiling, the kept
device assembly is scanned for packed-fp32 arithmetic: the build fails if the device pass did not honour
the feature switch that turns those instructions off.
"""
from __future__ import annotations

import glob
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
LIB_PATH = os.path.join(LIB_DIR, "liblomo.so")
OBJ_DIR = os.path.join(ROOT, "_build", "lomo")
SOURCES = ["lomo_api.hip", "lomo_gemm.hip", "lomo_gemm_fast.hip", "lomo_gemm_dma.hip", "lomo_gram.hip", "lomo_chain.hip",
           "lomo_attention.hip", "lomo_attention_fwd.hip", "lomo_forward.hip", "lomo_rowops.hip", "lomo_timing.hip",
           "lomo_ceiling.hip", "lomo_static.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# Packed fp32 VALU arithmetic is kept off on the test machines.  -Xclang reaches both passes of a HIP
# compile; the host pass says it does not know the feature (harmless), the device pass obeys it, which
# check_no_packed_fp32() verifies on the assembly it produced.
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
    "-Wno-inline-asm",      # the direct-to-LDS loads set M0 inside inline assembly and say so in the clobber list
]
PACKED_FP32 = re.compile(r"\bv_pk_(add|mul|fma)_f32\b")
JOBS = max(1, min(8, int(os.environ.get("MAX_JOBS", "8")), os.cpu_count() or 1))


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    return cmd, res


def check_no_packed_fp32(obj_dir: str) -> int:
    """Scans the device assembly kept by -save-temps; returns the number of files read."""
    files = glob.glob(os.path.join(obj_dir, "*gfx950*.s"))
    if not files:
        raise RuntimeError(f"no device assembly under {obj_dir}: cannot verify the packed-fp32 switch")
    for f in files:
        with open(f) as fh:
            for n, line in enumerate(fh, 1):
                if PACKED_FP32.search(line):
                    raise RuntimeError(f"{f}:{n}: packed fp32 instruction in device code: {line.strip()}")
    return len(files)


def _compile_all(sources, obj_dir, extra_flags, includes, verbose):
    os.makedirs(obj_dir, exist_ok=True)
    for old in glob.glob(os.path.join(obj_dir, "*")):
        if os.path.isfile(old):
            os.remove(old)
    objs, cmds = [], []
    for src in sources:
        obj = os.path.join(obj_dir, os.path.splitext(os.path.basename(src))[0] + ".o")
        objs.append(obj)
        cmds.append([HIPCC, *FLAGS, *extra_flags, "-save-temps=obj", *includes, "-c", src, "-o", obj])
    with ThreadPoolExecutor(JOBS) as pool:
        results = list(pool.map(lambda c: _run(c, verbose), cmds))
    failed = False
    for cmd, res in results:
        if verbose or res.returncode != 0:
            sys.stdout.write(res.stdout)
            sys.stderr.write(res.stderr)
        failed |= res.returncode != 0
    if failed:
        raise RuntimeError("hipcc failed")
    n = check_no_packed_fp32(obj_dir)
    if verbose:
        print(f"device assembly of {n} sources holds no packed fp32 arithmetic", flush=True)
    return objs


def build(verbose: bool = True, extra_flags=(), out_path: str = LIB_PATH) -> str:
    os.makedirs(os.path.dirname(out_path), exist_ok=True)
    objs = _compile_all([os.path.join(CSRC, s) for s in SOURCES], OBJ_DIR, list(extra_flags),
                        ["-I", os.path.join(ROOT, "include"), "-I", CSRC], verbose)
    cmd, res = _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", *objs, "-o", out_path], verbose)
    sys.stdout.write(res.stdout)
    sys.stderr.write(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("link failed")
    return out_path


def build_synth(verbose: bool = True) -> str:
    """The input-generator kernel of lomo_synth (not part of the product library)."""
    src = os.path.join(ROOT, "lomo_synth", "csrc", "synth_gen.hip")
    out = os.path.join(ROOT, "lomo_synth", "lib", "libsynthgen.so")
    os.makedirs(os.path.dirname(out), exist_ok=True)
    objs = _compile_all([src], os.path.join(ROOT, "_build", "synth"), [], [], verbose)
    cmd, res = _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", *objs, "-o", out], verbose)
    sys.stderr.write(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("link failed (synth generator)")
    return out


if __name__ == "__main__":
    build()
    build_synth()
