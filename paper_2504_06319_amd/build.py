"""Build libkvprefetch.so in-tree with hipcc for gfx950."""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libkvprefetch.so")
OBJ_DIR = os.path.join(PKG, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]
# keep MFMA accumulators in ordinary VGPRs (no AGPR copies around the softmax rescale)
VGPR_FORM = ["-mllvm", "-amdgpu-mfma-vgpr-form"]
# per-file additions; the operand-packed dense layer wants its 128 accumulator registers in AGPRs, so that the
# 256 architectural VGPRs are free for the weights it keeps in flight
FILE_FLAGS = {"layer_gemm_packed.hip": []}


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    noise = "is not a recognized feature for this target"

    def run(cmd):
        proc = subprocess.run(cmd, capture_output=True, text=True)
        out = "\n".join(l for l in (proc.stdout + proc.stderr).splitlines() if noise not in l)
        if proc.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + out)
        return out

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
        extra = FILE_FLAGS.get(os.path.basename(src), VGPR_FORM)
        return obj, run([hipcc, *HIPCC_FLAGS, *extra, "-c", "-o", obj, src])

    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(compile_one, sources()))
    log = "\n".join(r[1] for r in results if r[1].strip())
    log += run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", LIB, *[r[0] for r in results]])
    if verbose and log.strip():
        print(log, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
