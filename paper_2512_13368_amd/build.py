"""Builds libblossom.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libblossom.so")
OBJ_DIR = os.path.join(HERE, "_build")

# per-file extra flags; select.hip decides integers from fp32 arithmetic and must not be
# contracted into fused operations the source does not spell out
SOURCES = {
    "api.hip": [],
    "select.hip": ["-ffp-contract=off"],
    "select_pos.hip": ["-ffp-contract=off"],
    "generic.hip": [],
    # accumulators of the matrix instructions stay in VGPRs: the online softmax rescales them
    # with VALU instructions, and AGPR placement costs a register copy per element per tile
    # (the forward kernel also reuses its bf16 staging rows as fp32 exchange space between wavefronts)
    "mfma_fwd.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1", "-fno-strict-aliasing"],
    "mfma_fwd4.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1", "-fno-strict-aliasing"],
    "mfma_f32.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
    "mfma_bwd.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
    "probe.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
    "out_proj.hip": ["-fno-strict-aliasing"],
}

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for c in ("/opt/rocm/bin/hipcc", "hipcc"):
        if os.path.isabs(c) and not os.path.exists(c):
            continue
        return c
    return "hipcc"


def build_library(verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(item):
        src, extra = item
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        cmd = [hipcc, *COMMON, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
        if verbose and r.stderr.strip():
            print(r.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES.items()))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
