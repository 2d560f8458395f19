"""Builds the HIP library in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libastra_hip.so")

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wno-unused-command-line-argument"]
# Keeps MFMA accumulators in ordinary vector registers (no copies between the two register files around the
# softmax / argmin arithmetic).  Not for the GEMM: its 256x256 tile on four wavefronts holds 256 accumulator
# registers per lane, which only fit next to the operands when they live in the accumulation registers.
VGPR_FORM_FLAGS = ["-mllvm", "-amdgpu-mfma-vgpr-form"]
ACC_REGISTER_FILES = ("gemm_kernels.hip", "gemm_mlp_kernels.hip", "vq_encode_wide_kernels.hip")


def build(verbose: bool = False) -> str:
    """Compile every csrc/*.hip and link libastra_hip.so next to this file."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    objdir = os.path.join(_HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(objdir, os.path.basename(src)[:-4] + ".o")
        extra = [] if os.path.basename(src) in ACC_REGISTER_FILES else VGPR_FORM_FLAGS
        cmd = [hipcc, *HIPCC_FLAGS, *extra, "-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
        if verbose and r.stderr.strip():
            print(r.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, srcs))
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
