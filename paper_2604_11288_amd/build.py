"""Builds libta.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libta.so")
SOURCES = ["ta_api.hip", "ta_match.hip", "ta_score.hip", "ta_select.hip", "ta_compact.hip", "ta_decode.hip",
           "ta_detect.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# -ffp-contract=off: the utility, voucher and ranking arithmetic is specified operation by
# operation in fp32 (the rounded-operation intrinsics of the HIP headers are plain * and +, which
# the default contraction mode may fuse into an FMA and so change the last bit); the kernels that
# want fused multiply-adds call fmaf explicitly.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # MFMA accumulators in VGPRs: the softmax reads them with plain VALU ops
         "-mllvm", "-amdgpu-mfma-vgpr-form"]


def _compile(src):
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    subprocess.run([HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj], check=True)
    return obj


def build_lib(verbose=False):
    """Compile every source and link libta.so next to this file."""
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build_lib(verbose=True)
