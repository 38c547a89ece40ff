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


# Host-side sanitizers (the argument checks and launch logic of the C ABI; GPU code is not
# instrumented): every -fsanitize= goes to the host pass only.
LIB_HOSTSAN = os.path.join(HERE, "libta_hostsan.so")
HOSTSAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                 "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def _compile(src, extra=(), suffix=".o"):
    obj = os.path.join(CSRC, src.replace(".hip", suffix))
    subprocess.run([HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj], check=True)
    return obj


def build_lib(verbose=False, host_sanitizers=False):
    """Compile every source and link libta.so next to this file (host_sanitizers: libta_hostsan.so,
    the same code with AddressSanitizer and UndefinedBehaviorSanitizer in the host pass)."""
    extra, suffix, lib = ((HOSTSAN_FLAGS, ".san.o", LIB_HOSTSAN) if host_sanitizers else ((), ".o", LIB))
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra, suffix), SOURCES))
    link = ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"] if host_sanitizers else []
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *link, "-o", lib, *objs], check=True)
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    import sys
    build_lib(verbose=True, host_sanitizers="--host-sanitizers" in sys.argv)
