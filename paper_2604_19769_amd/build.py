"""Build libttkv.so for gfx950 with hipcc (cross-compiles without a GPU)."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libttkv.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# ttkv_quant.hip must keep every fp32 step a single IEEE operation (bit-exact codes).
SOURCES = {
    "ttkv_api.hip": [],
    "ttkv_quant.hip": ["-ffp-contract=off"],
    "ttkv_attn.hip": [],
    "ttkv_attn_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],   # MFMA results feed vector code: keep them out of the AGPRs
    "ttkv_select.hip": ["-ffp-contract=off"],
    "ttkv_probe.hip": [],
}
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _compile(item):
    src, extra = item
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    subprocess.run([HIPCC, *COMMON, *extra, "-c", os.path.join(CSRC, src), "-o", obj], check=True)
    return obj


def build(verbose=False):
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, SOURCES.items()))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
