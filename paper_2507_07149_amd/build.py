"""Build libdaf.so (HIP, gfx950 only) in-tree next to this file.

    python -m paper_2507_07149_amd.build

hipcc cross-compiles without a GPU.  Flags that matter:
  -ffp-contract=off      every float operation rounds once (fused multiply-add only where written)
  -fno-strict-aliasing   LDS staging is written as bytes/halfwords and read back as words
  -target-feature -packed-fp32-ops   no packed-FP32 instructions
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdaf.so")
SOURCES = ["daf_api.hip", "plan_scan.hip", "quantize_pack.hip", "unpack_dequantize.hip", "minmax.hip",
           "select_bits.hip", "unpack_matmul.hip", "page_store.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fno-strict-aliasing",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
HOST_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-Wall", "-Wextra", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    flags = HOST_FLAGS if src.endswith(".cpp") else FLAGS        # .cpp = host-only code
    r = subprocess.run([HIPCC, *flags, "-c", os.path.join(CSRC, src), "-o", obj],
                       stderr=subprocess.PIPE, text=True)
    # the host pass warns that it does not know the packed-fp32 target feature: harmless
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build() -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    print(build())
