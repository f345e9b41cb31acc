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
# (source, object name, extra flags): quantize_pack.hip is built once per element format
SOURCES = [("quantize_pack.hip", "quantize_pack_f32", ["-DDAF_DT=0"]),
           ("quantize_pack.hip", "quantize_pack_f16", ["-DDAF_DT=1"]),
           ("quantize_pack.hip", "quantize_pack_bf16", ["-DDAF_DT=2"]),
           ("daf_api.hip", "daf_api", []), ("quantize_dispatch.hip", "quantize_dispatch", []),
           ("plan_scan.hip", "plan_scan", []), ("unpack_dequantize.hip", "unpack_dequantize", []),
           ("minmax.hip", "minmax", []), ("select_bits.hip", "select_bits", []),
           ("unpack_matmul.hip", "unpack_matmul", []), ("linear_quantize.hip", "linear_quantize", []),
           ("page_store.cpp", "page_store", [])]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-ffp-contract=off", "-fno-strict-aliasing",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
HOST_FLAGS = ["-O2", "-std=c++17", "-fPIC", "-Wall", "-Wextra", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _compile(item) -> str:
    src, name, extra = item
    obj = os.path.join(OBJ, name + ".o")
    flags = HOST_FLAGS if src.endswith(".cpp") else FLAGS        # .cpp = host-only code
    r = subprocess.run([HIPCC, *flags, *extra, "-c", os.path.join(CSRC, src), "-o", obj],
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
