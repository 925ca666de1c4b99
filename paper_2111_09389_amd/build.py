"""Builds liblpdt.so (HIP, gfx950 only) in-tree, next to the sources."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblpdt.so")
SOURCES = ["common.cpp", "quantize.hip", "range_evonorm.hip", "ref_norms.hip", "gossip.hip", "glue.hip", "qconv.hip", "qconv_igemm.hip", "qconv_igemm_dma.hip", "qconv_patch.hip", "qconv_narrow.hip", "qconv_wgrad.hip", "qconv_wgrad_rows.hip", "qconv_wgrad_gemm.hip", "qconv_wgrad_bf16.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed-fp32 VALU forms are kept out of the generated code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# The quantizer's rounding decisions are defined as single IEEE operations (multiply, then
# subtract): fusing them into an FMA changes codes at the 1e-6 level, so contraction is off there.
EXTRA = {"quantize.hip": ["-ffp-contract=off"]}


def _compile(src):
    obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj] + FLAGS + EXTRA.get(src, [])
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose=True):
    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build()
