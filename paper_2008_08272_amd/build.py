"""Builds the HIP library in-tree: paper_2008_08272_amd/libonnxhip.so (gfx950 only)."""
import concurrent.futures
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libonnxhip.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SOURCES = ("api.hip", "contraction.hip", "conv_window.hip", "conv_window_lp.hip", "conv_stem_lp.hip", "conv_resident.hip", "window_kernels.hip", "window_lp.hip", "elementwise.hip", "gemm_lp.hip", "lp_generic.hip", "lp_layout.hip", "lstm.hip", "chain.hip")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src):
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    subprocess.check_call([HIPCC] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj])
    return obj


def build():
    """Compile every source (always) and link the shared library."""
    with concurrent.futures.ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    print(build())
