"""Build libtfx.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

Usage: python -m paper_1901_05350_amd.build [--force]
"""
import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtfx.so")
SOURCES = ["api.hip", "gemm.hip", "pointwise.hip", "conv.hip", "depthwise.hip", "tail.hip", "elementwise.hip", "gemm_f16.hip", "conv_f16.hip", "pointwise_f16.hip", "pointwise_slab_f16.hip", "conv_gemm_f16.hip", "conv_stream_f16.hip", "chain.hip", "block.hip", "block_stream.hip", "block_stream_f16.hip"]
HEADERS = [os.path.join(CSRC, "tfx_internal.h"), os.path.join(CSRC, "stream_f16.h"), os.path.join(HERE, "..", "include", "tfx.h")]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed fp32 VALU ops are kept off on this target
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc():
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(src, force):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    path = os.path.join(CSRC, src)
    if force or _stale(obj, [path] + HEADERS):
        subprocess.run([_hipcc()] + FLAGS + ["-c", path, "-o", obj], check=True)
    return obj


def build(force=False, verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or _stale(LIB, objs):
        subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, check=True)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(force="--force" in sys.argv, verbose=True)
