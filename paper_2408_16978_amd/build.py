"""Build libfpdt.so (HIP kernels + C ABI) and libfpdt_tokenwise.so for gfx950, in-tree.

    python -m paper_2408_16978_amd.build

Each .hip file is compiled to an object under _build/ (in parallel) and linked into
paper_2408_16978_amd/libfpdt.so.  hipcc cross-compiles without a GPU.
"""
import concurrent.futures
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
SRC_DIR = os.path.join(PKG, "csrc")
BUILD_DIR = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libfpdt.so")
SOURCES = ["api.hip", "pack.hip", "fwd_bf16.hip", "bwd_bf16.hip", "f32_path.hip", "calibrate.hip"]
# token-wise chunked neighbours (projection, feed-forward block, loss): a library of their own
TW_LIB = os.path.join(PKG, "libfpdt_tokenwise.so")
TW_SOURCES = ["tokenwise.hip", "tw_gemm.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# -packed-fp32-ops off: packed fp32 VALU forms are kept out of the generated code.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option"]


def _compile(name: str) -> str:
    obj = os.path.join(BUILD_DIR, name.replace(".hip", ".o"))
    cmd = [HIPCC] + FLAGS + ["-c", os.path.join(SRC_DIR, name), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (name, r.stderr))
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(BUILD_DIR, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + len(TW_SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES + TW_SOURCES))
    tw_objs = objs[len(SOURCES):]
    objs = objs[:len(SOURCES)]
    for lib, o, extra in ((LIB, objs, []), (TW_LIB, tw_objs, [])):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + o + extra
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n%s" % r.stderr)
        if verbose:
            print("built", lib)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    sys.exit(0)
