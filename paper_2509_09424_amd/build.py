"""Builds libensi_hip.so (gfx950) in-tree with hipcc: one object per source, compiled in parallel, then linked."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libensi_hip.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["api.hip", "api_keys.hip", "api_static.hip", "ntt.hip", "ntt16.hip", "keyswitch16.hip", "pmult.hip", "ccmm.hip", "kernels.hip",
           "accumulate_mfma.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # packed fp32 arithmetic is disabled for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unused-parameter",
]


def compile_one(src, out, extra=(), verbose=False):
    cmd = [HIPCC] + FLAGS + list(extra) + ["-I" + os.path.join(CSRC, "inc"), "-c", os.path.join(CSRC, src), "-o", out]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return out


def build(verbose=False, lib=LIB, defines=None):
    """defines: {source file: [-D...]} extra flags for single sources (used for kernel experiments)."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    defines = defines or {}
    tag = os.path.splitext(os.path.basename(lib))[0]
    jobs = [(s, os.path.join(OBJ_DIR, "%s.%s.o" % (tag, os.path.splitext(s)[0])), defines.get(s, ())) for s in SOURCES]
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
        objs = list(pool.map(lambda j: compile_one(j[0], j[1], j[2], verbose), jobs))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc"] + objs + ["-o", lib]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return lib


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
