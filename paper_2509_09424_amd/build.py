"""Builds libensi_hip.so (gfx950) in-tree with hipcc: one object per source, compiled in parallel, then linked."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libensi_hip.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["api.hip", "api_keys.hip", "api_static.hip", "api_matmul.hip", "api_pmult.hip", "api_ccmm.hip", "ntt.hip", "ntt16.hip", "keyswitch16.hip", "pmult.hip", "ccmm.hip", "kernels.hip",
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


def build_sanitized(lib=None):
    """The same library with AddressSanitizer and UndefinedBehaviorSanitizer on the HOST code only (device code is
    compiled as usual): for running the host logic under sanitizers on a CPU-only machine."""
    lib = lib or os.path.join(OBJ_DIR, "libensi_hip_san.so")
    os.makedirs(OBJ_DIR, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    jobs = [(s, os.path.join(OBJ_DIR, "san.%s.o" % os.path.splitext(s)[0])) for s in SOURCES]
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as pool:
        objs = list(pool.map(lambda j: compile_one(j[0], j[1], san), jobs))
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-fsanitize=address", "-fsanitize=undefined",
                           "-shared-libsan"] + objs + ["-o", lib])
    return lib


def sanitizer_runtime():
    """Path of the AddressSanitizer runtime that a process loading the sanitized library has to preload."""
    clang = os.path.join(os.path.dirname(os.path.realpath(HIPCC)), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang"
    return subprocess.check_output([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], text=True).strip()


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
