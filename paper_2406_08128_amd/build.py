"""Build libchela.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2406_08128_amd.build          # compile everything, link
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libchela.so")
SOURCES = ["chela_api.hip", "chela_kernels_f32.hip", "chela_kernels_bf16.hip", "chela_kernels_conv.hip",
           "chela_kernels_convmx.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 VALU forms are switched off for every device compile (they have given wrong results on this pool)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # keep MFMA accumulators in architectural VGPRs: every accumulator here is read back by the vector ALU
         # (rounding to bf16) once per chunk, and AGPR<->VGPR copies would double that work
         "-mllvm", "-amdgpu-mfma-vgpr-form",
         "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    msgs = [ln for ln in r.stdout.splitlines() if "packed-fp32-ops" not in ln and ln.strip()]
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, "\n".join(msgs)))
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(4, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    if verbose:
        print("built", LIB)
    return LIB


def build_host_ubsan(verbose: bool = False) -> str:
    """libchela with the HOST half of the API file (argument checks, planner, scratch bookkeeping) compiled under
    UndefinedBehaviorSanitizer in trap mode: undefined behaviour stops the process, and no sanitizer runtime has to be
    loaded.  The kernels' objects are the ordinary ones (built first if they are missing).  For the CPU test tier only:
    the result lives in the build folder and is never what the binding loads by default."""
    objs = [os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o") for src in SOURCES]
    if not all(os.path.exists(o) for o in objs):
        build(verbose=False)
    api_obj = os.path.join(OBJ_DIR, "chela_api_ubsan.o")
    san = ["-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fsanitize-trap=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    cmd = [HIPCC, *[f for f in FLAGS if f != "-O3"], "-O1", *san, "-c", os.path.join(CSRC, "chela_api.hip"), "-o", api_obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc (host UBSan) failed:\n" + r.stdout)
    lib = os.path.join(OBJ_DIR, "libchela_ubsan.so")
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, api_obj, *objs[1:]]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    build()
    sys.exit(0)
