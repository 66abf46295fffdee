"""Build libtlq.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2602_07899_amd.build

Compiles every translation unit under csrc/ and links them into
paper_2602_07899_amd/libtlq.so.  hipcc cross-compiles, so this works on a
machine without a GPU.
"""
from __future__ import annotations

import concurrent.futures as cf
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtlq.so")
CEILING = os.path.join(HERE, "mfma_ceiling")

SOURCES = ["api.hip", "stats.hip", "quant.hip", "gemm.hip", "glue.hip", "block.hip", "select.hip", "profile.hip", "noalloc.hip", "gram.hip"]
COMMON = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-I", os.path.join(ROOT, "include"),
          "-I", CSRC, "-Wall", "-Wno-unused-function",
          # keep hipcc from forming packed-fp32 instructions on its own
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# the quantiser's float arithmetic must round once per written operation
PER_FILE = {"quant.hip": ["-ffp-contract=off"]}


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _compile(src: str, extra=(), suffix=""):
    obj = os.path.join(OBJ, src.replace(".hip", suffix + ".o"))
    cmd = [hipcc(), *COMMON, *PER_FILE.get(src, []), *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                     if "not a recognized feature for this target" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{msgs}")
    return obj, msgs


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with cf.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        results = list(ex.map(_compile, SOURCES))
    objs = [o for o, _ in results]
    if verbose:
        for (_, m), s in zip(results, SOURCES):
            if m.strip():
                print(f"[{s}]\n{m}")
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    import ctypes
    ctypes.CDLL(LIB)  # an unresolved symbol must fail the build, not the first caller
    # stand-alone measurement of the sustained MFMA ceiling (used by bench.py for context)
    r = subprocess.run([hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", *COMMON[-4:],
                        os.path.join(CSRC, "mfma_ceiling.hip"), "-o", CEILING], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("mfma_ceiling build failed:\n" + r.stdout + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


# Host code of the argument-validation layer under AddressSanitizer + UndefinedBehaviorSanitizer.
# Only the host pass of the three translation units without kernels of their own logic on the
# validation paths is instrumented (device code cannot be sanitised here); the kernels' objects
# are reused from the normal build.  The result is a driver executable that calls every entry
# point with arguments that must be rejected before anything is launched, so it runs without a GPU.
SANITIZED = ["api.hip", "noalloc.hip", "profile.hip"]
SAN_FLAGS = ["-g", "-O1", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]


def build_sanitized_driver() -> str:
    """Build (and return the path of) the sanitizer driver; needs a finished normal build."""
    plain = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES if s not in SANITIZED]
    if not all(os.path.exists(o) for o in plain):
        build(verbose=False)
    with cf.ThreadPoolExecutor(max_workers=len(SANITIZED)) as ex:
        san = [o for o, _ in ex.map(lambda s: _compile(s, SAN_FLAGS, "_san"), SANITIZED)]
    exe = os.path.join(OBJ, "abi_validation_driver")
    src = os.path.join(ROOT, "tests", "native", "abi_validation_driver.cpp")
    cmd = [hipcc(), "--offload-arch=gfx950", "-std=c++17", "-g", "-O1", "-fsanitize=address", "-fsanitize=undefined",
           "-fno-sanitize-recover=undefined", "-fno-gpu-sanitize", "-I", os.path.join(ROOT, "include"),
           "-x", "c++", src, "-x", "none", *san, *plain, "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("sanitizer driver build failed:\n" + r.stdout + r.stderr)
    return exe


if __name__ == "__main__":
    build()
