"""Compile the HIP library for gfx950 into paper_1901_08924_amd/liblpc_hip.so.

Usage: python -m paper_1901_08924_amd.build   (or python paper_1901_08924_amd/build.py)
hipcc cross-compiles, so this works on a machine without a GPU.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "liblpc_hip.so")
OBJ_DIR = os.path.join(HERE, "_build")

# (source, extra flags).  The quantizer's float arithmetic decides integer codes:
# that translation unit is built without multiply-add contraction.
SOURCES = [
    ("lpc_api.hip", []),
    ("lpc_quant.hip", ["-ffp-contract=off"]),
    ("lpc_dense.hip", []),
    ("lpc_csr.hip", []),
    ("lpc_gemm.hip", []),
    ("lpc_mlp.hip", []),
    ("lpc_eval.hip", []),
    ("lpc_resident.hip", ["-ffp-contract=off"]),   # holds the quantizer's arithmetic too
    ("lpc_host.cpp", []),      # host-only logic: no device code (also built with sanitizers by the tests)
]
HEADERS = ["lpc_internal.h", "lpc_device.h"]

COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-fast-math",
          # packed-FP32 instructions are kept out of the generated code
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall", "-Wno-unused-function"]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _compile(src, extra, verbose):
    obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o").replace(".cpp", ".o"))
    cmd = [_hipcc()] + COMMON + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return obj


def build(verbose=False, jobs=4):
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda se: _compile(se[0], se[1], verbose), SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return OUT


def needs_build():
    if not os.path.exists(OUT):
        return True
    t = os.path.getmtime(OUT)
    deps = [os.path.join(CSRC, s) for s, _ in SOURCES] + [os.path.join(CSRC, h) for h in HEADERS]
    deps.append(os.path.join(ROOT, "include", "lpc.h"))
    return any(os.path.getmtime(p) > t for p in deps)


if __name__ == "__main__":
    build(verbose=True)
    print("built", OUT)
    sys.exit(0)
