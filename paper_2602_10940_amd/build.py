"""Build the C-ABI library (libusp.so) for gfx950 with hipcc, in-tree.

    python -m paper_2602_10940_amd.build          # rebuild
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ_DIR = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libusp.so")

SOURCES = ["usp_api.hip", "fp8_kernels.hip", "merge_kernel.hip", "attn_generic.hip", "attn_mfma.hip"]
# libusp_diag.so: the MFMA-rate probe of the benchmark and a test hook, outside the library's ABI
DIAG_LIB = os.path.join(PKG, "libusp_diag.so")
DIAG_SOURCES = [os.path.join("diag", "usp_diag.hip")]

# -packed-fp32-ops off: keep the compiler from forming packed fp32 VALU ops.
# IEEE fp32 division / denormals are required by the FP8 scale arithmetic (no fast-math).
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fhip-fp32-correctly-rounded-divide-sqrt", "-fno-gpu-flush-denormals-to-zero",
    "-fno-fast-math", "-ffp-contract=off",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


def _compile(src: str, extra) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(os.path.basename(src))[0] + ".o")
    cmd = [hipcc(), *HIPCC_FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, " ".join(cmd), r.stderr[-8000:]))
    return obj


def build(verbose: bool = False, extra_flags=()) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = SOURCES + DIAG_SOURCES
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags)), srcs))
    n = len(SOURCES)
    for lib, lib_objs, extra in ((LIB, objs[:n], []),
                                 (DIAG_LIB, objs[n:], ["-L", PKG, "-lusp", "-Wl,-rpath,$ORIGIN"])):
        cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *lib_objs, *extra]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n%s" % r.stderr[-8000:])
        if verbose:
            print("built", lib)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra_flags=sys.argv[1:])
