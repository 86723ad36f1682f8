"""Builds libbiq.so (the HIP kernels and their C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libbiq.so")
SOURCES = [os.path.join(CSRC, "biq_api.hip")]
HEADERS = [
    os.path.join(CSRC, "biq_common.h"),
    os.path.join(CSRC, "biq_kernels.h"),
    os.path.join(CSRC, "biq_gemv8.h"),
    os.path.join(CSRC, "biq_gemm8x2.h"),
    os.path.join(CSRC, "biq_gemv8h.h"),
    os.path.join(CSRC, "biq_gemm8x2h.h"),
    os.path.join(CSRC, "biq_query_wide.h"),
    os.path.join(CSRC, "biq_unpack_mfma.h"),
    os.path.join(CSRC, "biq_quantize.h"),
    os.path.join(ROOT, "include", "biq.h"),
]

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    # packed fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    built = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > built for p in SOURCES + HEADERS)


def build_library(verbose: bool = False) -> str:
    """Compiles every HIP source into libbiq.so (always recompiles). Returns the library path."""
    hipcc = os.environ.get("HIPCC", "hipcc")
    tmp = LIB_PATH + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + ["-I" + os.path.join(ROOT, "include"), "-I" + CSRC] + SOURCES + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass warns that it does not know the packed-fp32 feature; that is expected
    out = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
    sys.exit(0)
