"""Compiles the HIP sources into libecq.so next to this file (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
INCLUDE = os.path.join(os.path.dirname(PKG_DIR), "include")
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libecq.so")
SOURCES = ["ecq_api.hip", "ecq_kernels.hip", "ecq_huffman.hip", "ecq_zrun.hip"]

# -ffp-contract=off: every binary32 operation of the codec rounds on its own.
# packed-fp32-ops off: no v_pk_*_f32 instructions are generated.
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fno-fast-math", "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-fno-gpu-flush-denormals-to-zero",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build(verbose: bool = False, extra: list[str] | None = None, out: str | None = None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = out or LIB_PATH
    tmp = out + ".tmp.%d" % os.getpid()
    cmd = [hipcc, *HIPCC_FLAGS, "-I" + INCLUDE, *(extra or []), *[os.path.join(CSRC, s) for s in SOURCES], "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
