"""Build the C-ABI library (hipcc, gfx950 only) and the host-side input generator."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
SRCS = [os.path.join(_HERE, "csrc", n) for n in ("naut_attn.hip", "naut_decode.hip", "naut_fp8.hip")]
LIB = os.path.join(_HERE, "libnaut_attn.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # packed-fp32 VALU forms stay off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # device code only: no NaN can occur in the kernels (masks are -inf, the running maximum starts
    # finite), and knowing it lets max(max(a,b),c) become one instruction with no operand quieting
    "-Xarch_device", "-fno-honor-nans",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"),
]


def build_lib(extra=(), verbose=False) -> str:
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [HIPCC] + FLAGS + list(extra) + SRCS + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


def build_all(verbose=False):
    from . import synth
    synth.build(force=True)
    return build_lib(verbose=verbose)


if __name__ == "__main__":
    sys.path.insert(0, ROOT)
    from paper_2604_14825_amd import synth
    synth.build(force=True)
    print(build_lib(extra=sys.argv[1:], verbose=True))
