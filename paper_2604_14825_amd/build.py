"""Build the C-ABI library (hipcc, gfx950 only) and the host-side input generator."""
from __future__ import annotations

import os
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
_CSRC = os.path.join(_HERE, "csrc")
# (source, extra defines, object name).  The prefill kernels are instantiated in naut_attn_inst.hip, compiled
# once per (input type, output type) pair so that the four pairs build in parallel.
_DT = {"bf16": 0, "f16": 1, "f32": 2}  # naut_dtype
JOBS = [(os.path.join(_CSRC, n), [], n + ".o") for n in ("naut_attn.hip", "naut_decode.hip", "naut_fp8.hip", "naut_probe.hip")]
JOBS += [(os.path.join(_CSRC, "naut_attn_inst.hip"), ["-DNAUT_INST_IN=%d" % _DT[i], "-DNAUT_INST_OUT=%d" % _DT[o]],
          "naut_attn_inst_%s_%s.o" % (i, o))
         for i, o in (("bf16", "bf16"), ("bf16", "f32"), ("f16", "f16"), ("f16", "f32"))]
SRCS = sorted({j[0] for j in JOBS})
LIB = os.path.join(_HERE, "libnaut_attn.so")
# The same sources with every hand-made synchronisation replaced by its most conservative form (-DNAUT_SAFE_SYNC=1,
# see naut_common.h); tests/test_safe_sync_gpu.py requires the two libraries to agree bit for bit.
LIB_SAFE = os.path.join(_HERE, "libnaut_attn_safe.so")

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


def build_lib(extra=(), verbose=False, out=None) -> str:
    """Compile every translation unit to an object (in parallel: one hipcc each), then link the shared
    library (to `out` if given, else in place)."""
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    out = out or LIB
    compile_flags = [f for f in FLAGS if f != "-shared"]
    with tempfile.TemporaryDirectory(prefix="naut_build_") as tmpdir:
        objs = [os.path.join(tmpdir, j[2]) for j in JOBS]

        def compile_one(job):
            (src, defs, _), obj = job
            cmd = [HIPCC] + compile_flags + list(extra) + defs + ["-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.check_call(cmd)

        with ThreadPoolExecutor(max_workers=min(len(JOBS), os.cpu_count() or 1)) as pool:
            list(pool.map(compile_one, zip(JOBS, objs)))
        tmp = out + ".tmp%d" % os.getpid()
        link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", tmp]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.check_call(link)
        os.replace(tmp, out)
    return out


def build_all(verbose=False):
    from . import synth
    synth.build(force=True)
    build_lib(extra=["-DNAUT_SAFE_SYNC=1"], verbose=verbose, out=LIB_SAFE)
    return build_lib(verbose=verbose)


if __name__ == "__main__":
    sys.path.insert(0, ROOT)
    from paper_2604_14825_amd import synth
    synth.build(force=True)
    args = sys.argv[1:]
    out = None
    if args and args[0].startswith("--out="):  # link somewhere else (A/B builds with extra -D flags)
        out, args = args[0][len("--out="):], args[1:]
    if out is None and not args:
        print(build_lib(extra=["-DNAUT_SAFE_SYNC=1"], verbose=True, out=LIB_SAFE))
    print(build_lib(extra=args, verbose=True, out=out))
