#!/usr/bin/env python3
"""Times every compiled kernel variant of the attention forward over a grid of shapes.

The paper leaves tile shape, warp count and pipeline depth to an auto-tuner that picks per workload
(Section 4.4; Section 7.2 names the shapes it chose for short and long sequences).  This library
ships three compiled variants and a fixed rule that chooses among them from the shape; this script
is the measurement behind that rule: it runs each variant through the C ABI (selected with the
NAUT_ATTN_VARIANT environment variable, which the library reads at every call), prints one line per
shape with the time of each variant, the fastest one and the one the built-in rule picks, and
flags disagreements.  Inputs come from the seeded generator of the benchmark workloads (N(0,1) rounded to
bf16; timing only, parity is the test-suite's job); the variants take turns launch by launch and the time of
a variant is the median over its launches.

    python -m paper_2604_14825_amd.tune            # default grid
    python -m paper_2604_14825_amd.tune --shapes 1,32,32,16384,128,1  # B,Hq,Hkv,S,D,causal
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys

VARIANTS = ("w8q32", "w4q64", "bm128")
LONG_NAME = {"w8q32": "fwd_bm256_w8q32_bn64", "w4q64": "fwd_bm256_w4q64_bn64", "bm128": "fwd_bm128_w4q32_bn64"}


def default_grid():
    shapes = []
    for D in (64, 128):
        for causal in (0, 1):
            for nbh, S in ((2, 256), (8, 256), (32, 256), (128, 256), (8, 512), (32, 512), (128, 512), (512, 512),
                           (8, 1024), (32, 1024), (128, 1024), (512, 1024), (8, 2048), (32, 2048), (128, 2048),
                           (8, 4096), (32, 4096), (128, 4096), (8, 8192), (32, 8192), (128, 8192), (8, 16384),
                           (32, 16384)):
                shapes.append((1, nbh, nbh, S, D, causal))
    shapes.append((2, 64, 8, 8192, 128, 1))  # grouped-query case
    return shapes


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--shapes", nargs="*", default=None, help="B,Hq,Hkv,S,D,causal (repeatable); default: built-in grid")
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--json", default=None, help="also write the table to this file")
    args = ap.parse_args()

    import numpy as np
    import torch
    from . import binding as nb
    from . import synth

    if not torch.cuda.is_available():
        print("tune: no GPU visible", file=sys.stderr)
        return 3
    nb.lib()
    shapes = default_grid() if not args.shapes else [tuple(int(x) for x in s.split(",")) for s in args.shapes]
    stream = torch.cuda.current_stream()
    rows = []
    print("%-34s %s   best      rule" % ("B,Hq,Hkv,S,D,causal", " ".join("%9s" % v for v in VARIANTS)))
    for (B, Hq, Hkv, S, D, causal) in shapes:
        seed = synth.BASE_SEED + 5000
        q, k, v = (torch.from_numpy(synth.fill(B, H, S, D, seed, tag, synth.BF16).view(np.int16)).cuda().view(torch.bfloat16)
                   for H, tag in ((Hq, synth.TAG_Q), (Hkv, synth.TAG_K), (Hkv, synth.TAG_V)))
        o = torch.empty_like(q)
        lse = torch.empty((B, Hq, S), dtype=torch.float32, device="cuda")
        scale = D ** -0.5
        os.environ.pop("NAUT_ATTN_VARIANT", None)
        rule = nb.variant_name(B, Hq, S, D, bool(causal), synth.BF16, synth.BF16)
        def run(var):
            os.environ["NAUT_ATTN_VARIANT"] = var
            nb.naut_attn_fwd(q, k, v, o, lse, bool(causal), scale, stream=stream)

        for var in VARIANTS:
            for _ in range(3):
                run(var)
        # the variants take turns launch by launch, so that a drift of the clock during the measurement
        # falls on all of them alike
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2 * len(VARIANTS))] for _ in range(args.reps)]
        torch.cuda.synchronize()
        for r in range(args.reps):
            for i, var in enumerate(VARIANTS):
                ev[r][2 * i].record(stream)
                run(var)
                ev[r][2 * i + 1].record(stream)
        torch.cuda.synchronize()
        times = {}
        for i, var in enumerate(VARIANTS):
            per = sorted(ev[r][2 * i].elapsed_time(ev[r][2 * i + 1]) for r in range(args.reps))
            times[var] = per[len(per) // 2] * 1e3  # microseconds, median
        os.environ.pop("NAUT_ATTN_VARIANT", None)
        best = min(times, key=times.get)
        rule_short = [s for s, l in LONG_NAME.items() if l == rule][0]
        loss = times[rule_short] / times[best] - 1.0
        flops = 4.0 * B * Hq * S * S * D * (0.5 if causal else 1.0)
        print("%-34s %s   %-8s  %-8s %s  (%.0f TFLOP/s)" % (
            "%d,%d,%d,%d,%d,%d" % (B, Hq, Hkv, S, D, causal), " ".join("%7.1fus" % times[v] for v in VARIANTS), best,
            rule_short, "" if loss < 0.03 else "rule is %.0f%% slower" % (100 * loss), flops / times[best] / 1e6), flush=True)
        rows.append({"shape": [B, Hq, Hkv, S, D, causal], "us": times, "best": best, "rule": rule_short})
        del q, k, v, o, lse
    if args.json:
        with open(args.json, "w") as f:
            json.dump(rows, f, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())
