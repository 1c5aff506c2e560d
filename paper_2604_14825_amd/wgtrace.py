#!/usr/bin/env python3
"""Per-work-group timeline of the pipelined attention kernel, from a timing-only build of the library.

    python paper_2604_14825_amd/build.py --out=/tmp/libnaut_stamp.so -DNAUT_STAMP=1
    python -m paper_2604_14825_amd.wgtrace --lib /tmp/libnaut_stamp.so --workload long

In that build every wavefront of `naut_fwd_kernel_v2` stamps the constant 100 MHz clock at six points (entry;
Q and prologue tiles issued; landed and published; active iterations done; idle iterations done; stores
acknowledged) and writes them, the hardware id of the compute unit it ran on and its iteration count over
its work-group's lse rows (lse itself is not written; O is).  This script launches one of the synthetic
workloads (S a multiple of 256, D <= 128, a shape that the 256-query kernel serves), reads the records back
and prints: the time spent in each phase, a straight-line fit of work-group lifetime against iterations (the
intercept is the cost that does not scale with the key range), the gap between consecutive work-groups on a
compute unit, and when each XCD finishes.  It measures; parity is the test-suite's job.
"""
from __future__ import annotations

import argparse
import os
import sys

TICK_US = 0.01  # the constant clock runs at 100 MHz


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--lib", required=True, help="library built with -DNAUT_STAMP=1")
    ap.add_argument("--workload", default="long", help="name in synth.WORKLOADS (default: long)")
    ap.add_argument("--launches", type=int, default=30, help="launches in a row; the last one's records are read")
    args = ap.parse_args()

    import numpy as np
    import torch

    here = os.path.dirname(os.path.abspath(__file__))
    sys.path.insert(0, os.path.dirname(here))
    from paper_2604_14825_amd import binding as nb, synth

    nb.LIB_PATH = os.path.abspath(args.lib)
    os.environ["NAUT_ATTN_VARIANT"] = "w8q32"
    w = synth.WORKLOADS[args.workload]
    if w.S % 256 or w.D > 128 or w.in_dtype != synth.BF16:
        raise SystemExit("needs a bf16 workload with S a multiple of 256 and D <= 128")
    q, k, v = synth.make_inputs(w)
    dev = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    qd, kd, vd = dev(q), dev(k), dev(v)
    B, H, S, D = w.B, w.Hq, w.S, w.D
    o = torch.empty((B, H, S, D), dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros((B, H, S), dtype=torch.float32, device="cuda")
    for _ in range(max(1, args.launches)):  # every launch overwrites the records: the last one's are read
        nb.naut_attn_fwd(qd, kd, vd, o, lse, w.causal, w.scale)
    torch.cuda.synchronize()

    nq = S // 256
    rec = lse.cpu().numpy().view(np.int64).reshape(B * H, nq, 128)[:, :, :64].reshape(-1, 8, 8)  # [wg][wave][word]
    if not rec[:, :, 0].all():
        raise SystemExit("no time stamps found: was --lib built with -DNAUT_STAMP=1?")
    t0 = rec[:, :, 0].min()
    start = (rec[:, :, 0].min(1) - t0) * TICK_US
    end = (rec[:, :, 5].max(1) - t0) * TICK_US
    hw = rec[:, 0, 6]
    xcc = (hw >> 32) & 15
    cu = xcc * 256 + ((hw & 0xFFFFFFFF) >> 8 & 0xFF)  # XCC id, then shader engine / array / CU bits of HW_ID
    nit = rec[:, 0, 7]
    cus = sorted(set(cu.tolist()))
    print("%s: %d work-groups on %d compute units, kernel span %.1f us" % (args.workload, len(start), len(cus), end.max()))

    phase = lambda a, b: (rec[:, :, b] - rec[:, :, a]) * TICK_US
    for name, a, b in (("entry -> loads issued", 0, 1), ("loads issued -> published", 1, 2), ("active iterations", 2, 3),
                       ("idle iterations", 3, 4), ("epilogue + store drain", 4, 5)):
        x = phase(a, b)
        print("  %-26s mean %8.2f  min %8.2f  max %8.2f us   (first wavefront %.2f, last %.2f)"
              % (name, x.mean(), x.min(), x.max(), x[:, 0].mean(), x[:, -1].mean()))
    A = np.vstack([nit, np.ones_like(nit)]).T.astype(float)
    slope, icpt = np.linalg.lstsq(A, end - start, rcond=None)[0]
    print("  work-group lifetime = %.3f us x iterations + %.2f us" % (slope, icpt))

    gaps, last_end, busy = [], {}, {}
    for c in cus:
        idx = np.where(cu == c)[0]
        idx = idx[np.argsort(start[idx])]
        gaps += [start[b_] - end[a_] for a_, b_ in zip(idx[:-1], idx[1:])]
        last_end[c] = end[idx].max()
        busy[c] = (end[idx] - start[idx]).sum()
    if gaps:
        g = np.array(gaps)
        print("  gap between work-groups on a compute unit: mean %.2f  min %.2f  max %.2f us" % (g.mean(), g.min(), g.max()))
    le = np.array(list(last_end.values()))
    print("  last end per compute unit: mean %.1f  min %.1f  max %.1f us" % (le.mean(), le.min(), le.max()))
    loop = (rec[:, :, 4] - rec[:, :, 2]).max(1) * TICK_US
    for x in sorted(set(xcc.tolist())):
        cs = [c for c in cus if c // 256 == x]
        print("  XCD %d: %2d units, ends at %.1f us (mean unit %.1f), %.3f us per iteration"
              % (x, len(cs), max(last_end[c] for c in cs), np.mean([last_end[c] for c in cs]),
                 loop[xcc == x].sum() / nit[xcc == x].sum()))
    return 0


if __name__ == "__main__":
    sys.exit(main())
