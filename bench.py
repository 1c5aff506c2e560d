#!/usr/bin/env python3
"""Benchmark of the fused attention forward (one GPU).

A "step" is one pass of the whole hot path -- one naut_attn_fwd call over one
batch of synthetic input already resident in HBM.  The default workload is the
one the headline metric is quoted on: B=1, Hq=Hkv=32, S=16384, D=128, bf16,
causal, 1 % of the K rows scaled by 8.  Prints ONE JSON line.

The paper (Section 7, "Profiling and Performance Reporting") times with device
events, one discarded warm-up and 10 repetitions, and reports FLOPs of the
attention computation from the model configuration divided by latency; here
FLOPs = 4*B*Hq*S^2*D, halved for causal (work actually required).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6  # MI355X dense bf16/fp16 MFMA: 256 CU x 4096 FLOP/clk/CU x 2.4 GHz

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), scaled by a plain
# copy kernel of known size; filled in from profiles/ once measured, else null.
MEASURED_TRAFFIC_BYTES = {
    # profiles/naut_fwd_bm256_w8q32_long_S16384_D128_causal.md: 721930 KiB x 2.000 read + 133120 KiB x 1.000 written
    "long": 1.615e9,
    # profiles/naut_decode_B8_Hq32_Hkv8_Sk16384_D128.md: (262347 + 407) KiB x 2.000 read + (528 + 72) KiB written
    "decode": 5.387e8,
    # profiles/naut_fwd_fp8_long_S16384_D128_causal.md: 564080 KiB x 2.000 read + 133170 KiB written
    "long_fp8": 1.292e9,
    # profiles/naut_decode_fp8_B8_Hq32_Hkv8_Sk16384_D128.md: (131210 + 410) KiB x 2.000 read + (528 + 72) KiB written
    "decode_fp8": 2.702e8,
    # profiles/naut_fwd_bm128_w4q32_bn32_long_S16384_D256_causal.md: 2604500 KiB x 2.000 read + 264190 KiB written
    "long_d256": 5.60e9,
}

PEAK_FP8_TFLOPS = 5033.2   # MI355X dense fp8 MFMA: twice the bf16 figure
PEAK_HBM_GBS = 8000.0  # MI355X HBM3E
FP8_DESCALE = {"q": 1.0 / 64, "k": 1.0 / 8, "v": 1.0 / 64}  # per-tensor scales of the synthetic FP8 inputs

# Decode-time workload (the paper's second workload, Section 6): one new position per sequence against a
# 16k-token key/value cache, 32 query heads on 8 K/V heads (a Qwen/GLM-like layout), B = 8.
DECODE = {"B": 8, "Hq": 32, "Hkv": 8, "Sq": 1, "Sk": 16384, "D": 128, "outlier_frac": 0.01, "outlier_scale": 8.0}

PAPER_CONTEXT = ("paper reports relative gains only: up to 23% over state-of-the-art compilers on GH200 and "
                 "up to 42% on RTX 5090 (FP16/FP8, other hardware) -- context, not a target")


class HipEvents:
    """Minimal HIP event timing on an explicit stream (ctypes on libamdhip64)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        assert rc == 0, "hipEventCreate failed: %d" % rc
        return ev

    def record(self, ev, stream_ptr):
        rc = self.hip.hipEventRecord(ev, ctypes.c_void_p(stream_ptr))
        assert rc == 0, "hipEventRecord failed: %d" % rc

    def elapsed_ms(self, a, b) -> float:
        rc = self.hip.hipEventSynchronize(b)
        assert rc == 0, "hipEventSynchronize failed: %d" % rc
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        assert rc == 0, "hipEventElapsedTime failed: %d" % rc
        return float(ms.value)


def cpu_baseline(w, q, k, v, target_seconds: float):
    """The oracle, as it stands, timed on this machine's host cores on a bounded sample of query rows.

    A first small batch of rows calibrates the rate; the timed sample is then sized for about
    `target_seconds` of CPU work (each output row is independent, so a row subset is exact).
    """
    import numpy as np
    import oracle
    total = w.B * w.Hq * w.S
    perm = np.random.default_rng(2604).permutation(total)

    def run(rows):
        rows = np.sort(rows).astype(np.int64)
        t0 = time.perf_counter()
        oracle.attn_rows(q, k, v, w.in_dtype, w.causal, w.scale, rows=rows)
        dt = time.perf_counter() - t0
        keys = (rows % w.S) + 1 if w.causal else np.full(rows.shape, w.S)
        return dt, float((4.0 * w.D * keys).sum())

    n0 = min(512, total)
    dt0, fl0 = run(perm[:n0])
    # dt0 includes the fixed fp64 decode of K and V; size the real sample from the marginal rate
    dt_fixed, _ = run(perm[:1])
    rate = max(dt0 - dt_fixed, 1e-3) / n0
    n = int(min(total, max(n0, (target_seconds - dt_fixed) / rate)))
    dt, fl = run(perm[:n])
    return {
        "value": fl / dt / 1e12,
        "unit": "TFLOP/s",
        "cores": int(oracle.threads()),
        "kind": "oracle",
        "sample": "%d of %d query rows (uniform, seeded), %.1f s wall incl. fp64 decode of K,V; same FLOP convention"
                  % (n, total, dt),
        "seconds": dt,
    }


def bench_fp8(args, nb, synth, torch, np) -> int:
    """The long shape on FP8 (E4M3) inputs with per-tensor scales; one step = one naut_attn_fwd_fp8 call."""
    w = synth.WORKLOADS["long"]
    seed = synth.workload_seed(w)
    dq, dk, dv = FP8_DESCALE["q"], FP8_DESCALE["k"], FP8_DESCALE["v"]
    q = synth.fill_e4m3(w.B, w.Hq, w.S, w.D, seed, synth.TAG_Q, dq)
    k = synth.fill_e4m3(w.B, w.Hkv, w.S, w.D, seed, synth.TAG_K, dk, w.n_outlier, w.outlier_scale)
    v = synth.fill_e4m3(w.B, w.Hkv, w.S, w.D, seed, synth.TAG_V, dv)
    qd, kd, vd = (torch.from_numpy(a).cuda() for a in (q, k, v))
    o = torch.empty((w.B, w.Hq, w.S, w.D), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((w.B, w.Hq, w.S), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        nb.naut_attn_fwd_fp8(qd, kd, vd, o, lse, w.causal, w.scale, dq, dk, dv, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = HipEvents()
    e0, e1 = ev.create(), ev.create()
    t0 = time.perf_counter()
    ev.record(e0, stream.cuda_stream)
    for _ in range(args.steps):
        step()
    ev.record(e1, stream.cuda_stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_wall = (t1 - t0) * 1e3 / args.steps
    ms_kernel = ev.elapsed_ms(e0, e1) / args.steps
    flops = w.flops
    nq, nkv = w.B * w.Hq * w.S * w.D, w.B * w.Hkv * w.S * w.D
    io_bytes = nq + 2 * nkv + nq * 2 + w.B * w.Hq * w.S * 4
    out = {
        "metric": "attention fwd TFLOP/s, FP8 E4M3 inputs (S=16k causal D=128)",
        "value": flops / (ms_wall * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_wall,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp8_e4m3",
        "data": "synthetic",
        "config": {"workload": "long_fp8", "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "S": w.S, "D": w.D, "causal": w.causal,
                   "outlier_k_rows": w.n_outlier, "descale": FP8_DESCALE, "kernel": "fwd_fp8_bm128_w4q32_bn64",
                   "flop_convention": "4*B*Hq*S^2*D, halved for causal"},
        "roofline": {"bound": "mfma", "achieved": flops / (ms_kernel * 1e-3) / 1e12, "peak": PEAK_FP8_TFLOPS,
                     "unit": "TFLOP/s", "frac": flops / (ms_kernel * 1e-3) / 1e12 / PEAK_FP8_TFLOPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get("long_fp8"), "kernel_ms": ms_kernel,
                     "algorithmic_hbm_bytes": io_bytes},
        "context": PAPER_CONTEXT,
    }
    if args.cpu_seconds > 0 and args.cpu_rows != 0:
        import oracle
        total = w.B * w.Hq * w.S
        perm = np.random.default_rng(2604).permutation(total)

        def run(rows):
            rows = np.sort(rows).astype(np.int64)
            t0 = time.perf_counter()
            oracle.attn_rows_e4m3(q, k, v, dq, dk, dv, w.causal, w.scale, rows=rows)
            dt = time.perf_counter() - t0
            return dt, float((4.0 * w.D * ((rows % w.S) + 1)).sum())
        dt0, _ = run(perm[:512])
        dt_fixed, _ = run(perm[:1])
        rate = max(dt0 - dt_fixed, 1e-3) / 512
        n = int(min(total, max(512, (args.cpu_seconds - dt_fixed) / rate)))
        dt, fl = run(perm[:n])
        out["cpu_baseline"] = {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": int(oracle.threads()), "kind": "oracle",
                               "sample": "%d of %d query rows (uniform, seeded), %.1f s wall incl. fp64 decode of K,V"
                               % (n, total, dt), "seconds": dt}
    print(json.dumps(out))
    return 0


def bench_decode(args, nb, synth, torch, np, fp8=False) -> int:
    """One step = one naut_attn_decode (or naut_attn_decode_fp8) call (split kernel + merge kernel) over the
    resident cache."""
    c = DECODE
    B, Hq, Hkv, Sq, Sk, D = c["B"], c["Hq"], c["Hkv"], c["Sq"], c["Sk"], c["D"]
    seed = synth.BASE_SEED + 100
    if fp8:
        q = synth.fill_e4m3(B, Hq, Sq, D, seed, synth.TAG_Q, FP8_DESCALE["q"])
        k = synth.fill_e4m3(B, Hkv, Sk, D, seed, synth.TAG_K, FP8_DESCALE["k"], int(c["outlier_frac"] * Sk),
                            c["outlier_scale"])
        v = synth.fill_e4m3(B, Hkv, Sk, D, seed, synth.TAG_V, FP8_DESCALE["v"])
        dev = lambda a: torch.from_numpy(a).cuda()
    else:
        q = synth.fill(B, Hq, Sq, D, seed, synth.TAG_Q, synth.BF16)
        k = synth.fill(B, Hkv, Sk, D, seed, synth.TAG_K, synth.BF16, int(c["outlier_frac"] * Sk), c["outlier_scale"])
        v = synth.fill(B, Hkv, Sk, D, seed, synth.TAG_V, synth.BF16)
        dev = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    qd, kd, vd = dev(q), dev(k), dev(v)
    o = torch.empty((B, Hq, Sq, D), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((B, Hq, Sq), dtype=torch.float32, device="cuda")
    ws = torch.empty(nb.decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    scale = D ** -0.5

    def step():
        if fp8:
            nb.naut_attn_decode_fp8(qd, kd, vd, o, lse, True, scale, FP8_DESCALE["q"], FP8_DESCALE["k"],
                                    FP8_DESCALE["v"], ws, stream=stream)
        else:
            nb.naut_attn_decode(qd, kd, vd, o, lse, True, scale, ws, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = HipEvents()
    e0, e1 = ev.create(), ev.create()
    t0 = time.perf_counter()
    ev.record(e0, stream.cuda_stream)
    for _ in range(args.steps):
        step()
    ev.record(e1, stream.cuda_stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_wall = (t1 - t0) * 1e3 / args.steps
    ms_kernel = ev.elapsed_ms(e0, e1) / args.steps
    # algorithmic bytes: Q, K, V read once; O and LSE written once (the partials in the workspace are extra)
    in_b = 1 if fp8 else 2
    nbytes = (B * Hq * Sq * D + 2 * B * Hkv * Sk * D) * in_b + B * Hq * Sq * D * 2 + B * Hq * Sq * 4
    out = {
        "metric": "decode attention GB/s (B=8, 32/8 heads, Sk=16k, D=128)" + (", FP8 E4M3 cache" if fp8 else ""),
        "value": nbytes / (ms_wall * 1e-3) / 1e9,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_wall,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp8_e4m3" if fp8 else "bf16",
        "data": "synthetic",
        "config": {"workload": "decode_fp8" if fp8 else "decode", "B": B, "Hq": Hq, "Hkv": Hkv, "Sq": Sq, "Sk": Sk, "D": D, "causal": True,
                   "outlier_k_rows": int(c["outlier_frac"] * Sk),
                   "kernel": "decode_split_fp8_32x32x64 + merge" if fp8 else "decode_split32x32 + merge",
                   "workspace_bytes": int(ws.numel())},
        "roofline": {"bound": "hbm", "achieved": nbytes / (ms_kernel * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": nbytes / (ms_kernel * 1e-3) / 1e9 / PEAK_HBM_GBS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get("decode_fp8" if fp8 else "decode"), "kernel_ms": ms_kernel,
                     "algorithmic_hbm_bytes": nbytes},
        "context": PAPER_CONTEXT,
    }
    if args.cpu_seconds > 0 and args.cpu_rows != 0:
        import oracle
        # the whole workload is well under a second of CPU work, so the sample is all of it
        nb_s = B
        t0 = time.perf_counter()
        if fp8:
            oracle.attn_cross_e4m3(q[:nb_s], k[:nb_s], v[:nb_s], FP8_DESCALE["q"], FP8_DESCALE["k"], FP8_DESCALE["v"],
                                   True, scale)
        else:
            oracle.attn_cross16(q[:nb_s], k[:nb_s], v[:nb_s], synth.BF16, True, scale)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": nbytes * nb_s / B / dt / 1e9, "unit": "GB/s", "cores": int(oracle.threads()),
                               "kind": "oracle", "sample": "%d of %d batch entries, %.2f s wall incl. fp64 decode of K,V"
                               % (nb_s, B, dt), "seconds": dt}
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="long", help="tiny|encoder|prefill|gqa|long; long_d256 (the long shape at "
                    "D = 256); decode (a second, HBM-bound path: naut_attn_decode); decode_fp8 (the same on an E4M3 cache: "
                    "naut_attn_decode_fp8); long_fp8 (the long shape on "
                    "FP8 E4M3 inputs: naut_attn_fwd_fp8)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0,
                    help="seconds of CPU work the oracle baseline sample is sized for (0 = skip)")
    ap.add_argument("--cpu-rows", type=int, default=None, help="deprecated spelling: 0 skips the oracle baseline")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="only run a plain device copy of this many MiB (5 times): the known-size kernel "
                         "against which rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by construction (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2604_14825_amd import binding as nb
    from paper_2604_14825_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    nb.lib()  # fail loudly if the HIP library is missing

    if args.calibrate_copy > 0:
        n = args.calibrate_copy * (1 << 20)
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": n, "calibrate_copy_bytes_written": n, "launches": 5}))
        return 0

    if args.workload == "decode":
        return bench_decode(args, nb, synth, torch, np)
    if args.workload == "decode_fp8":
        return bench_decode(args, nb, synth, torch, np, fp8=True)
    if args.workload == "long_fp8":
        return bench_fp8(args, nb, synth, torch, np)

    w = synth.WORKLOADS[args.workload]
    q, k, v = synth.make_inputs(w)
    tdt = {synth.BF16: torch.bfloat16, synth.F16: torch.float16, synth.F32: torch.float32}
    dev = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(tdt[w.in_dtype])
    qd, kd, vd = dev(q), dev(k), dev(v)
    o = torch.empty((w.B, w.Hq, w.S, w.D), dtype=tdt[w.out_dtype], device="cuda")
    lse = torch.empty((w.B, w.Hq, w.S), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    sptr = stream.cuda_stream

    def step():
        nb.naut_attn_fwd(qd, kd, vd, o, lse, w.causal, w.scale, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    ev = HipEvents()
    e0, e1 = ev.create(), ev.create()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev.record(e0, sptr)
    for _ in range(args.steps):
        step()
    ev.record(e1, sptr)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_wall = (t1 - t0) * 1e3 / args.steps
    ms_kernel = ev.elapsed_ms(e0, e1) / args.steps  # average launch duration on the launch stream

    flops = w.flops
    tflops = flops / (ms_wall * 1e-3) / 1e12
    achieved = flops / (ms_kernel * 1e-3) / 1e12
    variant = nb.variant_name(w.B, w.Hq, w.S, w.D, w.causal, w.in_dtype, w.out_dtype)

    out = {
        "metric": "attention fwd TFLOP/s (S=16k causal D=128)" if w.name == "long" else "attention fwd TFLOP/s",
        "value": tflops,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_wall,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if w.in_dtype == synth.BF16 else "f16",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "S": w.S, "D": w.D,
                   "causal": w.causal, "outlier_k_rows": w.n_outlier, "kernel": variant,
                   "flop_convention": "4*B*Hq*S^2*D, halved for causal",
                   "pct_of_bf16_mfma_peak": 100.0 * tflops / PEAK_BF16_TFLOPS},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(w.name),
                     "kernel_ms": ms_kernel, "algorithmic_hbm_bytes": w.io_bytes},
        "context": PAPER_CONTEXT,
    }
    if args.cpu_seconds > 0 and args.cpu_rows != 0:
        cb = cpu_baseline(w, q, k, v, args.cpu_seconds)
        cb["gpu_over_cpu"] = tflops / cb["value"]
        out["cpu_baseline"] = cb
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
