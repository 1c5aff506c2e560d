#!/usr/bin/env python3
"""Benchmark of the fused attention forward (one GPU).

A "step" is one pass of the whole hot path -- one naut_attn_fwd call over one
batch of synthetic input already resident in HBM.  The default workload is the
one the headline metric is quoted on: B=1, Hq=Hkv=32, S=16384, D=128, bf16,
causal, 1 % of the K rows scaled by 8.  Prints ONE JSON line.

The paper (Section 7, "Profiling and Performance Reporting") times with device
events, one discarded warm-up and 10 repetitions, and reports FLOPs of the
attention computation from the model configuration divided by latency; here
FLOPs = 4*B*Hq*S^2*D, halved for causal (work actually required), every step has
an event pair of its own (minimum, median and mean are reported; the roofline
figure uses the median), and the output left in the timed buffers is compared
with the fp64 oracle on a declared sample of rows before the line is printed:
the error statistics of the paper's numerical-stability table (Appendix B: RMS,
90th and 99th percentile of the absolute error against an FP64 unfused reference)
plus the maximum and the mean, and a non-zero exit status if the acceptance bar
(max |dO| <= 2e-2, mean |dO| <= 2e-3, lse within 1e-3 relative) is missed.
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
PEAK_FP8_TFLOPS = 5033.2   # MI355X dense fp8 MFMA: twice the bf16 figure
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E
FP8_DESCALE = {"q": 1.0 / 64, "k": 1.0 / 8, "v": 1.0 / 64}  # per-tensor scales of the synthetic FP8 inputs
TOL_16BIT = {"max_abs": 2e-2, "mean_abs": 2e-3, "lse_rel": 1e-3}  # the acceptance bar for bf16/f16 inputs

# Decode-time workload (the paper's second workload, Section 6): one new position per sequence against a
# 16k-token key/value cache, 32 query heads on 8 K/V heads (a Qwen/GLM-like layout), B = 8.
DECODE = {"B": 8, "Hq": 32, "Hkv": 8, "Sq": 1, "Sk": 16384, "D": 128, "outlier_frac": 0.01, "outlier_scale": 8.0}

PAPER_CONTEXT = ("paper reports relative gains only: up to 23% over state-of-the-art compilers on GH200 and "
                 "up to 42% on RTX 5090 (FP16/FP8, other hardware) -- context, not a target")


def measured_traffic(workload: str):
    """HBM bytes per launch from the committed rocprofv3 counter summaries (profiles/traffic.json names the
    summary each figure comes from); None if the workload has not been measured."""
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            return float(json.load(f)[workload]["hbm_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


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


def timed_steps(step, stream, steps: int, warmup: int, torch) -> dict:
    """`warmup` untimed steps, then exactly `steps` timed ones between two synchronisations, an event before
    the first and one after each (all on the stream the kernels are launched on)."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ev = HipEvents()
    marks = [ev.create() for _ in range(steps + 1)]
    sptr = stream.cuda_stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev.record(marks[0], sptr)
    for i in range(steps):
        step()
        ev.record(marks[i + 1], sptr)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    per = sorted(ev.elapsed_ms(marks[i], marks[i + 1]) for i in range(steps))
    median = per[steps // 2] if steps % 2 else 0.5 * (per[steps // 2 - 1] + per[steps // 2])
    return {"ms_wall": (t1 - t0) * 1e3 / steps, "ms_mean": ev.elapsed_ms(marks[0], marks[steps]) / steps,
            "ms_min": per[0], "ms_median": median}


def kernel_ms_fields(t: dict) -> dict:
    return {"kernel_ms": t["ms_median"], "kernel_ms_min": t["ms_min"], "kernel_ms_median": t["ms_median"],
            "kernel_ms_mean": t["ms_mean"]}


def parity_stats(o_gpu, lse_gpu, o_ref, lse_ref, tol: dict, what: str) -> dict:
    """Error of the GPU rows against the oracle's: the figures of the paper's error table and the acceptance bar."""
    import numpy as np
    d = np.abs(np.asarray(o_gpu, dtype=np.float64) - o_ref)
    dl = np.abs(np.asarray(lse_gpu, dtype=np.float64) - lse_ref) / np.maximum(1.0, np.abs(lse_ref))
    finite = bool(np.isfinite(o_gpu).all() and np.isfinite(lse_gpu).all())
    st = {"rows": int(d.shape[0]), "sample": what, "max_abs": float(d.max()), "mean_abs": float(d.mean()),
          "rms": float(np.sqrt((d * d).mean())), "p90": float(np.percentile(d, 90)), "p99": float(np.percentile(d, 99)),
          "lse_rel": float(dl.max()), "tolerance": tol}
    st["pass"] = bool(finite and st["max_abs"] <= tol["max_abs"] and st["mean_abs"] <= tol["mean_abs"]
                      and st["lse_rel"] <= tol["lse_rel"])
    return st


def structured_rows(w, synth, np):
    """Query rows checked besides the random ones: the first and the last 256-query tile of the first and the
    last (batch, head), the rows on both sides of every 128-row boundary of a middle head, and the rows whose
    diagonal key is one of the scaled K rows (first and last head)."""
    S, nbh = w.S, w.B * w.Hq
    rows = set()
    for bh in (0, nbh - 1):
        rows.update(bh * S + i for i in range(0, min(256, S)))
        rows.update(bh * S + i for i in range(max(0, S - 256), S))
        if w.n_outlier > 0:
            b, h = divmod(bh, w.Hq)
            bhk = b * w.Hkv + h // (w.Hq // w.Hkv)
            rows.update(bh * S + int(i) for i in synth.outlier_rows(bhk, S, synth.workload_seed(w), synth.TAG_K, w.n_outlier))
    mid = nbh // 2
    for t in range(128, S, 128):
        rows.update((mid * S + t - 1, mid * S + t))
    return np.array(sorted(rows), dtype=np.int64)


def cpu_baseline(total_rows: int, run_rows, flops_of_rows, target_seconds: float, cores: int):
    """The oracle, as it stands, timed on this machine's host cores on a bounded sample of query rows.

    A first small batch of rows calibrates the rate; the timed sample is then sized for about
    `target_seconds` of CPU work (each output row is independent, so a row subset is exact).
    Returns the record and the sample (rows, O, LSE), which the parity check reuses.
    """
    import numpy as np
    perm = np.random.default_rng(2604).permutation(total_rows)

    def run(rows):
        rows = np.sort(rows).astype(np.int64)
        t0 = time.perf_counter()
        o, lse = run_rows(rows)
        return time.perf_counter() - t0, rows, o, lse

    n0 = min(512, total_rows)
    dt0 = run(perm[:n0])[0]
    dt_fixed = run(perm[:1])[0]  # the fixed fp64 decode of K and V; the sample is sized from the marginal rate
    rate = max(dt0 - dt_fixed, 1e-3) / n0
    n = int(min(total_rows, max(n0, (target_seconds - dt_fixed) / rate)))
    dt, rows, o, lse = run(perm[:n])
    fl = flops_of_rows(rows)
    rec = {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
           "sample": "%d of %d query rows (uniform, seeded), %.1f s wall incl. fp64 decode of K,V; same FLOP convention"
                     % (n, total_rows, dt), "seconds": dt}
    return rec, (rows, o, lse)


def prefill_parity(args, w, synth, np, oracle_rows, flops_of_rows, o_dev, lse_dev, tol, out, tflops):
    """cpu_baseline (unless switched off) and the check of the timed buffers; fills `out`; returns pass/fail."""
    import oracle
    total = w.B * w.Hq * w.S
    sample = None
    if args.cpu_seconds > 0:
        cb, sample = cpu_baseline(total, oracle_rows, flops_of_rows, args.cpu_seconds, int(oracle.threads()))
        cb["gpu_over_cpu"] = tflops / cb["value"]
        out["cpu_baseline"] = cb
    rows_s = structured_rows(w, synth, np)
    if sample is None:
        extra = np.random.default_rng(2604).permutation(total)[:1024]
        rows_s = np.unique(np.concatenate([rows_s, extra]))
        what = "%d structured + random rows" % len(rows_s)
    else:
        rows_s = np.setdiff1d(rows_s, sample[0])
        what = "the %d rows of the cpu_baseline sample + %d structured rows (first/last tiles, tile boundaries, outlier diagonals)" \
               % (len(sample[0]), len(rows_s))
    o_s, lse_s = oracle_rows(rows_s)
    if sample is not None:
        rows = np.concatenate([sample[0], rows_s])
        o_ref, lse_ref = np.concatenate([sample[1], o_s]), np.concatenate([sample[2], lse_s])
    else:
        rows, o_ref, lse_ref = rows_s, o_s, lse_s
    import torch
    idx = torch.from_numpy(rows).to(o_dev.device)
    o_gpu = o_dev.reshape(-1, w.D).index_select(0, idx).double().cpu().numpy()
    lse_gpu = lse_dev.reshape(-1).index_select(0, idx).double().cpu().numpy()
    out["parity"] = parity_stats(o_gpu, lse_gpu, o_ref, lse_ref, tol, what)
    return out["parity"]["pass"]


def fp8_tolerance(v_bits, dv, np):
    """Both sides see identical bytes and the first product is exact in fp32; P is rounded to E4M3 (relative
    2^-4) before the second product, so |dO| <= 2^-4 max|V| plus the bf16 rounding of O: checked as
    0.07 max|V|; the roundings are unbiased and independent, so the mean must stay below 1e-2 rms(V); l is
    summed from the unrounded P, so lse keeps the 16-bit bound."""
    import oracle
    vv = dv * oracle.decode_e4m3(v_bits)
    return {"max_abs": float(0.07 * np.abs(vv).max()), "mean_abs": float(1e-2 * np.sqrt((vv * vv).mean())), "lse_rel": 1e-3}


def bench_fp8(args, nb, synth, torch, np) -> int:
    """The long shape on FP8 (E4M3) inputs with per-tensor scales; one step = one naut_attn_fwd_fp8 call."""
    w = synth.WORKLOADS["long"]
    seed = synth.workload_seed(w)
    dq, dk, dv = FP8_DESCALE["q"], FP8_DESCALE["k"], FP8_DESCALE["v"]
    q = synth.fill_e4m3(w.B, w.Hq, w.S, w.D, seed, synth.TAG_Q, dq)
    k = synth.fill_e4m3(w.B, w.Hkv, w.S, w.D, seed, synth.TAG_K, dk, w.n_outlier, w.outlier_scale)
    v = synth.fill_e4m3(w.B, w.Hkv, w.S, w.D, seed, synth.TAG_V, dv)
    qd, kd, vd = (torch.from_numpy(a).cuda() for a in (q, k, v))
    o = torch.full((w.B, w.Hq, w.S, w.D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((w.B, w.Hq, w.S), float("nan"), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        nb.naut_attn_fwd_fp8(qd, kd, vd, o, lse, w.causal, w.scale, dq, dk, dv, stream=stream)

    t = timed_steps(step, stream, args.steps, args.warmup, torch)
    flops = w.flops
    nq, nkv = w.B * w.Hq * w.S * w.D, w.B * w.Hkv * w.S * w.D
    io_bytes = nq + 2 * nkv + nq * 2 + w.B * w.Hq * w.S * 4
    achieved = flops / (t["ms_median"] * 1e-3) / 1e12
    tflops = flops / (t["ms_wall"] * 1e-3) / 1e12
    roof = {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP8_TFLOPS, "unit": "TFLOP/s",
            "frac": achieved / PEAK_FP8_TFLOPS, "traffic": measured_traffic("long_fp8"),
            "algorithmic_hbm_bytes": io_bytes}
    roof.update(kernel_ms_fields(t))
    out = {
        "metric": "attention fwd TFLOP/s, FP8 E4M3 inputs (S=16k causal D=128)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t["ms_wall"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8_e4m3", "data": "synthetic",
        "config": {"workload": "long_fp8", "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "S": w.S, "D": w.D, "causal": w.causal,
                   "outlier_k_rows": w.n_outlier, "descale": FP8_DESCALE, "kernel": "fwd_fp8_bm128_w4q32_bn64",
                   "flop_convention": "4*B*Hq*S^2*D, halved for causal"},
        "roofline": roof, "context": PAPER_CONTEXT,
    }
    import oracle
    ok = prefill_parity(args, w, synth, np,
                        lambda rows: oracle.attn_rows_e4m3(q, k, v, dq, dk, dv, w.causal, w.scale, rows=rows),
                        lambda rows: float((4.0 * w.D * ((rows % w.S) + 1)).sum()), o, lse, fp8_tolerance(v, dv, np),
                        out, tflops)
    print(json.dumps(out))
    return 0 if ok else 4


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
    o = torch.full((B, Hq, Sq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(nb.decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    scale = D ** -0.5

    def step():
        if fp8:
            nb.naut_attn_decode_fp8(qd, kd, vd, o, lse, True, scale, FP8_DESCALE["q"], FP8_DESCALE["k"],
                                    FP8_DESCALE["v"], ws, stream=stream)
        else:
            nb.naut_attn_decode(qd, kd, vd, o, lse, True, scale, ws, stream=stream)

    t = timed_steps(step, stream, args.steps, args.warmup, torch)
    # algorithmic bytes: Q, K, V read once; O and LSE written once (the partials in the workspace are extra)
    in_b = 1 if fp8 else 2
    nbytes = (B * Hq * Sq * D + 2 * B * Hkv * Sk * D) * in_b + B * Hq * Sq * D * 2 + B * Hq * Sq * 4
    name = "decode_fp8" if fp8 else "decode"
    achieved = nbytes / (t["ms_median"] * 1e-3) / 1e9
    roof = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS,
            "traffic": measured_traffic(name), "algorithmic_hbm_bytes": nbytes}
    roof.update(kernel_ms_fields(t))
    out = {
        "metric": "decode attention GB/s (B=8, 32/8 heads, Sk=16k, D=128)" + (", FP8 E4M3 cache" if fp8 else ""),
        "value": nbytes / (t["ms_wall"] * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": t["ms_wall"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "fp8_e4m3" if fp8 else "bf16", "data": "synthetic",
        "config": {"workload": name, "B": B, "Hq": Hq, "Hkv": Hkv, "Sq": Sq, "Sk": Sk, "D": D, "causal": True,
                   "outlier_k_rows": int(c["outlier_frac"] * Sk),
                   "kernel": "decode_split_fp8_32x32x64 + merge" if fp8 else "decode_split32x32 + merge",
                   "workspace_bytes": int(ws.numel())},
        "roofline": roof, "context": PAPER_CONTEXT,
    }
    # The whole workload is well under a second of CPU work: the oracle computes all of it, once, timed, and the
    # timed buffers are compared with all of it.
    import oracle
    t0 = time.perf_counter()
    if fp8:
        o_ref, lse_ref = oracle.attn_cross_e4m3(q, k, v, FP8_DESCALE["q"], FP8_DESCALE["k"], FP8_DESCALE["v"], True, scale)
        tol = fp8_tolerance(v, FP8_DESCALE["v"], np)
    else:
        o_ref, lse_ref = oracle.attn_cross16(q, k, v, synth.BF16, True, scale)
        tol = TOL_16BIT
    dt = time.perf_counter() - t0
    out["cpu_baseline"] = {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": int(oracle.threads()), "kind": "oracle",
                           "sample": "all %d batch entries, %.2f s wall incl. fp64 decode of K,V" % (B, dt), "seconds": dt}
    out["parity"] = parity_stats(o.double().cpu().numpy().reshape(-1, D), lse.double().cpu().numpy().reshape(-1),
                                 o_ref.reshape(-1, D), lse_ref.reshape(-1), tol, "every output row")
    print(json.dumps(out))
    return 0 if out["parity"]["pass"] else 4


def mfma_ceiling(nb, torch, work_groups: int, min_ms: float = 50.0) -> dict:
    """What the matrix pipes of this box sustain on the bf16 kernels' MFMA instruction alone (a register-only
    loop, naut_probe_mfma), on all-zero operands and on random-valued ones, each run for at least `min_ms`."""
    out_buf = torch.empty(work_groups * 512, dtype=torch.float32, device="cuda")
    res = {}
    for kind, name in ((0, "zero_operands"), (1, "random_operands")):
        trips = 4000
        nb.naut_probe_mfma(out_buf, work_groups, trips, kind)
        torch.cuda.synchronize()
        while True:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fl = nb.naut_probe_mfma(out_buf, work_groups, trips, kind)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            if ms >= min_ms:
                break
            trips = int(trips * max(2.0, 1.2 * min_ms / max(ms, 1e-3)))
        tf = fl / (ms * 1e-3) / 1e12
        res[name] = {"tflops": tf, "ms": ms, "implied_clock_ghz": tf * 1e12 / (work_groups * 4096.0) / 1e9}
    res["instruction"] = "v_mfma_f32_32x32x16_bf16"
    res["work_groups"] = work_groups
    return res


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
                    help="seconds of CPU work the oracle baseline sample is sized for (0 = no cpu_baseline; the "
                         "parity check then uses a small sample of its own)")
    ap.add_argument("--cpu-rows", type=int, default=None, help="deprecated spelling: 0 means --cpu-seconds 0")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="only run a plain device copy of this many MiB (5 times): the known-size kernel "
                         "against which rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled")
    ap.add_argument("--calibrate-mfma", action="store_true",
                    help="only run the register-only MFMA loop (zero and random-valued operands, >= 50 ms each) "
                         "and print the sustained rates beside the published peak")
    ap.add_argument("--no-mfma-ceiling", action="store_true",
                    help="do not run the register-only MFMA loop after the timed region (profiler runs)")
    args = ap.parse_args()
    if args.cpu_rows == 0:
        args.cpu_seconds = 0.0
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
    ncu = torch.cuda.get_device_properties(0).multi_processor_count

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
    if args.calibrate_mfma:
        # on every compute unit, and on half of them: the second shows what one compute unit sustains when the
        # chip's power budget is shared by fewer of them
        res = {"all_compute_units": mfma_ceiling(nb, torch, ncu), "half_the_compute_units": mfma_ceiling(nb, torch, ncu // 2),
               "published_peak_tflops": PEAK_BF16_TFLOPS, "compute_units": ncu}
        print(json.dumps({"calibrate_mfma": res}))
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
    # NaN-filled: an output tile that a launch does not write shows up in the parity check
    o = torch.full((w.B, w.Hq, w.S, w.D), float("nan"), dtype=tdt[w.out_dtype], device="cuda")
    lse = torch.full((w.B, w.Hq, w.S), float("nan"), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        nb.naut_attn_fwd(qd, kd, vd, o, lse, w.causal, w.scale, stream=stream)

    t = timed_steps(step, stream, args.steps, args.warmup, torch)
    flops = w.flops
    tflops = flops / (t["ms_wall"] * 1e-3) / 1e12
    achieved = flops / (t["ms_median"] * 1e-3) / 1e12  # the median launch, measured on the launch stream
    variant = nb.variant_name(w.B, w.Hq, w.S, w.D, w.causal, w.in_dtype, w.out_dtype)
    roof = {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": achieved / PEAK_BF16_TFLOPS, "traffic": measured_traffic(w.name),
            "algorithmic_hbm_bytes": w.io_bytes}
    roof.update(kernel_ms_fields(t))
    out = {
        "metric": "attention fwd TFLOP/s (S=16k causal D=128)" if w.name == "long" else "attention fwd TFLOP/s",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": t["ms_wall"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.in_dtype == synth.BF16 else "f16", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "S": w.S, "D": w.D,
                   "causal": w.causal, "outlier_k_rows": w.n_outlier, "kernel": variant,
                   "flop_convention": "4*B*Hq*S^2*D, halved for causal",
                   "pct_of_bf16_mfma_peak": 100.0 * tflops / PEAK_BF16_TFLOPS},
        "roofline": roof, "context": PAPER_CONTEXT,
    }
    if not args.no_mfma_ceiling:
        # after the timed region, on the same box: the rate the MFMA instruction alone sustains here
        ceil = mfma_ceiling(nb, torch, ncu)
        roof["measured_mfma_ceiling"] = ceil
        roof["frac_of_measured_ceiling_random_operands"] = achieved / ceil["random_operands"]["tflops"]
    import oracle
    keys = lambda rows: (rows % w.S) + 1 if w.causal else np.full(rows.shape, w.S)
    ok = prefill_parity(args, w, synth, np,
                        lambda rows: oracle.attn_rows(q, k, v, w.in_dtype, w.causal, w.scale, rows=rows),
                        lambda rows: float((4.0 * w.D * keys(rows)).sum()), o, lse, TOL_16BIT, out, tflops)
    print(json.dumps(out))
    if not ok:
        print("bench.py: the timed output misses the acceptance bar: %s" % json.dumps(out["parity"]), file=sys.stderr)
        return 4
    return 0


if __name__ == "__main__":
    sys.exit(main())
