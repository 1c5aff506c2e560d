"""Helpers shared by the GPU parity tests: run the HIP path on synth bit patterns, compare with the oracle."""
import numpy as np
import torch

import oracle
from paper_2604_14825_amd import binding as nb
from paper_2604_14825_amd import synth

TORCH_DT = {synth.BF16: torch.bfloat16, synth.F16: torch.float16, synth.F32: torch.float32}

# Acceptance bar for bf16/fp16 inputs: max |dO| <= 2e-2, mean |dO| <= 2e-3, lse within 1e-3 relative
# (read as |d| <= 1e-3 * max(1, |lse|), since a relative bound is meaningless near zero).
TOL_MAX, TOL_MEAN, TOL_LSE = 2e-2, 2e-3, 1e-3


def to_device(bits: np.ndarray, dtype: int) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda().view(TORCH_DT[dtype])


def run_hip(q, k, v, in_dtype, out_dtype, causal, scale, want_lse=True):
    """q,k,v: uint16 numpy arrays. Returns (o fp64 numpy [B,Hq,S,D], lse fp64 numpy [B,Hq,S])."""
    qd, kd, vd = (to_device(a, in_dtype) for a in (q, k, v))
    B, Hq, S, D = q.shape
    o = torch.full((B, Hq, S, D), float("nan"), dtype=TORCH_DT[out_dtype], device="cuda")
    lse = torch.full((B, Hq, S), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    nb.naut_attn_fwd(qd, kd, vd, o, lse, causal, scale)
    torch.cuda.synchronize()
    return o.double().cpu().numpy(), (lse.double().cpu().numpy() if want_lse else None)


def check(o_gpu, lse_gpu, o_ref, lse_ref, what=""):
    d = np.abs(o_gpu - o_ref)
    assert np.isfinite(o_gpu).all(), what + ": non-finite O"
    assert d.max() <= TOL_MAX, "%s: max|dO| = %.3e" % (what, d.max())
    assert d.mean() <= TOL_MEAN, "%s: mean|dO| = %.3e" % (what, d.mean())
    if lse_gpu is not None:
        assert np.isfinite(lse_gpu).all(), what + ": non-finite lse"
        dl = np.abs(lse_gpu - lse_ref) / np.maximum(1.0, np.abs(lse_ref))
        assert dl.max() <= TOL_LSE, "%s: lse rel err = %.3e" % (what, dl.max())
    return float(d.max()), float(d.mean())


def sample_rows(w, n_random, seed, bm=128):
    """Row ids for a full-size check: first/last query tiles of the first and last (b,h), the rows on
    both sides of every tile boundary for one head, and n_random uniformly drawn rows."""
    S = w.S
    nbh = w.B * w.Hq
    g = np.random.default_rng(seed)
    rows = set()
    for bh in (0, nbh - 1):
        for i in list(range(0, min(bm, S))) + list(range(max(0, S - bm), S)):
            rows.add(bh * S + i)
    bh = nbh // 2
    for t in range(bm, S, bm):
        rows.add(bh * S + t - 1)
        rows.add(bh * S + t)
    for r in g.integers(0, nbh * S, n_random):
        rows.add(int(r))
    return np.array(sorted(rows), dtype=np.int64)


def run_hip_decode(q, k, v, in_dtype, out_dtype, causal, scale, want_lse=True, poison_workspace=True):
    """Decode-time attention through the C ABI.  q [B,Hq,Sq,D], k,v [B,Hkv,Sk,D] uint16 numpy arrays."""
    qd, kd, vd = (to_device(a, in_dtype) for a in (q, k, v))
    B, Hq, Sq, D = q.shape
    Hkv, Sk = k.shape[1], k.shape[2]
    o = torch.full((B, Hq, Sq, D), float("nan"), dtype=TORCH_DT[out_dtype], device="cuda")
    lse = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    nbytes = nb.decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D)
    assert nbytes > 0
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    if poison_workspace:
        ws.fill_(0xFF)  # NaN patterns: every partial the merge reads must have been written by the first kernel
    nb.naut_attn_decode(qd, kd, vd, o, lse, causal, scale, ws)
    torch.cuda.synchronize()
    return o.double().cpu().numpy(), (lse.double().cpu().numpy() if want_lse else None)
