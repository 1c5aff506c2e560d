"""GPU parity of the FP8 (E4M3) attention forward (through the C ABI) against the fp64 oracle on identical bytes.

Tolerance.  The inputs are exact E4M3 values for both sides and the first product accumulates them in fp32, so
the only FP8-specific error is the rounding of P to E4M3 (3 fraction bits: relative error at most 2^-4) before
the second product: |dO_d| <= 2^-4 * sum_j P_ij |v_jd| <= 2^-4 * max|V|, plus the bf16 rounding of O (2^-9 |O|).
The hard bound checked is 0.07 * max|V|; the roundings are unbiased and independent across keys, so the typical
error is far smaller (about 2^-4/sqrt(3) * sqrt(sum_j P_ij^2) * rms(V)), and the mean is required to stay below
1e-2 * rms(V).  l is summed from the unrounded P, so lse keeps the 16-bit paths' bound (1e-3 relative).
"""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2604_14825_amd import binding as nb
from paper_2604_14825_amd import synth

pytestmark = pytest.mark.gpu

DQ, DK, DV = 1.0 / 64, 1.0 / 8, 1.0 / 64   # per-tensor scales of the synthetic inputs


def make(B, Hq, Hkv, S, D, seed, n_outlier=0):
    q = synth.fill_e4m3(B, Hq, S, D, seed, synth.TAG_Q, DQ)
    k = synth.fill_e4m3(B, Hkv, S, D, seed, synth.TAG_K, DK, n_outlier, 8.0)
    v = synth.fill_e4m3(B, Hkv, S, D, seed, synth.TAG_V, DV)
    return q, k, v


def run(q, k, v, causal, scale, want_lse=True):
    B, Hq, S, D = q.shape
    dev = lambda a: torch.from_numpy(a).cuda()
    o = torch.full((B, Hq, S, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((B, Hq, S), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    nb.naut_attn_fwd_fp8(dev(q), dev(k), dev(v), o, lse, causal, scale, DQ, DK, DV)
    torch.cuda.synchronize()
    return o.double().cpu().numpy(), (lse.double().cpu().numpy() if want_lse else None)


def check(o, lse, o_ref, lse_ref, v_bits, what):
    vmax = DV * np.abs(oracle.decode_e4m3(v_bits)).max()
    vrms = DV * math.sqrt((oracle.decode_e4m3(v_bits) ** 2).mean())
    d = np.abs(o - o_ref)
    print("%s: max|dO| %.3e (bound %.3e) mean|dO| %.3e (bound %.3e)" % (what, d.max(), 0.07 * vmax, d.mean(), 1e-2 * vrms),
          flush=True)
    assert np.isfinite(o).all(), what + ": non-finite O"
    assert d.max() <= 0.07 * vmax, "%s: max|dO| = %.3e" % (what, d.max())
    assert d.mean() <= 1e-2 * vrms, "%s: mean|dO| = %.3e" % (what, d.mean())
    if lse is not None:
        assert np.isfinite(lse).all(), what + ": non-finite lse"
        dl = np.abs(lse - lse_ref) / np.maximum(1.0, np.abs(lse_ref))
        assert dl.max() <= 1e-3, "%s: lse rel err = %.3e" % (what, dl.max())


CASES = [
    (1, 1, 1, 1, 64, False), (1, 2, 1, 7, 128, True), (2, 2, 2, 63, 128, True), (1, 2, 2, 64, 64, False),
    (1, 2, 2, 65, 128, False), (2, 4, 2, 129, 128, True), (1, 3, 1, 200, 64, True), (1, 2, 2, 257, 128, False),
    (1, 8, 2, 400, 128, True), (1, 2, 1, 777, 64, False), (1, 4, 4, 1024, 128, True),
]


@pytest.mark.parametrize("B,Hq,Hkv,S,D,causal", CASES)
def test_fp8_small_shapes_elementwise(B, Hq, Hkv, S, D, causal):
    q, k, v = make(B, Hq, Hkv, S, D, 11000 + S + D, S // 50)
    scale = 1.0 / math.sqrt(D)
    print("fp8 case", B, Hq, Hkv, S, D, causal, flush=True)
    o, lse = run(q, k, v, causal, scale)
    o_ref, lse_ref = oracle.attn_rows_e4m3(q, k, v, DQ, DK, DV, causal, scale)
    check(o, lse, o_ref, lse_ref, v, "fp8 small")


def test_fp8_prefill_size_sampled_rows():
    B, Hq, Hkv, S, D = 2, 32, 32, 4096, 128
    q, k, v = make(B, Hq, Hkv, S, D, 11111, S // 100)
    scale = 1.0 / math.sqrt(D)
    o, lse = run(q, k, v, True, scale)
    g = np.random.default_rng(5)
    rows = np.unique(np.concatenate([np.arange(0, 130), np.arange(B * Hq * S - 130, B * Hq * S),
                                     g.integers(0, B * Hq * S, 1500)])).astype(np.int64)
    o_ref, lse_ref = oracle.attn_rows_e4m3(q, k, v, DQ, DK, DV, True, scale, rows=rows)
    check(o.reshape(-1, D)[rows], lse.reshape(-1)[rows], o_ref, lse_ref, v, "fp8 prefill")


def test_fp8_growing_keys_and_bit_identity():
    B, Hq, Hkv, S, D = 1, 4, 2, 700, 128
    q, k, v = make(B, Hq, Hkv, S, D, 11222)
    kf = oracle.decode_e4m3(k) * (0.1 + 2.4 * np.arange(S) / (S - 1))[None, None, :, None]   # stays within +-448
    k = synth.round_e4m3(kf.astype(np.float32))
    scale = 1.0 / math.sqrt(D)
    o, lse = run(q, k, v, True, scale)
    o2, _ = run(q, k, v, True, scale, want_lse=False)
    assert np.array_equal(o, o2)
    o_ref, lse_ref = oracle.attn_rows_e4m3(q, k, v, DQ, DK, DV, True, scale)
    check(o, lse, o_ref, lse_ref, v, "fp8 ascending keys")


@pytest.mark.parametrize("pad", [32, 4])
@pytest.mark.parametrize("B,Hq,Hkv,S,D,causal", [(2, 6, 2, 300, 128, True), (1, 4, 4, 777, 64, False),
                                                 (2, 8, 2, 129, 128, False)])
def test_fp8_sequence_major_layout(B, Hq, Hkv, S, D, causal, pad):
    """Tensors stored [B][S][H][D], passed as transposed views; O (rows padded to a wider pitch) written in the
    same layout, its gaps untouched.  pad = 4: O rows start on 8-byte boundaries only, the least the entry point
    accepts (the kernel writes O in 16-byte pieces)."""
    q, k, v = make(B, Hq, Hkv, S, D, 11300 + S + D, S // 50)
    scale = 1.0 / math.sqrt(D)
    bshd = lambda a: torch.from_numpy(np.ascontiguousarray(a.transpose(0, 2, 1, 3))).cuda().transpose(1, 2)
    qd, kd, vd = bshd(q), bshd(k), bshd(v)
    assert not kd.is_contiguous()
    P = D + pad
    o_mem = torch.full((B, S, Hq, P), 7.0, dtype=torch.bfloat16, device="cuda")
    od = o_mem[..., :D].transpose(1, 2)
    lse = torch.full((B, Hq, S), float("nan"), dtype=torch.float32, device="cuda")
    print("fp8 bshd", B, Hq, Hkv, S, D, causal, flush=True)
    nb.naut_attn_fwd_fp8_strided(qd, kd, vd, od, lse, causal, scale, DQ, DK, DV)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attn_rows_e4m3(q, k, v, DQ, DK, DV, causal, scale)
    check(od.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, v, "fp8 bshd")
    assert torch.all(o_mem[..., D:] == 7.0).item(), "the gaps between O rows were written"


DEC_CASES = [
    # B, Hq, Hkv, Sq, Sk, D, causal
    (1, 1, 1, 1, 1, 64, False), (1, 2, 2, 1, 63, 128, True), (1, 4, 4, 1, 100, 128, True),
    (2, 8, 2, 1, 777, 128, True), (1, 8, 1, 3, 500, 64, True), (1, 16, 2, 5, 300, 128, True),
    (1, 2, 2, 1, 4096, 128, False), (1, 2, 1, 64, 64, 64, True), (3, 6, 3, 2, 2049, 128, True),
]


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D,causal", DEC_CASES)
def test_fp8_decode_elementwise(B, Hq, Hkv, Sq, Sk, D, causal):
    """Decode-time attention on an FP8 K/V cache against the fp64 oracle on the same bytes."""
    q = synth.fill_e4m3(B, Hq, Sq, D, 11500 + Sk + D, synth.TAG_Q, DQ)
    k = synth.fill_e4m3(B, Hkv, Sk, D, 11500 + Sk + D, synth.TAG_K, DK, Sk // 50, 8.0)
    v = synth.fill_e4m3(B, Hkv, Sk, D, 11500 + Sk + D, synth.TAG_V, DV)
    scale = 1.0 / math.sqrt(D)
    dev = lambda a: torch.from_numpy(a).cuda()
    o = torch.full((B, Hq, Sq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(nb.decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    print("fp8 decode", B, Hq, Hkv, Sq, Sk, D, causal, flush=True)
    nb.naut_attn_decode_fp8(dev(q), dev(k), dev(v), o, lse, causal, scale, DQ, DK, DV, ws)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attn_cross_e4m3(q, k, v, DQ, DK, DV, causal, scale)
    check(o.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, v, "fp8 decode")
