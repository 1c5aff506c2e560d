"""GPU parity of the FP8 (E4M3) attention forward (through the C ABI) against the fp64 oracle on identical bytes.

Tolerance.  The inputs are exact E4M3 values for both sides and the first product accumulates them in fp32, so
the only FP8-specific error is the rounding of P to E4M3 (3 fraction bits: relative error at most 2^-4) before
the second product: |dO_d| <= 2^-4 * sum_j P_ij |v_jd| <= 2^-4 * max|V|, plus the bf16 rounding of O (2^-9 |O|).
The hard bound checked is 0.07 * max|V|; the roundings are unbiased and independent across keys, so the typical
error is far smaller (about 2^-4/sqrt(3) * sqrt(sum_j P_ij^2) * rms(V)), and the mean is required to stay below
1e-2 * rms(V).  l is summed from the unrounded P, so lse keeps the 16-bit paths' bound (1e-3 relative).

The worst-case bound alone would let a wrong contribution of a single key through (a key of weight 0.05 and
|v| = 3.4 moves O by 0.17, below 0.07 * max|V|), so the same error model is also applied element by element:
with weights w_ij = exp(s_ij - lse_i) the error of O_id is a sum of independent terms, one per key, each at
most 2^-4 w_ij |v_jd| and of either sign, so its standard deviation is at most
    sigma_id = sqrt( (2^-4)^2/3 * sum_j w_ij^2 v_jd^2  +  n_i * (2^-16)^2/12 * mean(v^2)  +  (2^-9 O_id)^2/3 )
(second term: weights below 2^-13 of the row's largest fall into E4M3's subnormal range, where the rounding
error is a fixed 2^-9 * 2^-7; third term: O's own rounding to bf16).  sigma uses the largest relative error
of a binade for every term, so a correct kernel stays well below one: checked on z = dO/sigma are
rms(z) <= 0.85, the 99th percentile of |z| <= 2.2 and max|z| <= 4.5 (a correct kernel measures up to 0.62,
1.67 and 3.2 over all cases here) -- a dropped, duplicated or misplaced key of weight w shows up as
|z| ~ 28 w|v| / sqrt(sum_j w_j^2 v_j^2), far outside.
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


def error_sigma(q_bits, k_bits, v_bits, o_ref, lse_ref, causal, scale, rows=None):
    """sigma_id of the file header for the rows checked (all of them if rows is None); q may be shorter than k
    (decode: its rows are the last positions).  o_ref, lse_ref: the oracle's, [n, D] and [n] or full-shaped."""
    B, Hq, Sq, D = q_bits.shape
    Hkv, Sk = k_bits.shape[1], k_bits.shape[2]
    qf, kf, vf = DQ * oracle.decode_e4m3(q_bits), DK * oracle.decode_e4m3(k_bits), DV * oracle.decode_e4m3(v_bits)
    if rows is None:
        rows = np.arange(B * Hq * Sq, dtype=np.int64)
    o_ref = np.asarray(o_ref).reshape(-1, D)
    lse_ref = np.asarray(lse_ref).reshape(-1)
    sig = np.empty((len(rows), D))
    bh = rows // Sq
    for x in np.unique(bh):
        sel = np.nonzero(bh == x)[0]
        i = rows[sel] % Sq
        b, h = divmod(int(x), Hq)
        hk = h // (Hq // Hkv)
        s_ = scale * (qf[b, h][i] @ kf[b, hk].T)
        lim = (Sk - Sq + i) if causal else np.full_like(i, Sk - 1)
        alive = np.arange(Sk)[None, :] <= lim[:, None]
        w = np.where(alive, np.exp(s_ - lse_ref[sel][:, None]), 0.0)
        v2 = vf[b, hk] ** 2
        var = (2.0 ** -4) ** 2 / 3 * ((w * w) @ v2)
        var += (lim + 1)[:, None] * (2.0 ** -16) ** 2 / 12 * v2.mean()
        var += (2.0 ** -9 * o_ref[sel]) ** 2 / 3
        sig[sel] = np.sqrt(var)
    return sig


def check(o, lse, o_ref, lse_ref, v_bits, what, sigma=None):
    if sigma is not None:
        z = np.abs((np.asarray(o).reshape(sigma.shape) - np.asarray(o_ref).reshape(sigma.shape)) / sigma)
        zr, z99, zm = math.sqrt((z * z).mean()), np.percentile(z, 99), z.max()
        print("%s: z = dO/sigma: rms %.3f p99 %.3f max %.3f" % (what, zr, z99, zm), flush=True)
        assert zr <= 0.85 and z99 <= 2.2 and zm <= 4.5, "%s: rms(z) %.3f p99 %.3f max %.3f" % (what, zr, z99, zm)
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
    check(o, lse, o_ref, lse_ref, v, "fp8 small", error_sigma(q, k, v, o_ref, lse_ref, causal, scale))


def test_fp8_prefill_size_sampled_rows():
    B, Hq, Hkv, S, D = 2, 32, 32, 4096, 128
    q, k, v = make(B, Hq, Hkv, S, D, 11111, S // 100)
    scale = 1.0 / math.sqrt(D)
    o, lse = run(q, k, v, True, scale)
    g = np.random.default_rng(5)
    rows = np.unique(np.concatenate([np.arange(0, 130), np.arange(B * Hq * S - 130, B * Hq * S),
                                     g.integers(0, B * Hq * S, 1500)])).astype(np.int64)
    o_ref, lse_ref = oracle.attn_rows_e4m3(q, k, v, DQ, DK, DV, True, scale, rows=rows)
    check(o.reshape(-1, D)[rows], lse.reshape(-1)[rows], o_ref, lse_ref, v, "fp8 prefill",
          error_sigma(q, k, v, o_ref, lse_ref, True, scale, rows))


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
    check(o, lse, o_ref, lse_ref, v, "fp8 ascending keys", error_sigma(q, k, v, o_ref, lse_ref, True, scale))


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
    check(od.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, v, "fp8 bshd",
          error_sigma(q, k, v, o_ref, lse_ref, causal, scale))
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
    check(o.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, v, "fp8 decode",
          error_sigma(q, k, v, o_ref, lse_ref, causal, scale))


def planted_key(B, Hq, Hkv, Sq, Sk, D, seed, weight=0.05, vmag=3.5):
    """Inputs in which one key of every K/V head carries about `weight` of every query's softmax and a value row
    of magnitude `vmag` (the other values are N(0,1)): all queries share a component a*u (u a fixed sign vector),
    that key is b*u, and b is set from the scores of the other keys so that exp(s*) = weight/(1-weight) of their sum."""
    g = np.random.default_rng(seed)
    u = g.choice([-1.0, 1.0], size=D)
    a = 0.5
    qf = a * u + g.standard_normal((B, Hq, Sq, D))
    kf = g.standard_normal((B, Hkv, Sk, D))
    vf = g.standard_normal((B, Hkv, Sk, D))
    scale = 1.0 / math.sqrt(D)
    jstar = Sk // 3
    # sum over the other keys of exp(score) ~ Sk * exp(var/2), var = scale^2 |q|^2 ~ a^2 + 1
    target = math.log(weight / (1 - weight) * Sk) + 0.5 * (a * a + 1)
    b = target / (scale * D * a)
    kf[:, :, jstar, :] = b * u
    vf[:, :, jstar, :] = vmag * g.choice([-1.0, 1.0], size=D)
    r8 = lambda x, d: synth.round_e4m3((x / d).astype(np.float32))
    return r8(qf, DQ), r8(kf, DK), r8(vf, DV), scale, jstar


@pytest.mark.parametrize("D", [128, 64])
def test_fp8_one_key_of_weight_a_twentieth_with_a_large_value(D):
    """A single key with about 5 % of every row's weight and |v| = 3.5 in every column: its contribution to O
    (0.17) is below the worst-case bound, so only the element-wise model can tell whether it was dropped,
    counted twice or given the wrong value row.  The oracle run without that key must fail the same check."""
    B, Hq, Hkv, S = 1, 4, 2, 512
    q, k, v, scale, jstar = planted_key(B, Hq, Hkv, S, S, D, 11700 + D)
    o, lse = run(q, k, v, False, scale)
    o_ref, lse_ref = oracle.attn_rows_e4m3(q, k, v, DQ, DK, DV, False, scale)
    w = np.exp(scale * DQ * DK * np.einsum("bhid,bhd->bhi", oracle.decode_e4m3(q),
                                          np.repeat(oracle.decode_e4m3(k)[:, :, jstar], Hq // Hkv, axis=1)) - lse_ref)
    print("weight of the planted key: median %.3f (%.3f .. %.3f)" % (np.median(w), w.min(), w.max()), flush=True)
    assert 0.02 < np.median(w) < 0.12
    sigma = error_sigma(q, k, v, o_ref, lse_ref, False, scale)
    check(o, lse, o_ref, lse_ref, v, "fp8 planted key", sigma)
    # the check has teeth: the exact result for the inputs without that key (its score pushed out of reach) fails it
    k_wo = k.copy()
    k_wo[:, :, jstar, :] = synth.round_e4m3((-oracle.decode_e4m3(k[:, :, jstar, :])).astype(np.float32))
    o_wo, _ = oracle.attn_rows_e4m3(q, k_wo, v, DQ, DK, DV, False, scale)
    z = np.abs((o_wo - o_ref).reshape(sigma.shape) / sigma)
    assert np.percentile(z, 99) > 2.2 and z.max() > 4.5


def test_fp8_decode_one_key_of_weight_a_twentieth_with_a_large_value():
    B, Hq, Hkv, Sq, Sk, D = 2, 8, 2, 1, 1024, 128
    q, k, v, scale, jstar = planted_key(B, Hq, Hkv, Sq, Sk, D, 11800)
    dev = lambda a: torch.from_numpy(a).cuda()
    o = torch.full((B, Hq, Sq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(nb.decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D), dtype=torch.uint8, device="cuda")
    nb.naut_attn_decode_fp8(dev(q), dev(k), dev(v), o, lse, True, scale, DQ, DK, DV, ws)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attn_cross_e4m3(q, k, v, DQ, DK, DV, True, scale)
    check(o.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, v, "fp8 decode planted key",
          error_sigma(q, k, v, o_ref, lse_ref, True, scale))


NARROW = [(1, 2, 2, 200, 16, True), (2, 4, 2, 129, 32, False), (1, 3, 1, 300, 48, True), (1, 4, 2, 257, 80, True),
          (2, 2, 2, 130, 96, False), (1, 8, 2, 400, 112, True)]


@pytest.mark.parametrize("B,Hq,Hkv,S,D,causal", NARROW)
def test_fp8_head_dimensions_between_the_compiled_ones(B, Hq, Hkv, S, D, causal):
    """D = 16k below 64 or 128 runs on the next wider kernel; contiguous tensors, so a chunk read past a row's end
    would show up as the next row's data.  O is checked with a guard band behind every row's D columns."""
    q, k, v = make(B, Hq, Hkv, S, D, 11900 + S + D, S // 50)
    scale = 1.0 / math.sqrt(D)
    print("fp8 narrow head", B, Hq, Hkv, S, D, causal, flush=True)
    o, lse = run(q, k, v, causal, scale)
    o_ref, lse_ref = oracle.attn_rows_e4m3(q, k, v, DQ, DK, DV, causal, scale)
    check(o, lse, o_ref, lse_ref, v, "fp8 narrow head", error_sigma(q, k, v, o_ref, lse_ref, causal, scale))
    # the same through padded O rows: nothing may be written behind column D
    dev = lambda a: torch.from_numpy(a).cuda()
    o_mem = torch.full((B, Hq, S, D + 8), 7.0, dtype=torch.bfloat16, device="cuda")
    od = o_mem[..., :D]
    nb.naut_attn_fwd_fp8_strided(dev(q), dev(k), dev(v), od, None, causal, scale, DQ, DK, DV)
    torch.cuda.synchronize()
    assert np.array_equal(od.double().cpu().numpy(), o)
    assert torch.all(o_mem[..., D:] == 7.0).item(), "columns behind D were written"


DEC_STRIDED = [(2, 8, 2, 1, 777, 128, True), (1, 16, 2, 5, 300, 64, True), (1, 4, 4, 1, 1000, 96, False),
               (2, 6, 3, 2, 513, 48, True), (1, 8, 1, 1, 4096, 32, False)]


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D,causal", DEC_STRIDED)
def test_fp8_decode_sequence_major_cache_and_narrow_heads(B, Hq, Hkv, Sq, Sk, D, causal):
    """The FP8 cache stored [B][Sk][Hkv][D] (how serving engines keep it), q and o [B][Sq][Hq][D], passed as
    transposed views through the strided entry point; head dimensions between the compiled ones included."""
    seed = 12000 + Sk + D
    q = synth.fill_e4m3(B, Hq, Sq, D, seed, synth.TAG_Q, DQ)
    k = synth.fill_e4m3(B, Hkv, Sk, D, seed, synth.TAG_K, DK, Sk // 50, 8.0)
    v = synth.fill_e4m3(B, Hkv, Sk, D, seed, synth.TAG_V, DV)
    scale = 1.0 / math.sqrt(D)
    bshd = lambda a: torch.from_numpy(np.ascontiguousarray(a.transpose(0, 2, 1, 3))).cuda().transpose(1, 2)
    qd, kd, vd = bshd(q), bshd(k), bshd(v)
    o_mem = torch.full((B, Sq, Hq, D + 8), 7.0, dtype=torch.bfloat16, device="cuda")
    od = o_mem[..., :D].transpose(1, 2)
    lse = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(nb.decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    print("fp8 decode strided", B, Hq, Hkv, Sq, Sk, D, causal, flush=True)
    nb.naut_attn_decode_fp8_strided(qd, kd, vd, od, lse, causal, scale, DQ, DK, DV, ws)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attn_cross_e4m3(q, k, v, DQ, DK, DV, causal, scale)
    check(od.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, v, "fp8 decode strided",
          error_sigma(q, k, v, o_ref, lse_ref, causal, scale))
    assert torch.all(o_mem[..., D:] == 7.0).item(), "columns behind D were written"
    if D in (64, 128):  # the contiguous entry point must give the same bits
        dev = lambda a: torch.from_numpy(a).cuda()
        o2 = torch.empty((B, Hq, Sq, D), dtype=torch.bfloat16, device="cuda")
        nb.naut_attn_decode_fp8(dev(q), dev(k), dev(v), o2, None, causal, scale, DQ, DK, DV, ws)
        torch.cuda.synchronize()
        assert torch.equal(o2, od.contiguous())


@pytest.mark.parametrize("D", [64, 128])
def test_fp8_rows_8_mib_apart(D):
    """FP8 K and V rows at the largest row stride the entry points admit (2^23 bytes), prefill and decode: S times
    the stride passes 2^32, so tile addresses must be formed in 64 bits, and 63 rows of it must fit 32-bit offsets."""
    B, Hq, Hkv, S = 1, 2, 1, 600
    stride = 1 << 23
    q, k, v = make(B, Hq, Hkv, S, D, 12100 + D, S // 50)
    scale = 1.0 / math.sqrt(D)

    def spread(a):
        buf = torch.empty(S * stride, dtype=torch.uint8, device="cuda")  # 4.7 GiB, rows at the start of each pitch
        rows = buf.view(S, stride)[:, :D]
        rows.copy_(torch.from_numpy(a).cuda()[0, 0])
        return rows.unsqueeze(0).unsqueeze(0)  # logical [1,1,S,D]
    kd, vd = spread(k), spread(v)
    assert kd.stride(2) * S > 1 << 32
    qd = torch.from_numpy(q).cuda()
    o = torch.full((B, Hq, S, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((B, Hq, S), float("nan"), dtype=torch.float32, device="cuda")
    print("fp8, 8 MiB row stride", D, flush=True)
    nb.naut_attn_fwd_fp8_strided(qd, kd, vd, o, lse, True, scale, DQ, DK, DV)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attn_rows_e4m3(q, k, v, DQ, DK, DV, True, scale)
    check(o.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, v, "fp8 row stride 2^23",
          error_sigma(q, k, v, o_ref, lse_ref, True, scale))
    # the last two positions as a decode call on the same cache
    Sq = 2
    qs = np.ascontiguousarray(q[:, :, S - Sq:])
    od = torch.full((B, Hq, Sq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lsed = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(nb.decode_workspace_bytes(B, Hq, Hkv, Sq, S, D), dtype=torch.uint8, device="cuda")
    nb.naut_attn_decode_fp8_strided(torch.from_numpy(qs).cuda(), kd, vd, od, lsed, True, scale, DQ, DK, DV, ws)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attn_cross_e4m3(qs, k, v, DQ, DK, DV, True, scale)
    check(od.double().cpu().numpy(), lsed.double().cpu().numpy(), o_ref, lse_ref, v, "fp8 decode row stride 2^23",
          error_sigma(qs, k, v, o_ref, lse_ref, True, scale))
