"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle on identical seeded inputs."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2604_14825_amd import binding as nb
from paper_2604_14825_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu

SMALL = [
    # B, Hq, Hkv, S, D, causal, in, out      (several tiles, ragged tails, degenerate sizes)
    (1, 1, 1, 1, 64, False, synth.BF16, synth.BF16),
    (1, 1, 1, 1, 128, True, synth.BF16, synth.BF16),
    (1, 2, 1, 7, 64, True, synth.F16, synth.F32),
    (2, 2, 2, 63, 128, True, synth.BF16, synth.BF16),
    (1, 2, 2, 64, 128, False, synth.BF16, synth.BF16),
    (1, 2, 2, 65, 64, False, synth.BF16, synth.F32),
    (2, 4, 2, 129, 128, True, synth.BF16, synth.BF16),
    (1, 3, 1, 200, 64, True, synth.BF16, synth.BF16),
    (1, 2, 2, 257, 128, False, synth.F16, synth.F16),
    (2, 4, 2, 333, 64, True, synth.F16, synth.F16),
    (1, 8, 2, 400, 128, True, synth.BF16, synth.F32),
    (1, 2, 2, 512, 128, True, synth.BF16, synth.BF16),
    (1, 2, 1, 777, 128, False, synth.BF16, synth.BF16),
    (1, 4, 2, 300, 256, True, synth.BF16, synth.BF16),    # the widest head dimension through the dense entry point
    (2, 2, 2, 33, 256, False, synth.F16, synth.F32),
]


@pytest.mark.parametrize("B,Hq,Hkv,S,D,causal,idt,odt", SMALL)
def test_small_shapes_elementwise(B, Hq, Hkv, S, D, causal, idt, odt):
    seed = 1000 + S * 7 + D
    q = synth.fill(B, Hq, S, D, seed, synth.TAG_Q, idt)
    k = synth.fill(B, Hkv, S, D, seed, synth.TAG_K, idt, S // 50, 8.0)
    v = synth.fill(B, Hkv, S, D, seed, synth.TAG_V, idt)
    scale = 1.0 / math.sqrt(D)
    print("case", B, Hq, Hkv, S, D, causal, idt, odt, flush=True)
    o, lse = gu.run_hip(q, k, v, idt, odt, causal, scale)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, causal, scale)
    gu.check(o, lse, o_ref, lse_ref, "small")


def _bits_to_f32(bits, dtype):
    if dtype == synth.F16:
        return bits.view(np.float16).astype(np.float32)
    return (bits.astype(np.uint32) << 16).view(np.float32)


def _key_profile(kind, S):
    """Per-key multipliers that drive the running maximum the hard way."""
    j = np.arange(S, dtype=np.float32)
    if kind == "ascending":      # later keys ever larger: the reference maximum moves again and again
        return 0.25 + 12.0 * j / max(S - 1, 1)
    if kind == "descending":     # the first block holds the maximum: the reference never moves after it
        return 12.25 - 12.0 * j / max(S - 1, 1)
    if kind == "late_spike":     # one key, late in the sequence, dwarfs everything before it
        f = np.ones(S, dtype=np.float32)
        f[(3 * S) // 4] = 60.0
        return f
    raise ValueError(kind)


@pytest.mark.parametrize("variant", ["w8q32", "w4q64", "bm128"])
@pytest.mark.parametrize("kind", ["ascending", "descending", "late_spike"])
def test_moving_reference_maximum(kind, variant, monkeypatch):
    """Score profiles that exercise the repair path of the online softmax: a maximum that keeps growing,
    one that is met in the first block, and a single late key far above the rest (near one-hot rows)."""
    monkeypatch.setenv("NAUT_ATTN_VARIANT", variant)
    B, Hq, Hkv, S, D, causal, idt, odt = 1, 4, 2, 700, 128, True, synth.BF16, synth.F32
    seed = 4242
    q = synth.fill(B, Hq, S, D, seed, synth.TAG_Q, idt)
    k = synth.fill(B, Hkv, S, D, seed, synth.TAG_K, idt)
    v = synth.fill(B, Hkv, S, D, seed, synth.TAG_V, idt)
    kf = _bits_to_f32(k, idt) * _key_profile(kind, S)[None, None, :, None]
    k = synth.round16(kf, idt)
    scale = 1.0 / math.sqrt(D)
    print("case", kind, variant, flush=True)
    o, lse = gu.run_hip(q, k, v, idt, odt, causal, scale)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, causal, scale)
    gu.check(o, lse, o_ref, lse_ref, kind + "/" + variant)
    for causal2 in (False,):
        o, lse = gu.run_hip(q, k, v, idt, odt, causal2, 4.0 * scale)  # hotter softmax: scores in the hundreds
        o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, causal2, 4.0 * scale)
        gu.check(o, lse, o_ref, lse_ref, kind + "/" + variant + "/hot")


@pytest.mark.parametrize("variant,D", [("w8q32", 128), ("w4q64", 128), ("bm128", 128), ("bm128", 64), ("bm128", 256)])
def test_dominant_key_behind_a_lagging_reference(variant, D, monkeypatch):
    """The last key of every fourth row (its diagonal, under the causal mask) dominates the row by a few binades --
    too few to make a kernel move its reference maximum -- and carries values of magnitude 4 to 5.5, where one
    bf16 step of O is 3e-2.  The largest P of such a row is an arbitrary number, not 1; unless O is divided by the sum of the
    P that went into it, the rounding of that P (up to 2^-8) is an error of 2^-8 |v| on top of the rounding of O, and
    the 2e-2 bar is missed."""
    if D <= 128:
        monkeypatch.setenv("NAUT_ATTN_VARIANT", variant)
    B, H, S, idt, odt = 1, 4, 1500, synth.BF16, synth.BF16
    seed = 4545 + D
    q = synth.fill(B, H, S, D, seed, synth.TAG_Q, idt)
    k = synth.fill(B, H, S, D, seed, synth.TAG_K, idt)
    v = synth.fill(B, H, S, D, seed, synth.TAG_V, idt)
    scale = 1.0 / math.sqrt(D)
    qf, vf = _bits_to_f32(q, idt), _bits_to_f32(v, idt)
    g = np.random.default_rng(seed)
    # Every fourth row gets a last key of its own: key i = q_i * t_i scores `target` with row i and about
    # target / sqrt(D) with any other row; target lies 1 to 4.5 (0.3 to 6.8 binades) above the usual maximum of
    # a row's other scores, and that key's values have magnitude 4 to 5.5.  Everything else stays N(0,1).
    kf = _bits_to_f32(k, idt)
    dom = np.arange(S) % 4 == 3
    target = (3.6 + g.uniform(1.0, 4.5, size=(B, H, S))).astype(np.float32)
    t = target / (scale * (qf * qf).sum(-1))
    kf[:, :, dom] = (qf * t[..., None])[:, :, dom]
    k = synth.round16(kf, idt)
    sign = np.where(g.random((B, H, S, D)) < 0.5, -1.0, 1.0).astype(np.float32)
    vf[:, :, dom] = (sign * g.uniform(4.0, 5.5, size=(B, H, S, D)).astype(np.float32))[:, :, dom]
    v = synth.round16(vf, idt)
    print("case dominant key", variant, D, flush=True)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, True, scale)
    assert np.abs(o_ref).max() > 4.0, "the case must reach the range where one bf16 step of O exceeds the bar"
    # fp32 output: the kernel's own error, against the whole bar
    o, lse = gu.run_hip(q, k, v, idt, synth.F32, True, scale)
    gu.check(o, lse, o_ref, lse_ref, "dominant key/%s/D%d/f32 out" % (variant, D))
    # bf16 output: the maximum only (values of magnitude 4 to 8 round to bf16 with a mean error of 8e-3 by themselves)
    o, lse = gu.run_hip(q, k, v, idt, odt, True, scale)
    d = np.abs(o - o_ref)
    print("bf16 out: max|dO| %.3e mean %.3e" % (d.max(), d.mean()), flush=True)
    assert np.isfinite(o).all() and d.max() <= gu.TOL_MAX, "dominant key/%s/D%d: max|dO| = %.3e" % (variant, D, d.max())


@pytest.mark.parametrize("kind", ["ascending", "descending", "late_spike"])
def test_moving_reference_maximum_wide(kind):
    """The same score profiles on the D = 256 kernel, whose rescale block moves O between register files."""
    B, Hq, Hkv, S, D, idt, odt = 1, 4, 2, 500, 256, synth.BF16, synth.F32
    seed = 4343
    q = synth.fill(B, Hq, S, D, seed, synth.TAG_Q, idt)
    k = synth.fill(B, Hkv, S, D, seed, synth.TAG_K, idt)
    v = synth.fill(B, Hkv, S, D, seed, synth.TAG_V, idt)
    k = synth.round16(_bits_to_f32(k, idt) * _key_profile(kind, S)[None, None, :, None], idt)
    scale = 1.0 / math.sqrt(D)
    print("case wide", kind, flush=True)
    for causal, sc in ((True, scale), (False, 4.0 * scale)):
        o, lse = gu.run_hip(q, k, v, idt, odt, causal, sc)
        o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, causal, sc)
        gu.check(o, lse, o_ref, lse_ref, "wide/" + kind)


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("variant", ["w8q32", "bm128"])
def test_every_tile_count(variant, causal, monkeypatch):
    """Sequence lengths just below, at and just above every multiple of 64 up to 704: every residue of the key-tile
    count modulo the unrolled loops' period (4 LDS buffers in the 256-query kernel, 2 in the 128-query one), with
    and without a ragged last tile, and every position of the causal diagonal inside a 256-query work-group."""
    monkeypatch.setenv("NAUT_ATTN_VARIANT", variant)
    B, Hq, Hkv, D, idt, odt = 1, 2, 1, 128, synth.BF16, synth.F32
    scale = 1.0 / math.sqrt(D)
    for t in range(1, 12):
        for S in (64 * t - 1, 64 * t, 64 * t + 1):
            q = synth.fill(B, Hq, S, D, 6000 + S, synth.TAG_Q, idt)
            k = synth.fill(B, Hkv, S, D, 6000 + S, synth.TAG_K, idt, S // 50, 8.0)
            v = synth.fill(B, Hkv, S, D, 6000 + S, synth.TAG_V, idt)
            o, lse = gu.run_hip(q, k, v, idt, odt, causal, scale)
            o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, causal, scale)
            gu.check(o, lse, o_ref, lse_ref, "S=%d %s causal=%d" % (S, variant, causal))


VARIANT_SHAPES = [
    (1, 2, 1, 1, 64, True, synth.BF16, synth.BF16),
    (2, 4, 2, 129, 128, True, synth.BF16, synth.BF16),
    (1, 2, 2, 257, 128, False, synth.F16, synth.F16),
    (1, 3, 1, 333, 64, True, synth.F16, synth.F32),
    (1, 4, 2, 600, 128, True, synth.BF16, synth.BF16),
    (1, 2, 2, 1024, 64, False, synth.BF16, synth.BF16),
]


@pytest.mark.parametrize("variant", ["w8q32", "w4q64", "bm128"])
def test_every_kernel_variant(variant, monkeypatch):
    """Each tile shape / wavefront layout the library can choose gives the same attention."""
    monkeypatch.setenv("NAUT_ATTN_VARIANT", variant)
    for B, Hq, Hkv, S, D, causal, idt, odt in VARIANT_SHAPES:
        seed = 2000 + S + D
        q = synth.fill(B, Hq, S, D, seed, synth.TAG_Q, idt)
        k = synth.fill(B, Hkv, S, D, seed, synth.TAG_K, idt, S // 40, 8.0)
        v = synth.fill(B, Hkv, S, D, seed, synth.TAG_V, idt)
        scale = 1.0 / math.sqrt(D)
        print("variant", variant, "case", B, Hq, Hkv, S, D, causal, idt, odt, flush=True)
        o, lse = gu.run_hip(q, k, v, idt, odt, causal, scale)
        o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, causal, scale)
        gu.check(o, lse, o_ref, lse_ref, variant)


@pytest.mark.parametrize("variant", ["w4q64", "bm128"])
def test_variants_on_prefill_sampled_rows(variant, monkeypatch):
    monkeypatch.setenv("NAUT_ATTN_VARIANT", variant)
    w = synth.WORKLOADS["prefill"]
    q, k, v = synth.make_inputs(w)
    o, lse = gu.run_hip(q, k, v, w.in_dtype, w.out_dtype, w.causal, w.scale)
    rows = gu.sample_rows(w, 1024, seed=23, bm=256)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, w.in_dtype, w.causal, w.scale, rows=rows)
    gu.check(o.reshape(-1, w.D)[rows], lse.reshape(-1)[rows], o_ref, lse_ref, variant)


def test_tiny_workload_full():
    w = synth.WORKLOADS["tiny"]
    q, k, v = synth.make_inputs(w)
    o, lse = gu.run_hip(q, k, v, w.in_dtype, w.out_dtype, w.causal, w.scale)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, w.in_dtype, w.causal, w.scale)
    mx, mean = gu.check(o, lse, o_ref, lse_ref, "tiny")
    # fp16 inputs, fp32 output: only P's rounding to fp16 and fp32 accumulation remain
    assert mx < 5e-3


def test_encoder_workload_full():
    w = synth.WORKLOADS["encoder"]
    q, k, v = synth.make_inputs(w)
    o, lse = gu.run_hip(q, k, v, w.in_dtype, w.out_dtype, w.causal, w.scale)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, w.in_dtype, w.causal, w.scale)
    gu.check(o, lse, o_ref, lse_ref, "encoder")


@pytest.mark.parametrize("name,nrand", [("prefill", 4096), ("gqa", 3072), ("long", 3072)])
def test_large_workloads_sampled_rows(name, nrand):
    """Full-size launch (the configuration bench.py times); the oracle computes a declared row subset
    (every output row depends only on its own query row, so a subset is exact)."""
    w = synth.WORKLOADS[name]
    print("workload", name, flush=True)
    q, k, v = synth.make_inputs(w)
    o, lse = gu.run_hip(q, k, v, w.in_dtype, w.out_dtype, w.causal, w.scale)
    assert np.isfinite(o).all() and np.isfinite(lse).all()
    rows = gu.sample_rows(w, nrand, seed=17)
    if w.n_outlier:
        # rows whose diagonal tile holds an outlier key, and the outlier rows themselves
        out = synth.outlier_rows(0, w.S, synth.workload_seed(w), synth.TAG_K, w.n_outlier)
        rows = np.unique(np.concatenate([rows, out[:64].astype(np.int64), np.minimum(out[:64].astype(np.int64) + 1, w.S - 1)]))
    o_ref, lse_ref = oracle.attn_rows(q, k, v, w.in_dtype, w.causal, w.scale, rows=rows)
    gu.check(o.reshape(-1, w.D)[rows], lse.reshape(-1)[rows], o_ref, lse_ref, name)


@pytest.mark.parametrize("S,causal", [(32768, True), (65573, True), (40000, False)])
def test_longest_sequences_sampled_rows(S, causal):
    """The paper's longest sequence (2^15, Section 6) and beyond it, with a ragged tail: grouped-query heads,
    outlier keys, the first and last tiles and random rows against the oracle."""
    B, Hq, Hkv, D, idt = 1, 8, 2, 128, synth.BF16
    q = synth.fill(B, Hq, S, D, 31000 + S, synth.TAG_Q, idt)
    k = synth.fill(B, Hkv, S, D, 31000 + S, synth.TAG_K, idt, S // 100, 8.0)
    v = synth.fill(B, Hkv, S, D, 31000 + S, synth.TAG_V, idt)
    scale = 1.0 / math.sqrt(D)
    print("long sequence", S, causal, flush=True)
    o, lse = gu.run_hip(q, k, v, idt, idt, causal, scale)
    assert np.isfinite(o).all() and np.isfinite(lse).all()
    g = np.random.default_rng(S)
    rows = np.unique(np.concatenate([np.arange(0, 260), np.arange(B * Hq * S - 260, B * Hq * S),
                                     g.integers(0, B * Hq * S, 400)])).astype(np.int64)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, causal, scale, rows=rows)
    gu.check(o.reshape(-1, D)[rows], lse.reshape(-1)[rows], o_ref, lse_ref, "S=%d" % S)


def test_run_to_run_bit_identical():
    w = synth.WORKLOADS["encoder"]
    q, k, v = synth.make_inputs(w)
    o1, l1 = gu.run_hip(q, k, v, w.in_dtype, w.out_dtype, w.causal, w.scale)
    o2, l2 = gu.run_hip(q, k, v, w.in_dtype, w.out_dtype, w.causal, w.scale)
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(l1, l2)


def test_lse_null_and_side_stream():
    w = synth.WORKLOADS["tiny"]
    q, k, v = synth.make_inputs(w)
    o_ref, _ = gu.run_hip(q, k, v, w.in_dtype, w.out_dtype, w.causal, w.scale)
    qd, kd, vd = (gu.to_device(a, w.in_dtype) for a in (q, k, v))
    o = torch.zeros((w.B, w.Hq, w.S, w.D), dtype=torch.float32, device="cuda")
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    nb.naut_attn_fwd(qd, kd, vd, o, None, w.causal, w.scale, stream=st)
    st.synchronize()
    np.testing.assert_array_equal(o.double().cpu().numpy(), o_ref)


def test_zero_scale_and_property_checks():
    # scale = 0: uniform attention -> prefix means of V, lse = ln(i+1)
    B, H, S, D = 1, 2, 300, 64
    q = synth.fill(B, H, S, D, 5, synth.TAG_Q, synth.BF16)
    k = synth.fill(B, H, S, D, 5, synth.TAG_K, synth.BF16)
    v = synth.fill(B, H, S, D, 5, synth.TAG_V, synth.BF16)
    o, lse = gu.run_hip(q, k, v, synth.BF16, synth.F32, True, 0.0)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, synth.BF16, True, 0.0)
    gu.check(o, lse, o_ref, lse_ref, "scale0")
    np.testing.assert_allclose(lse[0, 0], np.log(np.arange(1, S + 1)), atol=1e-4)
