"""Seeded input generator: determinism, rounding, distribution, outlier rows."""
import numpy as np
import torch

from paper_2604_14825_amd import synth


def test_deterministic_and_order_independent():
    a = synth.fill(2, 3, 64, 16, 123, synth.TAG_K, synth.BF16)
    b = synth.fill(2, 3, 64, 16, 123, synth.TAG_K, synth.BF16)
    np.testing.assert_array_equal(a, b)
    # element value depends on (seed, tag, linear index) only: a [1,6,..] fill is the same stream
    c = synth.fill(1, 6, 64, 16, 123, synth.TAG_K, synth.BF16)
    np.testing.assert_array_equal(a.reshape(-1), c.reshape(-1))
    assert (synth.fill(2, 3, 64, 16, 124, synth.TAG_K, synth.BF16) != a).mean() > 0.9
    assert (synth.fill(2, 3, 64, 16, 123, synth.TAG_V, synth.BF16) != a).mean() > 0.9


def test_bf16_rounding_matches_torch_rne():
    g = np.random.default_rng(0)
    x = np.concatenate([g.standard_normal(200000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40], dtype=np.float32)])
    got = synth.round16(x, synth.BF16)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(got, want)


def test_f16_rounding_matches_numpy_rne():
    g = np.random.default_rng(1)
    x = np.concatenate([g.standard_normal(200000).astype(np.float32) * 3,
                        (g.standard_normal(50000) * 1e-6).astype(np.float32),
                        (g.standard_normal(50000) * 3e4).astype(np.float32),
                        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e6, 2.0 ** -24, 2.0 ** -25,
                                  1.5 * 2.0 ** -25, 2.0 ** -14, 0.99999 * 2.0 ** -14, 1.0009765625,
                                  1.00048828125, 1.00146484375], dtype=np.float32)])
    got = synth.round16(x, synth.F16)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    np.testing.assert_array_equal(got, want)


def test_distribution_moments():
    a = synth.fill(1, 4, 4096, 64, 7, synth.TAG_Q, synth.BF16)
    x = (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    n = x.size
    assert abs(x.mean()) < 5 / np.sqrt(n)
    assert abs(x.var() - 1.0) < 0.01
    assert abs((x ** 3).mean()) < 0.02
    assert abs((x ** 4).mean() - 3.0) < 0.05
    assert np.abs(x).max() < 7.0
    # no visible correlation between neighbours
    assert abs(np.corrcoef(x.reshape(-1)[:-1], x.reshape(-1)[1:])[0, 1]) < 0.005


def test_outlier_rows_exact_count_and_scale():
    w = synth.WORKLOADS["long"]
    assert w.n_outlier == 163
    S, D = 2048, 32
    n_out = 20
    base = synth.fill(1, 2, S, D, 99, synth.TAG_K, synth.BF16)
    out = synth.fill(1, 2, S, D, 99, synth.TAG_K, synth.BF16, n_out, 8.0)
    fb = (base.astype(np.uint32) << 16).view(np.float32)
    fo = (out.astype(np.uint32) << 16).view(np.float32)
    for bh in range(2):
        rows = synth.outlier_rows(bh, S, 99, synth.TAG_K, n_out)
        assert len(set(rows.tolist())) == n_out and rows.min() >= 0 and rows.max() < S
        changed = np.where((fo[0, bh] != fb[0, bh]).any(axis=1))[0]
        assert sorted(changed.tolist()) == sorted(rows.tolist())
        # x8 is a power of two: scaling before rounding == scaling the rounded value
        np.testing.assert_array_equal(fo[0, bh, rows], 8.0 * fb[0, bh, rows])
    assert sorted(synth.outlier_rows(0, S, 99, synth.TAG_K, n_out).tolist()) != \
        sorted(synth.outlier_rows(1, S, 99, synth.TAG_K, n_out).tolist())


def test_workload_table_matches_declared_shapes():
    w = synth.WORKLOADS
    assert (w["tiny"].B, w["tiny"].Hq, w["tiny"].S, w["tiny"].D, w["tiny"].causal) == (1, 2, 256, 64, False)
    assert w["tiny"].in_dtype == synth.F16 and w["tiny"].out_dtype == synth.F32
    assert (w["encoder"].B, w["encoder"].Hq, w["encoder"].S, w["encoder"].D) == (8, 16, 1024, 64)
    assert (w["prefill"].B, w["prefill"].Hq, w["prefill"].S, w["prefill"].causal) == (4, 32, 4096, True)
    assert (w["gqa"].Hq, w["gqa"].Hkv, w["gqa"].S) == (64, 8, 8192)
    assert (w["long"].B, w["long"].Hq, w["long"].S, w["long"].D, w["long"].causal) == (1, 32, 16384, 128, True)
    assert abs(w["long"].flops - 2.199e12) / 2.199e12 < 1e-3
    assert abs(w["long"].io_bytes - 539e6) / 539e6 < 5e-3
    q, k, v = synth.make_inputs(w["tiny"])
    assert q.shape == (1, 2, 256, 64) and k.shape == q.shape and q.dtype == np.uint16


def test_round_e4m3_matches_library_rounding():
    """Nearest-even rounding to FP8 E4M3 against PyTorch's CPU conversion on every in-range float16 value
    (all exactly representable in float32) and on random float32 values; saturation beyond 448."""
    import torch
    vals = np.arange(0, 1 << 16, dtype=np.uint16).view(np.float16).astype(np.float32)
    vals = vals[np.isfinite(vals) & (np.abs(vals) <= 448.0)]
    g = np.random.default_rng(3)
    vals = np.concatenate([vals, (g.standard_normal(20000) * 40).astype(np.float32),
                           (g.standard_normal(20000) * 0.01).astype(np.float32)])
    vals = vals[np.abs(vals) <= 448.0]
    got = synth.round_e4m3(vals)
    want = torch.from_numpy(vals.copy()).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    np.testing.assert_array_equal(got, want)
    big = np.array([449.0, 464.0, 465.0, 1e4, -1e30], dtype=np.float32)
    np.testing.assert_array_equal(synth.round_e4m3(big), np.array([0x7E, 0x7E, 0x7E, 0x7E, 0xFE], dtype=np.uint8))


def test_fill_e4m3_is_the_scaled_rounded_fill():
    a = synth.fill_e4m3(1, 2, 50, 16, 11, synth.TAG_K, 0.125, 2, 8.0)
    b16 = synth.fill(1, 2, 50, 16, 11, synth.TAG_K, synth.BF16, 2, 8.0)
    x = (b16.astype(np.uint32) << 16).view(np.float32) / np.float32(0.125)
    np.testing.assert_array_equal(a, synth.round_e4m3(x))
    assert a.dtype == np.uint8 and a.shape == (1, 2, 50, 16)
