"""Pins for the fp64 oracle: closed forms, invariants, brute force, library second opinion.

None of these re-types the oracle's loops: each checks it against something the
mathematics of softmax attention fixes independently (Section 1 of the paper
names the operator; the operator table of Section 6 its Global / Causal / GQA
variants; Appendix B uses the same FP64 unfused computation as ground truth).
"""
import math

import numpy as np
import pytest
import scipy.special

import oracle


def rng(seed):
    return np.random.default_rng(seed)


def rand_qkv(seed, B, Hq, Hkv, S, D, scale_q=1.0):
    g = rng(seed)
    q = g.standard_normal((B, Hq, S, D)) * scale_q
    k = g.standard_normal((B, Hkv, S, D))
    v = g.standard_normal((B, Hkv, S, D))
    return q, k, v


# ---------------------------------------------------------------------------
# brute force, hand-expanded (no loops shared with the oracle)
# ---------------------------------------------------------------------------

def test_hand_expanded_S2_D2_noncausal():
    q = np.array([[[[1.0, 2.0], [-0.5, 0.25]]]])
    k = np.array([[[[0.5, -1.0], [1.5, 0.75]]]])
    v = np.array([[[[2.0, -3.0], [0.5, 4.0]]]])
    scale = 0.7
    s00 = scale * (1.0 * 0.5 + 2.0 * -1.0)
    s01 = scale * (1.0 * 1.5 + 2.0 * 0.75)
    s10 = scale * (-0.5 * 0.5 + 0.25 * -1.0)
    s11 = scale * (-0.5 * 1.5 + 0.25 * 0.75)
    z0 = math.exp(s00) + math.exp(s01)
    z1 = math.exp(s10) + math.exp(s11)
    want_o = np.array([
        [(math.exp(s00) * 2.0 + math.exp(s01) * 0.5) / z0, (math.exp(s00) * -3.0 + math.exp(s01) * 4.0) / z0],
        [(math.exp(s10) * 2.0 + math.exp(s11) * 0.5) / z1, (math.exp(s10) * -3.0 + math.exp(s11) * 4.0) / z1],
    ])
    want_lse = np.array([math.log(z0), math.log(z1)])
    o, lse = oracle.attn_f64(q, k, v, False, scale)
    np.testing.assert_allclose(o[0, 0], want_o, rtol=0, atol=1e-14)
    np.testing.assert_allclose(lse[0, 0], want_lse, rtol=0, atol=1e-14)


def test_hand_expanded_S3_D1_causal():
    # D = 1 so every score is one product; causal: row i sees keys 0..i.
    q = np.array([0.3, -1.2, 2.0]).reshape(1, 1, 3, 1)
    k = np.array([1.1, 0.4, -0.9]).reshape(1, 1, 3, 1)
    v = np.array([5.0, -2.0, 7.0]).reshape(1, 1, 3, 1)
    sc = 1.3
    e = math.exp
    o0 = 5.0
    l0 = sc * 0.3 * 1.1
    a, b = e(sc * -1.2 * 1.1), e(sc * -1.2 * 0.4)
    o1 = (a * 5.0 + b * -2.0) / (a + b)
    l1 = math.log(a + b)
    c, d, f = e(sc * 2.0 * 1.1), e(sc * 2.0 * 0.4), e(sc * 2.0 * -0.9)
    o2 = (c * 5.0 + d * -2.0 + f * 7.0) / (c + d + f)
    l2 = math.log(c + d + f)
    o, lse = oracle.attn_f64(q, k, v, True, sc)
    np.testing.assert_allclose(o.ravel(), [o0, o1, o2], rtol=0, atol=1e-14)
    np.testing.assert_allclose(lse.ravel(), [l0, l1, l2], rtol=0, atol=1e-14)


def test_hand_expanded_gqa_S2_causal():
    # Hq = 4, Hkv = 2, D = 1: heads 0,1 read kv head 0; heads 2,3 read kv head 1.
    q = np.array([[1.0, 2.0], [0.5, -1.0], [-2.0, 0.25], [3.0, 1.5]]).reshape(1, 4, 2, 1)
    k = np.array([[0.2, -0.7], [1.4, 0.6]]).reshape(1, 2, 2, 1)
    v = np.array([[10.0, 20.0], [-1.0, 3.0]]).reshape(1, 2, 2, 1)
    sc = 0.9
    e = math.exp
    o, lse = oracle.attn_f64(q, k, v, True, sc)
    # row 0 of every head sees only key 0 of its kv head
    np.testing.assert_allclose(o[0, :, 0, 0], [10.0, 10.0, -1.0, -1.0], rtol=0, atol=1e-14)
    np.testing.assert_allclose(lse[0, :, 0], [sc * 1.0 * 0.2, sc * 0.5 * 0.2, sc * -2.0 * 1.4, sc * 3.0 * 1.4],
                               rtol=0, atol=1e-14)
    # row 1: two keys
    w = []
    z = []
    for qv, (k0, k1), (v0, v1) in [(2.0, (0.2, -0.7), (10.0, 20.0)), (-1.0, (0.2, -0.7), (10.0, 20.0)),
                                   (0.25, (1.4, 0.6), (-1.0, 3.0)), (1.5, (1.4, 0.6), (-1.0, 3.0))]:
        a, b = e(sc * qv * k0), e(sc * qv * k1)
        w.append((a * v0 + b * v1) / (a + b))
        z.append(math.log(a + b))
    np.testing.assert_allclose(o[0, :, 1, 0], w, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse[0, :, 1], z, rtol=0, atol=1e-13)


def test_hand_expanded_S4_D2_noncausal_row():
    # One row of a 4-key problem with the operands' roles made asymmetric
    # (a transposed q/k or k/v would change the answer).
    q = np.array([[0.5, -1.5]]).reshape(1, 1, 1, 2).repeat(4, axis=2).copy()
    q[0, 0, 1] = [2.0, 0.1]
    q[0, 0, 2] = [-0.3, 0.9]
    q[0, 0, 3] = [1.0, 1.0]
    k = np.array([[1.0, 0.0], [0.0, 1.0], [2.0, -1.0], [-0.5, 0.5]]).reshape(1, 1, 4, 2)
    v = np.array([[1.0, 10.0], [2.0, 20.0], [3.0, 30.0], [4.0, 40.0]]).reshape(1, 1, 4, 2)
    sc = 0.5
    # row 1: q = (2.0, 0.1)
    s = [sc * (2.0 * 1.0 + 0.1 * 0.0), sc * (2.0 * 0.0 + 0.1 * 1.0), sc * (2.0 * 2.0 + 0.1 * -1.0),
         sc * (2.0 * -0.5 + 0.1 * 0.5)]
    ex = [math.exp(x) for x in s]
    z = ex[0] + ex[1] + ex[2] + ex[3]
    want0 = (ex[0] * 1.0 + ex[1] * 2.0 + ex[2] * 3.0 + ex[3] * 4.0) / z
    want1 = (ex[0] * 10.0 + ex[1] * 20.0 + ex[2] * 30.0 + ex[3] * 40.0) / z
    o, lse = oracle.attn_f64(q, k, v, False, sc)
    np.testing.assert_allclose(o[0, 0, 1], [want0, want1], rtol=0, atol=1e-13)
    assert abs(lse[0, 0, 1] - math.log(z)) < 1e-14


# ---------------------------------------------------------------------------
# invariants and closed forms
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("causal", [False, True])
def test_probs_row_stochastic_and_masked(causal):
    q, k, v = rand_qkv(1, 2, 4, 2, 37, 16)
    o, lse, p = oracle.attn_f64(q, k, v, causal, 0.25, want_probs=True)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=0, atol=1e-14)
    assert (p >= 0).all()
    if causal:
        iu = np.triu_indices(37, k=1)
        assert (p[..., iu[0], iu[1]] == 0).all()
        # the diagonal is allowed
        assert (p[..., np.arange(37), np.arange(37)] > 0).all()
    # O is P @ V with the grouped head map
    vrep = np.repeat(v, 2, axis=1)
    np.testing.assert_allclose(o, np.einsum("bhij,bhjd->bhid", p, vrep), rtol=0, atol=1e-13)


@pytest.mark.parametrize("causal", [False, True])
def test_all_ones_V_gives_ones(causal):
    q, k, _ = rand_qkv(2, 1, 3, 3, 50, 8)
    v = np.ones((1, 3, 50, 8))
    o, _ = oracle.attn_f64(q, k, v, causal, 0.35)
    np.testing.assert_allclose(o, 1.0, rtol=0, atol=1e-14)


def test_zero_Q_gives_column_mean_and_log_count():
    _, k, v = rand_qkv(3, 2, 2, 2, 33, 8)
    q = np.zeros((2, 2, 33, 8))
    o, lse = oracle.attn_f64(q, k, v, False, 0.5)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(axis=2, keepdims=True), o.shape), rtol=0, atol=1e-14)
    np.testing.assert_allclose(lse, math.log(33), rtol=0, atol=1e-14)
    # causal: prefix means and ln(i+1)
    o, lse = oracle.attn_f64(q, k, v, True, 0.5)
    prefix = np.cumsum(v, axis=2) / np.arange(1, 34).reshape(1, 1, 33, 1)
    np.testing.assert_allclose(o, prefix, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, np.broadcast_to(np.log(np.arange(1, 34)), lse.shape), rtol=0, atol=1e-14)


def test_key_permutation_invariance_noncausal():
    q, k, v = rand_qkv(4, 1, 2, 2, 41, 8)
    perm = rng(40).permutation(41)
    o1, l1 = oracle.attn_f64(q, k, v, False, 0.3)
    o2, l2 = oracle.attn_f64(q, k[:, :, perm], v[:, :, perm], False, 0.3)
    np.testing.assert_allclose(o1, o2, rtol=0, atol=1e-13)
    np.testing.assert_allclose(l1, l2, rtol=0, atol=1e-13)


def test_causal_row0_is_V0():
    q, k, v = rand_qkv(5, 2, 2, 1, 9, 4)
    o, lse = oracle.attn_f64(q, k, v, True, 0.6)
    np.testing.assert_array_equal(o[:, :, 0], np.repeat(v[:, :, 0], 2, axis=1))
    s00 = 0.6 * np.einsum("bhd,bhd->bh", q[:, :, 0], np.repeat(k[:, :, 0], 2, axis=1))
    np.testing.assert_allclose(lse[:, :, 0], s00, rtol=0, atol=1e-14)


def test_causal_prefix_property():
    # causal row i == global attention of q_i over the first i+1 keys
    q, k, v = rand_qkv(6, 1, 2, 2, 19, 8)
    oc, lc = oracle.attn_f64(q, k, v, True, 0.4)
    for i in (0, 1, 7, 18):
        og, lg = oracle.attn_f64(q[:, :, : i + 1], k[:, :, : i + 1], v[:, :, : i + 1], False, 0.4)
        np.testing.assert_allclose(oc[:, :, i], og[:, :, i], rtol=0, atol=1e-14)
        np.testing.assert_allclose(lc[:, :, i], lg[:, :, i], rtol=0, atol=1e-14)


@pytest.mark.parametrize("causal", [False, True])
def test_gqa_equals_repeated_head_mha(causal):
    q, k, v = rand_qkv(7, 2, 6, 2, 21, 8)
    o1, l1 = oracle.attn_f64(q, k, v, causal, 0.3)
    o2, l2 = oracle.attn_f64(q, np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1), causal, 0.3)
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(l1, l2)
    # and heads that share a kv head but have different q differ
    assert not np.allclose(o1[:, 0], o1[:, 1])


def test_scale_identity_and_key_shift():
    q, k, v = rand_qkv(8, 1, 2, 2, 25, 8)
    o1, l1 = oracle.attn_f64(q, k, v, True, 0.5)
    o2, l2 = oracle.attn_f64(2.0 * q, k, v, True, 0.25)  # exact in binary fp
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(l1, l2)
    # scale matters: halving it alone changes the result
    o3, _ = oracle.attn_f64(q, k, v, True, 0.25)
    assert np.abs(o3 - o1).max() > 1e-3
    # adding c to every key row shifts lse_i by scale * q_i . c and leaves O alone
    c = rng(80).standard_normal(8)
    o4, l4 = oracle.attn_f64(q, k + c, v, True, 0.5)
    np.testing.assert_allclose(o4, o1, rtol=0, atol=1e-12)
    np.testing.assert_allclose(l4 - l1, 0.5 * np.einsum("bhid,d->bhi", q, c), rtol=0, atol=1e-12)


def test_split_merge_identity():
    q, k, v = rand_qkv(9, 1, 2, 2, 40, 8)
    o, lse = oracle.attn_f64(q, k, v, False, 0.45)
    mask = rng(90).random(40) < 0.4
    mask[0], mask[1] = True, False
    A, Bs = np.where(mask)[0], np.where(~mask)[0]
    # attention of all 40 queries over subset A of the keys == global attention with K,V restricted;
    # pad the query count by running every query against the restricted keys one block at a time.
    def over(keys):
        n = len(keys)
        outs, lses = [], []
        for start in range(0, 40, n):
            qq = q[:, :, start:start + n]
            m = qq.shape[2]
            if m < n:
                qq = np.concatenate([qq, np.zeros((1, 2, n - m, 8))], axis=2)
            oo, ll = oracle.attn_f64(qq, k[:, :, keys], v[:, :, keys], False, 0.45)
            outs.append(oo[:, :, :m])
            lses.append(ll[:, :, :m])
        return np.concatenate(outs, axis=2), np.concatenate(lses, axis=2)
    oa, la = over(A)
    ob, lb = over(Bs)
    lm = np.logaddexp(la, lb)
    om = np.exp(la - lm)[..., None] * oa + np.exp(lb - lm)[..., None] * ob
    np.testing.assert_allclose(lm, lse, rtol=0, atol=1e-13)
    np.testing.assert_allclose(om, o, rtol=0, atol=1e-13)


def test_one_hot_limit():
    g = rng(10)
    D, S = 4, 12
    k = g.standard_normal((1, 1, S, D)) * 0.1
    v = g.standard_normal((1, 1, S, D))
    q = g.standard_normal((1, 1, S, D)) * 0.1
    k[0, 0, 5] = [100.0, 0, 0, 0]
    q[0, 0, :, 0] = 1.0
    o, lse = oracle.attn_f64(q, k, v, False, 1.0)
    np.testing.assert_allclose(o[0, 0], np.broadcast_to(v[0, 0, 5], (S, D)), rtol=0, atol=1e-30)
    # big scores must not overflow: lse ~ the dominating score
    np.testing.assert_allclose(lse[0, 0], np.einsum("id,d->i", q[0, 0], k[0, 0, 5]), rtol=0, atol=1e-12)


def test_large_scores_do_not_overflow():
    q, k, v = rand_qkv(11, 1, 1, 1, 16, 8)
    o, lse = oracle.attn_f64(q * 400.0, k, v, False, 1.0)   # scores ~ +-2000, exp() alone would overflow
    assert np.isfinite(o).all() and np.isfinite(lse).all()


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("Hq,Hkv", [(2, 2), (4, 1)])
def test_scipy_second_opinion(causal, Hq, Hkv):
    B, S, D = 2, 96, 16
    q, k, v = rand_qkv(12 + Hq, B, Hq, Hkv, S, D)
    scale = 1.0 / math.sqrt(D)
    o, lse = oracle.attn_f64(q, k, v, causal, scale)
    g = Hq // Hkv
    kk = np.repeat(k, g, axis=1)
    vv = np.repeat(v, g, axis=1)
    s = scale * (q @ np.swapaxes(kk, -1, -2))
    if causal:
        s = np.where(np.tril(np.ones((S, S), dtype=bool)), s, -np.inf)
    want_o = scipy.special.softmax(s, axis=-1) @ vv
    want_lse = scipy.special.logsumexp(s, axis=-1)
    np.testing.assert_allclose(o, want_o, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, want_lse, rtol=0, atol=1e-12)


# ---------------------------------------------------------------------------
# 16-bit entry point: decoders and row selection
# ---------------------------------------------------------------------------

def test_decoders_exact_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    f16 = oracle.decode16(bits, oracle.F16)
    want = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(want)
    assert (np.isnan(f16) == nan).all()
    np.testing.assert_array_equal(f16[~nan], want[~nan])
    bf = oracle.decode16(bits, oracle.BF16)
    want = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    nan = np.isnan(want)
    assert (np.isnan(bf) == nan).all()
    np.testing.assert_array_equal(bf[~nan], want[~nan])


@pytest.mark.parametrize("dtype", [oracle.BF16, oracle.F16])
@pytest.mark.parametrize("causal", [False, True])
def test_rows_entry_matches_f64_entry(dtype, causal):
    g = rng(20)
    B, Hq, Hkv, S, D = 2, 4, 2, 29, 8
    qb = g.integers(0, 65536, (B, Hq, S, D)).astype(np.uint16)
    kb = g.integers(0, 65536, (B, Hkv, S, D)).astype(np.uint16)
    vb = g.integers(0, 65536, (B, Hkv, S, D)).astype(np.uint16)
    # keep magnitudes moderate and finite: clear the top exponent bits
    if dtype == oracle.F16:
        for a in (qb, kb, vb):
            a &= np.uint16(0xBFFF)     # |x| < 2
    else:
        for a in (qb, kb, vb):
            a &= np.uint16(0xBFFF)     # exponent < 128 -> |x| < 2
    q, k, v = (oracle.decode16(a, dtype) for a in (qb, kb, vb))
    want_o, want_l = oracle.attn_f64(q, k, v, causal, 0.2)
    o, lse = oracle.attn_rows(qb, kb, vb, dtype, causal, 0.2)
    np.testing.assert_array_equal(o, want_o)
    np.testing.assert_array_equal(lse, want_l)
    rows = np.array([0, 5, S - 1, S, (B * Hq) * S - 1, 3 * S + 7], dtype=np.int64)
    o2, l2 = oracle.attn_rows(qb, kb, vb, dtype, causal, 0.2, rows=rows)
    np.testing.assert_array_equal(o2, want_o.reshape(-1, D)[rows])
    np.testing.assert_array_equal(l2, want_l.reshape(-1)[rows])


def test_bad_arguments_rejected():
    q = np.zeros((1, 3, 4, 2))
    k = np.zeros((1, 2, 4, 2))
    with pytest.raises(RuntimeError):
        oracle.attn_f64(q, k, k, False, 1.0)          # Hq % Hkv != 0


# ---------------------------------------------------------------------------
# decode-time attention (Section 6 of the paper, workload "DC"): Sq queries, the last positions of
# a sequence of Sk, against all Sk keys
# ---------------------------------------------------------------------------

def rand_cross(seed, B, Hq, Hkv, Sq, Sk, D):
    g = rng(seed)
    return (g.standard_normal((B, Hq, Sq, D)), g.standard_normal((B, Hkv, Sk, D)),
            g.standard_normal((B, Hkv, Sk, D)))


@pytest.mark.parametrize("causal", [False, True])
def test_cross_equals_self_attention_when_Sq_is_Sk(causal):
    q, k, v = rand_qkv(31, 2, 4, 2, 13, 8)
    o1, l1 = oracle.attn_f64(q, k, v, causal, 0.3)
    o2, l2 = oracle.attn_cross_f64(q, k, v, causal, 0.3)
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(l1, l2)


@pytest.mark.parametrize("Sq", [1, 3, 8])
def test_cross_causal_is_the_tail_of_causal_self_attention(Sq):
    # the last Sq rows of a causal self-attention over Sk positions, computed from those queries alone
    Sk = 17
    q, k, v = rand_qkv(32, 2, 6, 3, Sk, 4)
    o_full, l_full = oracle.attn_f64(q, k, v, True, 0.7)
    o, lse = oracle.attn_cross_f64(q[:, :, Sk - Sq:], k, v, True, 0.7)
    np.testing.assert_allclose(o, o_full[:, :, Sk - Sq:], rtol=0, atol=1e-15)
    np.testing.assert_allclose(lse, l_full[:, :, Sk - Sq:], rtol=0, atol=1e-15)


def test_cross_noncausal_is_global_attention_with_padded_queries():
    # without the mask every query sees all keys: same as a global self-attention whose first Sq
    # queries are ours (the other query rows are irrelevant to ours)
    Sq, Sk = 3, 11
    q, k, v = rand_cross(33, 1, 4, 2, Sq, Sk, 8)
    qpad = np.concatenate([q, rng(1).standard_normal((1, 4, Sk - Sq, 8))], axis=2)
    o_full, l_full = oracle.attn_f64(qpad, k, v, False, 0.25)
    o, lse = oracle.attn_cross_f64(q, k, v, False, 0.25)
    np.testing.assert_allclose(o, o_full[:, :, :Sq], rtol=0, atol=1e-15)
    np.testing.assert_allclose(lse, l_full[:, :, :Sq], rtol=0, atol=1e-15)


def test_cross_hand_expanded_Sq2_Sk3_causal():
    # query 0 is position 1 (sees keys 0,1), query 1 is position 2 (sees keys 0,1,2); D = 1
    q = np.array([[[[2.0], [-1.0]]]])
    k = np.array([[[[0.5], [1.0], [-2.0]]]])
    v = np.array([[[[1.0], [10.0], [100.0]]]])
    sc = 0.5
    o, lse = oracle.attn_cross_f64(q, k, v, True, sc)
    e00, e01 = math.exp(sc * 2.0 * 0.5), math.exp(sc * 2.0 * 1.0)
    assert abs(o[0, 0, 0, 0] - (e00 * 1.0 + e01 * 10.0) / (e00 + e01)) < 1e-14
    assert abs(lse[0, 0, 0] - math.log(e00 + e01)) < 1e-14
    f0, f1, f2 = math.exp(sc * -1.0 * 0.5), math.exp(sc * -1.0 * 1.0), math.exp(sc * -1.0 * -2.0)
    assert abs(o[0, 0, 1, 0] - (f0 * 1.0 + f1 * 10.0 + f2 * 100.0) / (f0 + f1 + f2)) < 1e-13
    assert abs(lse[0, 0, 1] - math.log(f0 + f1 + f2)) < 1e-14


def test_cross_closed_forms_and_gqa():
    Sq, Sk = 4, 9
    q, k, v = rand_cross(34, 2, 6, 2, Sq, Sk, 8)
    o, _ = oracle.attn_cross_f64(q, k, np.ones_like(v), True, 0.4)
    np.testing.assert_allclose(o, 1.0, rtol=0, atol=1e-14)
    o, lse = oracle.attn_cross_f64(np.zeros_like(q), k, v, True, 0.4)
    for i in range(Sq):
        n = Sk - Sq + i + 1
        np.testing.assert_allclose(lse[:, :, i], math.log(n), rtol=0, atol=1e-14)
        np.testing.assert_allclose(o[:, :, i], np.repeat(v[:, :, :n].mean(axis=2), 3, axis=1), rtol=0, atol=1e-14)
    # grouped-query == multi-head with each K/V head repeated for its group of consecutive query heads
    o1, l1 = oracle.attn_cross_f64(q, k, v, True, 0.4)
    o2, l2 = oracle.attn_cross_f64(q, np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1), True, 0.4)
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(l1, l2)


@pytest.mark.parametrize("dtype", [oracle.BF16, oracle.F16])
def test_cross16_matches_f64_entry(dtype):
    g = rng(35)
    Sq, Sk = 2, 40
    bits = lambda shape: (g.integers(0, 1 << 15, shape).astype(np.uint16) & (0x3FFF if dtype == oracle.F16 else 0x3FFF)) \
        | (g.integers(0, 2, shape).astype(np.uint16) << 15)
    q, k, v = bits((1, 4, Sq, 8)), bits((1, 2, Sk, 8)), bits((1, 2, Sk, 8))
    o1, l1 = oracle.attn_cross16(q, k, v, dtype, True, 0.35)
    o2, l2 = oracle.attn_cross_f64(oracle.decode16(q, dtype), oracle.decode16(k, dtype), oracle.decode16(v, dtype),
                                   True, 0.35)
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(l1, l2)


def test_cross_bad_arguments_rejected():
    q, k, v = rand_cross(36, 1, 2, 2, 5, 3, 4)
    with pytest.raises(RuntimeError):
        oracle.attn_cross_f64(q, k, v, True, 1.0)   # causal needs Sk >= Sq
    oracle.attn_cross_f64(q, k, v, False, 1.0)      # fine without the mask


# ---------------------------------------------------------------------------
# FP8 (OCP E4M3) inputs, the paper's second precision (Section 6)
# ---------------------------------------------------------------------------

def test_e4m3_decoder_exact_all_codes():
    import torch  # an independent, library decode of all 256 codes (CPU)
    codes = np.arange(256, dtype=np.uint8)
    want = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = oracle.decode_e4m3(codes)
    assert np.isnan(got[[0x7F, 0xFF]]).all() and np.isnan(want[[0x7F, 0xFF]]).all()
    ok = ~np.isnan(want)
    np.testing.assert_array_equal(got[ok], want[ok])
    assert got[0x7E] == 448.0 and got[0x38] == 1.0 and got[0x01] == 2.0 ** -9 and got[0xC6] == -3.5


@pytest.mark.parametrize("causal", [False, True])
def test_e4m3_rows_entry_matches_f64_entry(causal):
    g = rng(41)
    B, Hq, Hkv, S, D = 2, 4, 2, 19, 8
    bits = lambda shape: (g.integers(0, 0x7F, shape).astype(np.uint8) | (g.integers(0, 2, shape).astype(np.uint8) << 7))
    q, k, v = bits((B, Hq, S, D)), bits((B, Hkv, S, D)), bits((B, Hkv, S, D))
    dq, dk, dv = 1 / 64, 1 / 8, 1 / 32
    o1, l1 = oracle.attn_rows_e4m3(q, k, v, dq, dk, dv, causal, 0.35)
    o2, l2 = oracle.attn_f64(dq * oracle.decode_e4m3(q), dk * oracle.decode_e4m3(k), dv * oracle.decode_e4m3(v),
                             causal, 0.35)
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(l1, l2)
    rows = np.array([0, 5, B * Hq * S - 1], dtype=np.int64)
    o3, l3 = oracle.attn_rows_e4m3(q, k, v, dq, dk, dv, causal, 0.35, rows=rows)
    np.testing.assert_array_equal(o3, o2.reshape(-1, D)[rows])
    np.testing.assert_array_equal(l3, l2.reshape(-1)[rows])


def test_e4m3_cross_entry_agrees_with_the_rows_entry_and_with_a_tail():
    """attn_cross_e4m3 (decoder + fp64 cross entry) against attn_rows_e4m3 (its own C path) at Sq = Sk, and
    against the last Sq rows of a causal self-attention over Sk (bottom-right alignment)."""
    from paper_2604_14825_amd import synth
    B, Hq, Hkv, S, D = 2, 4, 2, 37, 64
    dq, dk, dv = 1 / 64, 1 / 8, 1 / 64
    q = synth.fill_e4m3(B, Hq, S, D, 31, synth.TAG_Q, dq)
    k = synth.fill_e4m3(B, Hkv, S, D, 31, synth.TAG_K, dk, 1, 8.0)
    v = synth.fill_e4m3(B, Hkv, S, D, 31, synth.TAG_V, dv)
    for causal in (False, True):
        o1, l1 = oracle.attn_cross_e4m3(q, k, v, dq, dk, dv, causal, 0.2)
        o2, l2 = oracle.attn_rows_e4m3(q, k, v, dq, dk, dv, causal, 0.2)
        np.testing.assert_allclose(o1, o2, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(l1, l2, rtol=1e-12, atol=1e-14)
    Sq = 5
    o_t, l_t = oracle.attn_cross_e4m3(np.ascontiguousarray(q[:, :, S - Sq:]), k, v, dq, dk, dv, True, 0.2)
    o_f, l_f = oracle.attn_rows_e4m3(q, k, v, dq, dk, dv, True, 0.2)
    np.testing.assert_allclose(o_t, o_f[:, :, S - Sq:], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(l_t, l_f[:, :, S - Sq:], rtol=1e-12, atol=1e-14)
