"""The pins must be able to fail: plant one plausible mistake at a time in a COPY of the
oracle's source (on the CPU, in a temp dir), and require that the pin suite rejects it."""
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "naut_oracle.c")

MUTANTS = {
    "scores_read_V_instead_of_K": ("acc += qrow[d] * K[j * D + d];", "acc += qrow[d] * V[j * D + d];"),
    "scores_transposed_index": ("acc += qrow[d] * K[j * D + d];", "acc += qrow[d] * K[(j % D) * D + (d + j - j % D) % D];"),
    "dropped_scale": ("s[j] = scale * acc;", "s[j] = acc;"),
    "causal_excludes_diagonal": ("causal ? i + 1 : S", "causal ? (i > 0 ? i : 1) : S"),
    "causal_off_by_one_more": ("causal ? i + 1 : S", "causal ? (i + 2 < S ? i + 2 : S) : S"),
    "gqa_interleaved_map": ("const int64_t hk = h / g;", "const int64_t hk = h % Hkv;"),
    "lse_without_max": ("*lse = m + log(l);", "*lse = log(l);"),
    "no_normalisation": ("s[j] /= l;", ";"),
    "min_instead_of_max": ("if (s[j] > m)", "if (s[j] < m)"),
    "exp_wrong_sign": ("s[j] = exp(s[j] - m);", "s[j] = exp(m - s[j]);"),
    "pv_reversed_d": ("o[d] += s[j] * V[j * D + d];", "o[d] += s[j] * V[j * D + (D - 1 - d)];"),
    "pv_reads_K": ("o[d] += s[j] * V[j * D + d];", "o[d] += s[j] * K[j * D + d];"),
    "f16_bias": ("expo - 15)", "expo - 16)"),
    "bf16_shift": ("(uint32_t)bits << 16", "(uint32_t)bits << 15"),
    "batch_stride": ("const int64_t b = r / ((int64_t)S * Hq);", "const int64_t b = 0;"),
    # decode-time entry points (Sq queries against Sk keys)
    "cross_causal_top_left_aligned": ("causal ? (int64_t)Sk - Sq + i + 1 : Sk", "causal ? i + 1 : Sk"),
    "cross_causal_drops_diagonal": ("causal ? (int64_t)Sk - Sq + i + 1 : Sk", "causal ? (int64_t)Sk - Sq + i + (i > 0 || Sk > Sq ? 0 : 1) : Sk"),
    "cross_kv_head_stride_uses_Sq": ("const double *Kh = k + (b * Hkv + hk) * (int64_t)Sk * D;", "const double *Kh = k + (b * Hkv + hk) * (int64_t)Sq * D;"),
    "cross_row_split_uses_Sk": ("const int64_t h = (r / Sq) % Hq;", "const int64_t h = (r / Sk) % Hq;"),
    "e4m3_bias_8": ("ldexp(1.0 + (double)frac / 8.0, expo - 7)", "ldexp(1.0 + (double)frac / 8.0, expo - 8)"),
    "e4m3_subnormal_step": ("mag = ldexp((double)frac, -9);", "mag = ldexp((double)frac, -10);"),
    "e4m3_four_fraction_bits": ("const int frac = bits & 7;", "const int frac = bits & 15;"),
    "e4m3_scales_swapped": ("V64[t] = dv * decode_e4m3(v[t]);", "V64[t] = dk * decode_e4m3(v[t]);"),
    "cross16_decodes_V_from_K": ("V64[t] = decode16(v[t], in_dtype);\n        }\n        rc =", "V64[t] = decode16(k[t], in_dtype);\n        }\n        rc ="),
}


def run_pins():
    pins.test_hand_expanded_S2_D2_noncausal()
    pins.test_hand_expanded_S3_D1_causal()
    pins.test_hand_expanded_gqa_S2_causal()
    pins.test_hand_expanded_S4_D2_noncausal_row()
    for causal in (False, True):
        pins.test_probs_row_stochastic_and_masked(causal)
        pins.test_all_ones_V_gives_ones(causal)
        pins.test_gqa_equals_repeated_head_mha(causal)
        for hq, hkv in ((2, 2), (4, 1)):
            pins.test_scipy_second_opinion(causal, hq, hkv)
        for dt in (oracle.BF16, oracle.F16):
            pins.test_rows_entry_matches_f64_entry(dt, causal)
    pins.test_zero_Q_gives_column_mean_and_log_count()
    pins.test_key_permutation_invariance_noncausal()
    pins.test_causal_row0_is_V0()
    pins.test_causal_prefix_property()
    pins.test_scale_identity_and_key_shift()
    pins.test_split_merge_identity()
    pins.test_one_hot_limit()
    pins.test_large_scores_do_not_overflow()
    pins.test_decoders_exact_all_patterns()
    for causal in (False, True):
        pins.test_cross_equals_self_attention_when_Sq_is_Sk(causal)
    for sq in (1, 3, 8):
        pins.test_cross_causal_is_the_tail_of_causal_self_attention(sq)
    pins.test_cross_noncausal_is_global_attention_with_padded_queries()
    pins.test_cross_hand_expanded_Sq2_Sk3_causal()
    pins.test_cross_closed_forms_and_gqa()
    for dt in (oracle.BF16, oracle.F16):
        pins.test_cross16_matches_f64_entry(dt)
    pins.test_e4m3_decoder_exact_all_codes()
    for causal in (False, True):
        pins.test_e4m3_rows_entry_matches_f64_entry(causal)


def test_unmutated_copy_passes(tmp_path, monkeypatch):
    lib = tmp_path / "liborig.so"
    subprocess.check_call(["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", SRC, "-o", str(lib), "-lm"])
    monkeypatch.setattr(oracle, "_lib", oracle._bind(str(lib)))
    run_pins()


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_reject_mutant(name, tmp_path, monkeypatch):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) >= 1, "mutation site vanished: " + old
    src = tmp_path / (name + ".c")
    src.write_text(text.replace(old, new))
    lib = tmp_path / (name + ".so")
    subprocess.check_call(["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", "-w", str(src), "-o", str(lib), "-lm"])
    monkeypatch.setattr(oracle, "_lib", oracle._bind(str(lib)))
    with pytest.raises((AssertionError, RuntimeError, FloatingPointError)):
        with __import__("numpy").errstate(all="ignore"):
            run_pins()
