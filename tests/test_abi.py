"""C-ABI: the library loads, exports what the header declares, and validates arguments on the host
(no compute call needs a GPU here: every check below returns before any HIP call)."""
import ctypes
import os
import re

import pytest

from paper_2604_14825_amd import binding as nb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "naut_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(naut_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_exported():
    syms = declared_symbols()
    assert set(syms) == set(nb.EXPORTS)
    L = ctypes.CDLL(nb.LIB_PATH)
    for s in syms:
        assert hasattr(L, s), s


def test_version_and_variant_name():
    assert nb.version() >= 100
    assert nb.variant_name(1, 32, 16384, 128, True, nb.NAUT_BF16, nb.NAUT_BF16) == "fwd_bm256_w8q32_bn64"
    assert nb.variant_name(1, 2, 256, 64, False, nb.NAUT_F16, nb.NAUT_F32) == "fwd_bm128_w4q32_bn64"
    assert nb.variant_name(8, 16, 1024, 96, False, nb.NAUT_BF16, nb.NAUT_BF16) is None
    assert nb.variant_name(2, 8, 4096, 256, True, nb.NAUT_BF16, nb.NAUT_BF16) == "fwd_bm128_w4q32_bn32"


def test_variant_rule_and_override(monkeypatch):
    """The fixed selection rule on the five benchmark shapes and on a short causal one; the override."""
    monkeypatch.delenv("NAUT_ATTN_VARIANT", raising=False)
    bf = nb.NAUT_BF16
    big, small = "fwd_bm256_w8q32_bn64", "fwd_bm128_w4q32_bn64"
    assert nb.variant_name(1, 2, 256, 64, False, nb.NAUT_F16, nb.NAUT_F32) == small      # tiny
    assert nb.variant_name(8, 16, 1024, 64, False, bf, bf) == small                      # encoder: short key loop
    assert nb.variant_name(4, 32, 4096, 128, True, bf, bf) == big                        # prefill
    assert nb.variant_name(2, 64, 8192, 128, True, bf, bf) == big                        # grouped-query
    assert nb.variant_name(1, 32, 16384, 128, True, bf, bf) == big                       # long
    assert nb.variant_name(1, 512, 512, 128, True, bf, bf) == small                      # many heads, short causal loop
    assert nb.variant_name(1, 8, 4096, 128, False, bf, bf) == small                      # too few work-groups for 256 CUs
    assert nb.variant_name(1, 128, 2048, 128, True, bf, bf) == small                     # causal: 1024 keys per query on average
    assert nb.variant_name(1, 128, 2048, 128, False, bf, bf) == big                      # the same shape without the mask
    assert nb.variant_name(1, 128, 512, 128, False, bf, bf) == small
    assert nb.variant_name(1, 32, 8192, 64, True, bf, bf) == small                       # D = 64: the softmax sets the pace
    assert nb.variant_name(1, 32, 16384, 64, True, bf, bf) == small                      # ... even on long loops with many work-groups
    assert nb.variant_name(1, 8, 16384, 64, True, bf, bf) == big                         # long loop, two tiles per CU
    monkeypatch.setenv("NAUT_ATTN_VARIANT", "w4q64")
    assert nb.variant_name(1, 2, 256, 64, False, bf, bf) == "fwd_bm256_w4q64_bn64"
    monkeypatch.setenv("NAUT_ATTN_VARIANT", "nonsense")   # a name that selects nothing is reported, not ignored
    assert nb.variant_name(1, 32, 16384, 128, True, bf, bf) is None
    assert nb.naut_attn_fwd_raw(A, A, A, A, A, 1, 32, 32, 16384, 128, 1, 0.1, None) == nb.NAUT_ERR_UNSUPPORTED
    assert "NAUT_ATTN_VARIANT" in nb.last_error_string()


A = 0x10000  # a fake, 16-byte aligned, never dereferenced device address


def call(q=A, k=A, v=A, o=A, lse=A, B=1, Hq=2, Hkv=2, S=128, D=64, causal=0, scale=0.125, dt=None):
    if dt is None:
        return nb.naut_attn_fwd_raw(q, k, v, o, lse, B, Hq, Hkv, S, D, causal, scale, None)
    return nb.naut_attn_fwd_raw(q, k, v, o, lse, B, Hq, Hkv, S, D, causal, scale, None, dt[0], dt[1])


@pytest.mark.parametrize("kw,code", [
    (dict(q=None), nb.NAUT_ERR_NULL),
    (dict(k=None), nb.NAUT_ERR_NULL),
    (dict(v=None), nb.NAUT_ERR_NULL),
    (dict(o=None), nb.NAUT_ERR_NULL),
    (dict(B=0), nb.NAUT_ERR_SHAPE),
    (dict(S=0), nb.NAUT_ERR_SHAPE),
    (dict(S=-5), nb.NAUT_ERR_SHAPE),
    (dict(Hq=3, Hkv=2), nb.NAUT_ERR_SHAPE),
    (dict(Hkv=0), nb.NAUT_ERR_SHAPE),
    (dict(scale=float("nan")), nb.NAUT_ERR_SHAPE),
    (dict(scale=float("inf")), nb.NAUT_ERR_SHAPE),
    (dict(scale=-1.0), nb.NAUT_ERR_UNSUPPORTED),
    (dict(D=96), nb.NAUT_ERR_UNSUPPORTED),
    (dict(D=192), nb.NAUT_ERR_UNSUPPORTED),
    (dict(D=512), nb.NAUT_ERR_UNSUPPORTED),
    (dict(dt=(nb.NAUT_F32, nb.NAUT_F32)), nb.NAUT_ERR_UNSUPPORTED),
    (dict(dt=(nb.NAUT_BF16, nb.NAUT_F16)), nb.NAUT_ERR_UNSUPPORTED),
    (dict(dt=(7, 0)), nb.NAUT_ERR_UNSUPPORTED),
    (dict(q=A + 8), nb.NAUT_ERR_ALIGN),
    (dict(o=A + 2), nb.NAUT_ERR_ALIGN),
    (dict(lse=A + 2), nb.NAUT_ERR_ALIGN),
])
def test_argument_validation(kw, code):
    assert call(**kw) == code
    msg = nb.last_error_string()
    assert isinstance(msg, str) and len(msg) > 0


def test_missing_library_is_loud(monkeypatch, tmp_path):
    monkeypatch.setattr(nb, "_lib", None)
    monkeypatch.setattr(nb, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        nb.lib()


def test_decode_argument_checks():
    """Validation of the decode entry point runs on the host before any HIP call."""
    ws = nb.decode_workspace_bytes(1, 8, 2, 1, 4096, 128)
    assert ws > 0 and ws % 16 == 0
    assert nb.decode_workspace_bytes(1, 8, 3, 1, 4096, 128) == 0   # Hq % Hkv
    assert nb.decode_workspace_bytes(1, 8, 2, 1, 4096, 96) == ws   # a narrower head runs on the 128-wide kernel
    assert nb.decode_workspace_bytes(1, 8, 2, 1, 4096, 100) == 0   # D not a multiple of 8
    assert nb.decode_workspace_bytes(1, 8, 2, 1, 4096, 136) > 0    # runs on the 256-wide kernel
    assert nb.decode_workspace_bytes(1, 8, 2, 1, 4096, 136) == nb.decode_workspace_bytes(1, 8, 2, 1, 4096, 256)
    assert nb.decode_workspace_bytes(1, 8, 2, 1, 4096, 264) == 0   # D too wide
    ok = dict(B=1, Hq=8, Hkv=2, Sq=1, Sk=4096, D=128, causal=1, scale=0.1)

    def dec(q=A, k=A, v=A, o=A, lse=A, wsp=A, wsb=ws, **kw):
        a = dict(ok)
        a.update(kw)
        return nb.naut_attn_decode_raw(q, k, v, o, lse, a["B"], a["Hq"], a["Hkv"], a["Sq"], a["Sk"], a["D"], a["causal"],
                                       a["scale"], wsp, wsb, None)
    assert dec(q=None) == nb.NAUT_ERR_NULL
    assert dec(Sk=0) == nb.NAUT_ERR_SHAPE
    assert dec(Hkv=3) == nb.NAUT_ERR_SHAPE
    assert dec(Sq=5000) == nb.NAUT_ERR_SHAPE            # causal needs Sk >= Sq
    assert dec(scale=float("inf")) == nb.NAUT_ERR_SHAPE
    assert dec(scale=-1.0) == nb.NAUT_ERR_UNSUPPORTED
    assert dec(D=96) == nb.NAUT_ERR_UNSUPPORTED
    assert dec(k=A + 8) == nb.NAUT_ERR_ALIGN
    assert dec(wsp=None) == nb.NAUT_ERR_NULL
    assert dec(wsb=ws - 1) == nb.NAUT_ERR_SHAPE
    assert "workspace" in nb.last_error_string()

    # the entry point without a workspace argument: the same checks, all of them before its first HIP call
    def dec0(q=A, k=A, **kw):
        a = dict(ok)
        a.update(kw)
        return nb.naut_attn_decode_static_raw(q, k, A, A, A, a["B"], a["Hq"], a["Hkv"], a["Sq"], a["Sk"], a["D"],
                                              a["causal"], a["scale"], None)
    assert dec0(q=None) == nb.NAUT_ERR_NULL
    assert dec0(Sk=0) == nb.NAUT_ERR_SHAPE
    assert dec0(Sq=5000) == nb.NAUT_ERR_SHAPE
    assert dec0(D=96) == nb.NAUT_ERR_UNSUPPORTED
    assert dec0(k=A + 8) == nb.NAUT_ERR_ALIGN
    assert dec0(B=64, Hq=64, Hkv=64) == nb.NAUT_ERR_UNSUPPORTED   # partials beyond the 16 MiB static scratch
    assert "static scratch" in nb.last_error_string()

    # strided variant: same stride rules as the strided prefill entry point
    bf = nb.NAUT_BF16
    B, Hq, Hkv, Sq, Sk, D = 1, 8, 2, 1, 4096, 128
    good = (Hq * Sq * D, Sq * D, D, Sk * Hkv * D, D, Hkv * D, Sk * Hkv * D, D, Hkv * D, Hq * Sq * D, Sq * D, D)

    def dec_s(strides, q=A, **kw):
        a = dict(ok)
        a.update(kw)
        return nb.naut_attn_decode_strided_raw(q, A, A, A, A, a["B"], a["Hq"], a["Hkv"], a["Sq"], a["Sk"], a["D"],
                                               a["causal"], a["scale"], A, ws, None, bf, bf, strides)
    assert dec_s(good, q=None) == nb.NAUT_ERR_NULL
    assert dec_s(good[:5] + (Hkv * D + 4,) + good[6:]) == nb.NAUT_ERR_ALIGN          # k rows not 16-byte aligned
    assert dec_s(good[:5] + (D - 8,) + good[6:]) == nb.NAUT_ERR_SHAPE                # k rows overlap
    assert dec_s(good[:8] + (1 << 24,) + good[9:]) == nb.NAUT_ERR_UNSUPPORTED        # v row stride too large
    assert dec_s(good[:9] + (0,) + good[10:]) == nb.NAUT_ERR_ALIGN                   # o batch stride must be positive
    assert dec_s(good, D=100) == nb.NAUT_ERR_UNSUPPORTED
    assert dec_s(good, D=264) == nb.NAUT_ERR_UNSUPPORTED


def test_decode_fp8_argument_checks():
    ws = nb.decode_workspace_bytes(1, 8, 2, 1, 4096, 128)

    def d8(q=A, k=A, wsp=A, wsb=ws, B=1, Hq=8, Hkv=2, Sq=1, Sk=4096, D=128, causal=1, scale=0.1, dq=1.0, dk=1.0, dv=1.0):
        return nb.naut_attn_decode_fp8_raw(q, k, A, A, A, B, Hq, Hkv, Sq, Sk, D, causal, scale, dq, dk, dv, wsp, wsb, None)
    assert d8(q=None) == nb.NAUT_ERR_NULL
    assert d8(Sk=0) == nb.NAUT_ERR_SHAPE
    assert d8(Sq=5000) == nb.NAUT_ERR_SHAPE
    assert d8(dk=float("inf")) == nb.NAUT_ERR_SHAPE
    assert d8(dv=0.0) == nb.NAUT_ERR_UNSUPPORTED
    assert d8(D=96) == nb.NAUT_ERR_UNSUPPORTED
    assert d8(k=A + 8) == nb.NAUT_ERR_ALIGN
    assert d8(wsp=None) == nb.NAUT_ERR_NULL
    assert d8(wsb=16) == nb.NAUT_ERR_SHAPE

    # strided variant: any multiple of 16 up to 128, strides in bytes = elements
    B, Hq, Hkv, Sq, Sk, D = 1, 8, 2, 1, 4096, 128
    good = (Hq * Sq * D, Sq * D, D, Sk * Hkv * D, D, Hkv * D, Sk * Hkv * D, D, Hkv * D, Hq * Sq * D, Sq * D, D)

    def d8s(strides, q=A, D=128, wsb=ws):
        return nb.naut_attn_decode_fp8_strided_raw(q, A, A, A, A, B, Hq, Hkv, Sq, Sk, D, 1, 0.1, 1.0, 1.0, 1.0, A, wsb,
                                                   None, strides)
    assert d8s(good, q=None) == nb.NAUT_ERR_NULL
    assert d8s(good, D=72) == nb.NAUT_ERR_UNSUPPORTED                                 # not a multiple of 16
    assert d8s(good, D=144) == nb.NAUT_ERR_UNSUPPORTED                                # wider than the widest FP8 kernel
    assert d8s(good[:5] + (Hkv * D + 8,) + good[6:]) == nb.NAUT_ERR_ALIGN            # k rows not 16-byte aligned
    assert d8s(good[:5] + (D - 16,) + good[6:]) == nb.NAUT_ERR_SHAPE                 # k rows overlap
    assert d8s(good[:8] + (1 << 24,) + good[9:]) == nb.NAUT_ERR_UNSUPPORTED          # v row stride too large
    assert d8s(good[:9] + (0,) + good[10:]) == nb.NAUT_ERR_ALIGN                     # o batch stride must be positive
    assert d8s(good, wsb=16) == nb.NAUT_ERR_SHAPE


def test_strided_argument_checks():
    bf = nb.NAUT_BF16
    D = 96
    base = dict(q=A, k=A, v=A, o=A, lse=A, B=1, Hq=2, Hkv=2, S=128, D=D, causal=1, scale=0.1)

    def call_s(strides, **kw):
        a = dict(base)
        a.update(kw)
        return nb.naut_attn_fwd_strided_raw(a["q"], a["k"], a["v"], a["o"], a["lse"], a["B"], a["Hq"], a["Hkv"], a["S"],
                                            a["D"], a["causal"], a["scale"], None, bf, bf, strides)
    bshd = lambda H, S, D: (S * H * D, D, H * D)
    good = bshd(2, 128, D) * 4
    assert call_s(good, D=100) == nb.NAUT_ERR_UNSUPPORTED     # not a multiple of 8
    assert call_s(good, D=264) == nb.NAUT_ERR_UNSUPPORTED     # wider than the widest kernel
    assert call_s((good[0], good[1], good[2] + 4) + good[3:]) == nb.NAUT_ERR_ALIGN    # q rows not 16-byte aligned
    assert call_s(good[:9] + (good[9], good[10], 0)) == nb.NAUT_ERR_ALIGN             # o rows would coincide
    assert call_s(good[:5] + (D - 8,) + good[6:]) == nb.NAUT_ERR_SHAPE                # k rows overlap
    assert call_s(good[:8] + (1 << 24,) + good[9:]) == nb.NAUT_ERR_UNSUPPORTED        # v row stride too large
    assert call_s(good, q=None) == nb.NAUT_ERR_NULL
    # the dense entry points keep their contract: only 64, 128 and 256
    assert call(D=96) == nb.NAUT_ERR_UNSUPPORTED


def test_fp8_argument_checks():
    def f8(q=A, k=A, v=A, o=A, lse=A, B=1, Hq=2, Hkv=2, S=128, D=128, causal=1, scale=0.1, dq=1.0, dk=1.0, dv=1.0):
        return nb.naut_attn_fwd_fp8_raw(q, k, v, o, lse, B, Hq, Hkv, S, D, causal, scale, dq, dk, dv, None)
    assert f8(v=None) == nb.NAUT_ERR_NULL
    assert f8(S=0) == nb.NAUT_ERR_SHAPE
    assert f8(Hkv=3) == nb.NAUT_ERR_SHAPE
    assert f8(dk=float("nan")) == nb.NAUT_ERR_SHAPE
    assert f8(dq=0.0) == nb.NAUT_ERR_UNSUPPORTED
    assert f8(D=24) == nb.NAUT_ERR_UNSUPPORTED       # not a multiple of 16
    assert f8(D=144) == nb.NAUT_ERR_UNSUPPORTED      # wider than the widest FP8 kernel
    assert f8(q=A + 4) == nb.NAUT_ERR_ALIGN

    def f8s(strides, **kw):
        a = dict(q=A, B=1, Hq=2, Hkv=2, S=128, D=128)
        a.update(kw)
        return nb.naut_attn_fwd_fp8_strided_raw(a["q"], A, A, A, A, a["B"], a["Hq"], a["Hkv"], a["S"], a["D"], 1, 0.1,
                                                1.0, 1.0, 1.0, None, strides)
    H, S, D = 2, 128, 128
    good = (S * H * D, D, H * D) * 4                                                  # sequence-major
    assert f8s(good, q=None) == nb.NAUT_ERR_NULL
    assert f8s(good, D=72) == nb.NAUT_ERR_UNSUPPORTED
    assert f8s(good[:2] + (H * D + 8,) + good[3:]) == nb.NAUT_ERR_ALIGN              # q rows not 16-byte aligned
    assert f8s(good[:5] + (D - 16,) + good[6:]) == nb.NAUT_ERR_SHAPE                 # k rows overlap
    assert f8s(good[:8] + (1 << 24,) + good[9:]) == nb.NAUT_ERR_UNSUPPORTED          # v row stride too large
    assert f8s(good[:11] + (0,)) == nb.NAUT_ERR_ALIGN                                # o rows would coincide
