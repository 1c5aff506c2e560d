"""fp64 CPU oracle for softmax attention -- TEST INFRASTRUCTURE ONLY.

Thin ctypes loader around ``naut_oracle.c`` (plain C, three passes per query
row: scores, explicit softmax, weighted sum; Section 1 and the operator table
of Section 6 of the paper define the operator, Appendix B its role as the FP64
unfused reference).  Only the tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the product package never does.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "naut_oracle.c")
_LIB = os.path.join(_HERE, "libnaut_oracle.so")

BF16 = 0
F16 = 1

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE arithmetic, OpenMP over rows)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def build_sanitize_check(out: str, sanitize: bool = True) -> str:
    """Compile sanitize_check.c with the oracle and the generator sources into the executable `out`
    (under -fsanitize=address,undefined unless `sanitize` is False)."""
    root = os.path.dirname(_HERE)
    cmd = ["gcc", "-std=c99", "-O1", "-g", "-fopenmp", "-Wall", "-Wextra"]
    if sanitize:
        cmd += ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan"]
    cmd += [os.path.join(_HERE, "sanitize_check.c"), _SRC,
            os.path.join(root, "paper_2604_14825_amd", "synth", "naut_synth.c"), "-o", out, "-lm"]
    subprocess.check_call(cmd)
    return out


def _bind(path: str):
    """Load one compiled copy of the oracle and declare its signatures."""
    lib = ctypes.CDLL(path)
    dp = ctypes.POINTER(ctypes.c_double)
    u16p = ctypes.POINTER(ctypes.c_uint16)
    i64p = ctypes.POINTER(ctypes.c_int64)
    lib.naut_oracle_attn_f64.restype = ctypes.c_int
    lib.naut_oracle_attn_f64.argtypes = [dp, dp, dp, dp, dp, dp] + [ctypes.c_int] * 6 + [ctypes.c_double]
    lib.naut_oracle_attn_rows.restype = ctypes.c_int
    lib.naut_oracle_attn_rows.argtypes = ([u16p, u16p, u16p, ctypes.c_int, i64p, ctypes.c_int64, dp, dp]
                                          + [ctypes.c_int] * 6 + [ctypes.c_double])
    lib.naut_oracle_attn_cross_f64.restype = ctypes.c_int
    lib.naut_oracle_attn_cross_f64.argtypes = [dp, dp, dp, dp, dp] + [ctypes.c_int] * 7 + [ctypes.c_double]
    lib.naut_oracle_attn_cross16.restype = ctypes.c_int
    lib.naut_oracle_attn_cross16.argtypes = ([u16p, u16p, u16p, ctypes.c_int, dp, dp] + [ctypes.c_int] * 7
                                             + [ctypes.c_double])
    u8p = ctypes.POINTER(ctypes.c_uint8)
    lib.naut_oracle_decode_e4m3.restype = ctypes.c_int
    lib.naut_oracle_decode_e4m3.argtypes = [u8p, dp, ctypes.c_int64]
    lib.naut_oracle_attn_rows_e4m3.restype = ctypes.c_int
    lib.naut_oracle_attn_rows_e4m3.argtypes = ([u8p, u8p, u8p, ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                                i64p, ctypes.c_int64, dp, dp] + [ctypes.c_int] * 6
                                               + [ctypes.c_double])
    lib.naut_oracle_decode16.restype = ctypes.c_int
    lib.naut_oracle_decode16.argtypes = [u16p, ctypes.c_int, dp, ctypes.c_int64]
    lib.naut_oracle_threads.restype = ctypes.c_int
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _bind(build())
    return _lib


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if a is not None else None


def _u16ptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def threads() -> int:
    return int(_load().naut_oracle_threads())


def attn_f64(q, k, v, causal: bool, scale: float, want_probs: bool = False):
    """Attention on fp64 arrays q [B,Hq,S,D], k,v [B,Hkv,S,D] -> (o, lse[, probs])."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    k = np.ascontiguousarray(k, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64)
    B, Hq, S, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (B, Hkv, S, D) and v.shape == k.shape
    o = np.empty((B, Hq, S, D), dtype=np.float64)
    lse = np.empty((B, Hq, S), dtype=np.float64)
    probs = np.empty((B, Hq, S, S), dtype=np.float64) if want_probs else None
    rc = _load().naut_oracle_attn_f64(_dptr(q), _dptr(k), _dptr(v), _dptr(o), _dptr(lse), _dptr(probs),
                                      B, Hq, Hkv, S, D, int(bool(causal)), float(scale))
    if rc != 0:
        raise RuntimeError("naut_oracle_attn_f64 failed: %d" % rc)
    return (o, lse, probs) if want_probs else (o, lse)


def attn_rows(q_bits, k_bits, v_bits, in_dtype: int, causal: bool, scale: float, rows=None):
    """Attention on 16-bit patterns (uint16 arrays shaped like q/k/v) for selected rows.

    rows: int64 array of linear row ids (b*Hq + h)*S + i, or None for all rows.
    Returns (o [n,D] fp64, lse [n] fp64); with rows=None they are reshaped to
    [B,Hq,S,D] and [B,Hq,S].
    """
    for a in (q_bits, k_bits, v_bits):
        assert a.dtype == np.uint16 and a.flags["C_CONTIGUOUS"]
    B, Hq, S, D = q_bits.shape
    Hkv = k_bits.shape[1]
    assert k_bits.shape == (B, Hkv, S, D) and v_bits.shape == k_bits.shape
    if rows is None:
        n = B * Hq * S
        rptr = None
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        n = int(rows.size)
        rptr = rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
    o = np.empty((n, D), dtype=np.float64)
    lse = np.empty((n,), dtype=np.float64)
    rc = _load().naut_oracle_attn_rows(_u16ptr(q_bits), _u16ptr(k_bits), _u16ptr(v_bits), int(in_dtype),
                                       rptr, n, _dptr(o), _dptr(lse), B, Hq, Hkv, S, D,
                                       int(bool(causal)), float(scale))
    if rc != 0:
        raise RuntimeError("naut_oracle_attn_rows failed: %d" % rc)
    if rows is None:
        return o.reshape(B, Hq, S, D), lse.reshape(B, Hq, S)
    return o, lse


def attn_cross_f64(q, k, v, causal: bool, scale: float):
    """Decode-time attention on fp64 arrays: q [B,Hq,Sq,D] (the last Sq positions), k,v [B,Hkv,Sk,D] -> (o, lse)."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    k = np.ascontiguousarray(k, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64)
    B, Hq, Sq, D = q.shape
    Hkv, Sk = k.shape[1], k.shape[2]
    assert k.shape == (B, Hkv, Sk, D) and v.shape == k.shape
    o = np.empty((B, Hq, Sq, D), dtype=np.float64)
    lse = np.empty((B, Hq, Sq), dtype=np.float64)
    rc = _load().naut_oracle_attn_cross_f64(_dptr(q), _dptr(k), _dptr(v), _dptr(o), _dptr(lse), B, Hq, Hkv, Sq, Sk,
                                            D, int(bool(causal)), float(scale))
    if rc != 0:
        raise RuntimeError("naut_oracle_attn_cross_f64 failed: %d" % rc)
    return o, lse


def attn_cross16(q_bits, k_bits, v_bits, in_dtype: int, causal: bool, scale: float):
    """The same on 16-bit patterns (uint16 arrays shaped like q/k/v)."""
    q = np.ascontiguousarray(q_bits, dtype=np.uint16)
    k = np.ascontiguousarray(k_bits, dtype=np.uint16)
    v = np.ascontiguousarray(v_bits, dtype=np.uint16)
    B, Hq, Sq, D = q.shape
    Hkv, Sk = k.shape[1], k.shape[2]
    assert k.shape == (B, Hkv, Sk, D) and v.shape == k.shape
    o = np.empty((B, Hq, Sq, D), dtype=np.float64)
    lse = np.empty((B, Hq, Sq), dtype=np.float64)
    rc = _load().naut_oracle_attn_cross16(_u16ptr(q), _u16ptr(k), _u16ptr(v), int(in_dtype), _dptr(o), _dptr(lse),
                                          B, Hq, Hkv, Sq, Sk, D, int(bool(causal)), float(scale))
    if rc != 0:
        raise RuntimeError("naut_oracle_attn_cross16 failed: %d" % rc)
    return o, lse


def decode16(bits, dtype: int):
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float64)
    rc = _load().naut_oracle_decode16(_u16ptr(bits), int(dtype), _dptr(out), bits.size)
    if rc != 0:
        raise RuntimeError("naut_oracle_decode16 failed: %d" % rc)
    return out


def decode_e4m3(bits):
    """Exact decode of OCP FP8 E4M3 bytes to fp64 (0x7f and 0xff are NaN)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    out = np.empty(bits.shape, dtype=np.float64)
    rc = _load().naut_oracle_decode_e4m3(bits.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), _dptr(out), bits.size)
    if rc != 0:
        raise RuntimeError("naut_oracle_decode_e4m3 failed: %d" % rc)
    return out


def attn_rows_e4m3(q_bits, k_bits, v_bits, dq: float, dk: float, dv: float, causal: bool, scale: float, rows=None):
    """Attention on FP8 E4M3 bytes with per-tensor scales (real tensor = scale * decoded) for selected rows.

    Same conventions as attn_rows."""
    q = np.ascontiguousarray(q_bits, dtype=np.uint8)
    k = np.ascontiguousarray(k_bits, dtype=np.uint8)
    v = np.ascontiguousarray(v_bits, dtype=np.uint8)
    B, Hq, S, D = q.shape
    Hkv = k.shape[1]
    assert k.shape == (B, Hkv, S, D) and v.shape == k.shape
    u8 = lambda a: a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))
    if rows is None:
        n, rp = B * Hq * S, None
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        n, rp = rows.size, rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
    o = np.empty((n, D), dtype=np.float64)
    lse = np.empty((n,), dtype=np.float64)
    rc = _load().naut_oracle_attn_rows_e4m3(u8(q), u8(k), u8(v), float(dq), float(dk), float(dv), rp, n, _dptr(o),
                                            _dptr(lse), B, Hq, Hkv, S, D, int(bool(causal)), float(scale))
    if rc != 0:
        raise RuntimeError("naut_oracle_attn_rows_e4m3 failed: %d" % rc)
    if rows is None:
        return o.reshape(B, Hq, S, D), lse.reshape(B, Hq, S)
    return o, lse


def attn_cross_e4m3(q_bits, k_bits, v_bits, dq: float, dk: float, dv: float, causal: bool, scale: float):
    """Decode-time attention on FP8 E4M3 bytes with per-tensor scales: q [B,Hq,Sq,D] (the last Sq positions),
    k,v [B,Hkv,Sk,D] -> (o, lse).  The exact decoder followed by the fp64 cross-attention entry point (both
    pinned on their own); at Sq = Sk it must agree with attn_rows_e4m3, which is a separate C path."""
    return attn_cross_f64(float(dq) * decode_e4m3(q_bits), float(dk) * decode_e4m3(k_bits),
                          float(dv) * decode_e4m3(v_bits), causal, scale)
