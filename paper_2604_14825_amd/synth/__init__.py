"""Seeded synthetic attention inputs (host side, no attention arithmetic).

The five workloads are the shapes the paper evaluates (operator table of
Section 6: Global / Causal / Grouped-Query attention taken from ViT, 7B-class
LLMs and GLM-4; batch 1 and 8, sequence lengths 2^10..2^15), filled with iid
N(0,1) values rounded to bf16/fp16 in place of the model activations the paper
records, which are not available offline.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "naut_synth.c")
_LIB = os.path.join(_HERE, "libnaut_synth.so")

BF16 = 0
F16 = 1
F32 = 2  # output only

TAG_Q, TAG_K, TAG_V = 1, 2, 3
BASE_SEED = 0x2604_14825


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    S: int
    D: int
    causal: bool
    in_dtype: int
    out_dtype: int
    outlier_frac: float = 0.0
    outlier_scale: float = 1.0

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.D)

    @property
    def n_outlier(self) -> int:
        return int(math.floor(self.outlier_frac * self.S + 1e-9))

    @property
    def flops(self) -> float:
        """4*B*Hq*S^2*D, halved for causal (work actually required)."""
        f = 4.0 * self.B * self.Hq * float(self.S) ** 2 * self.D
        return f / 2 if self.causal else f

    @property
    def io_bytes(self) -> int:
        """Compulsory HBM traffic: Q, K, V read once, O and LSE written once."""
        in_b = 2
        out_b = 4 if self.out_dtype == F32 else 2
        q = self.B * self.Hq * self.S * self.D
        kv = self.B * self.Hkv * self.S * self.D
        return q * in_b + 2 * kv * in_b + q * out_b + self.B * self.Hq * self.S * 4


WORKLOADS = {
    "tiny": Workload("tiny", 1, 2, 2, 256, 64, False, F16, F32),
    "encoder": Workload("encoder", 8, 16, 16, 1024, 64, False, BF16, BF16),
    "prefill": Workload("prefill", 4, 32, 32, 4096, 128, True, BF16, BF16),
    "gqa": Workload("gqa", 2, 64, 8, 8192, 128, True, BF16, BF16),
    "long": Workload("long", 1, 32, 32, 16384, 128, True, BF16, BF16, 0.01, 8.0),
    # not one of the five benchmark configurations: the long shape at the widest head dimension
    "long_d256": Workload("long_d256", 1, 32, 32, 16384, 256, True, BF16, BF16, 0.01, 8.0),
}
WORKLOAD_ORDER = ["tiny", "encoder", "prefill", "gqa", "long"]

_lib = None


def build(force: bool = False) -> str:
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u16p = ctypes.POINTER(ctypes.c_uint16)
        lib.naut_synth_fill.restype = ctypes.c_int
        lib.naut_synth_fill.argtypes = [u16p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                        ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int, ctypes.c_int,
                                        ctypes.c_float]
        lib.naut_synth_outlier_rows.restype = ctypes.c_int
        lib.naut_synth_outlier_rows.argtypes = [ctypes.POINTER(ctypes.c_int32), ctypes.c_int64, ctypes.c_int,
                                                ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int]
        lib.naut_synth_round16.restype = ctypes.c_int
        lib.naut_synth_round16.argtypes = [ctypes.POINTER(ctypes.c_float), u16p, ctypes.c_int64, ctypes.c_int]
        lib.naut_synth_round_e4m3.restype = ctypes.c_int
        lib.naut_synth_round_e4m3.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_uint8),
                                              ctypes.c_int64]
        _lib = lib
    return _lib


def fill(B: int, H: int, S: int, D: int, seed: int, tag: int, dtype: int,
         n_outlier: int = 0, outlier_scale: float = 1.0) -> np.ndarray:
    """uint16 array [B,H,S,D] of N(0,1) samples rounded to `dtype` storage."""
    out = np.empty((B, H, S, D), dtype=np.uint16)
    rc = _load().naut_synth_fill(out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), B, H, S, D,
                                 ctypes.c_uint64(seed & (2 ** 64 - 1)), tag, dtype, n_outlier,
                                 float(outlier_scale))
    if rc != 0:
        raise RuntimeError("naut_synth_fill failed: %d" % rc)
    return out


def outlier_rows(bh: int, S: int, seed: int, tag: int, n_outlier: int) -> np.ndarray:
    rows = np.empty((n_outlier,), dtype=np.int32)
    rc = _load().naut_synth_outlier_rows(rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), bh, S,
                                         ctypes.c_uint64(seed & (2 ** 64 - 1)), tag, n_outlier)
    if rc != 0:
        raise RuntimeError("naut_synth_outlier_rows failed: %d" % rc)
    return rows


def round16(x: np.ndarray, dtype: int) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    rc = _load().naut_synth_round16(x.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                    out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), x.size, dtype)
    if rc != 0:
        raise RuntimeError("naut_synth_round16 failed: %d" % rc)
    return out


def workload_seed(w: Workload) -> int:
    return BASE_SEED + WORKLOAD_ORDER.index(w.name) if w.name in WORKLOAD_ORDER else BASE_SEED + 1000


def make_inputs(w: Workload, seed: int | None = None):
    """(q, k, v) uint16 bit patterns for a workload; K carries the outlier rows."""
    if seed is None:
        seed = workload_seed(w)
    q = fill(w.B, w.Hq, w.S, w.D, seed, TAG_Q, w.in_dtype)
    k = fill(w.B, w.Hkv, w.S, w.D, seed, TAG_K, w.in_dtype, w.n_outlier, w.outlier_scale)
    v = fill(w.B, w.Hkv, w.S, w.D, seed, TAG_V, w.in_dtype)
    return q, k, v


def round_e4m3(x: np.ndarray) -> np.ndarray:
    """float32 -> OCP FP8 E4M3 bytes (nearest even, saturating at +-448)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint8)
    rc = _load().naut_synth_round_e4m3(x.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                       out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), x.size)
    if rc != 0:
        raise RuntimeError("naut_synth_round_e4m3 failed: %d" % rc)
    return out


def fill_e4m3(B: int, H: int, S: int, D: int, seed: int, tag: int, descale: float,
              n_outlier: int = 0, outlier_scale: float = 1.0) -> np.ndarray:
    """uint8 array [B,H,S,D]: the N(0,1) samples of `fill` (with its outlier rows) divided by `descale` and
    stored as FP8 E4M3; the tensor's real values are descale * decoded."""
    bits = fill(B, H, S, D, seed, tag, BF16, n_outlier, outlier_scale)
    x = (bits.astype(np.uint32) << 16).view(np.float32)
    return round_e4m3(x / np.float32(descale))
