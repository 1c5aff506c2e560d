"""ctypes binding of the C-ABI library: argument marshalling only.

Every step of the attention forward runs inside ``libnaut_attn.so`` (HIP,
gfx950).  There is no CPU or PyTorch fallback: if the library has not been
built, importing its symbols raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnaut_attn.so")
# the same sources built with -DNAUT_SAFE_SYNC=1 (conservative synchronisation; used by the race check only)
LIB_SAFE_PATH = os.path.join(_HERE, "libnaut_attn_safe.so")

NAUT_OK = 0
NAUT_ERR_NULL = -1
NAUT_ERR_SHAPE = -2
NAUT_ERR_UNSUPPORTED = -3
NAUT_ERR_ALIGN = -4
NAUT_ERR_HIP = -5

NAUT_BF16 = 0
NAUT_F16 = 1
NAUT_F32 = 2

EXPORTS = ("naut_attn_fwd", "naut_attn_fwd_dt", "naut_last_error_string", "naut_version",
           "naut_attn_variant_name", "naut_attn_decode", "naut_attn_decode_dt", "naut_attn_decode_workspace_bytes",
           "naut_attn_fwd_strided", "naut_attn_fwd_fp8", "naut_attn_decode_strided", "naut_attn_fwd_fp8_strided", "naut_attn_decode_fp8", "naut_attn_decode_fp8_strided",
           "naut_attn_decode_static", "naut_probe_mfma")


class NautStrides(ctypes.Structure):
    """Element strides of the batch, head and sequence axes of q, k, v, o (mirror of naut_strides)."""
    _fields_ = [(n, ctypes.c_longlong) for n in ("q_b", "q_h", "q_s", "k_b", "k_h", "k_s", "v_b", "v_h", "v_s",
                                                 "o_b", "o_h", "o_s")]

_lib = None


class NautError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("naut_attn status %d: %s" % (code, msg))
        self.code = code


def load(path: str):
    """A loaded copy of the C-ABI library at `path` with its signatures declared."""
    L = ctypes.CDLL(path)
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    L.naut_attn_fwd.restype = ci
    L.naut_attn_fwd.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, cf, vp]
    L.naut_attn_fwd_dt.restype = ci
    L.naut_attn_fwd_dt.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, cf, vp, ci, ci]
    L.naut_last_error_string.restype = ctypes.c_char_p
    L.naut_last_error_string.argtypes = []
    L.naut_version.restype = ci
    L.naut_version.argtypes = []
    L.naut_attn_variant_name.restype = ctypes.c_char_p
    L.naut_attn_variant_name.argtypes = [ci, ci, ci, ci, ci, ci, ci]
    L.naut_attn_fwd_strided.restype = ci
    L.naut_attn_fwd_strided.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, cf, vp, ci, ci,
                                        ctypes.POINTER(NautStrides)]
    L.naut_attn_fwd_fp8.restype = ci
    L.naut_attn_fwd_fp8.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, cf, cf, cf, cf, vp]
    sz = ctypes.c_size_t
    L.naut_attn_decode.restype = ci
    L.naut_attn_decode.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, cf, vp, sz, vp]
    L.naut_attn_decode_dt.restype = ci
    L.naut_attn_decode_dt.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, cf, vp, sz, vp, ci, ci]
    L.naut_attn_decode_workspace_bytes.restype = sz
    L.naut_attn_decode_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci]
    L.naut_attn_fwd_fp8_strided.restype = ci
    L.naut_attn_fwd_fp8_strided.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, cf, cf, cf, cf, vp,
                                            ctypes.POINTER(NautStrides)]
    L.naut_attn_decode_fp8.restype = ci
    L.naut_attn_decode_fp8.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, cf, cf, cf, cf, vp, sz, vp]
    L.naut_attn_decode_fp8_strided.restype = ci
    L.naut_attn_decode_fp8_strided.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, cf, cf, cf, cf, vp, sz, vp,
                                               ctypes.POINTER(NautStrides)]
    L.naut_attn_decode_strided.restype = ci
    L.naut_attn_decode_strided.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, cf, vp, sz, vp, ci, ci,
                                           ctypes.POINTER(NautStrides)]
    L.naut_probe_mfma.restype = ci
    L.naut_probe_mfma.argtypes = [vp, sz, ci, ci, ci, vp]
    L.naut_attn_decode_static.restype = ci
    L.naut_attn_decode_static.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, cf, vp]
    return L


def lib():
    """The loaded C-ABI library (raises if it was never built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libnaut_attn.so is missing: build it with `python -m paper_2604_14825_amd.build` "
                "(there is no fallback implementation)")
        _lib = load(LIB_PATH)
    return _lib


def last_error_string() -> str:
    return lib().naut_last_error_string().decode()


def version() -> int:
    return int(lib().naut_version())


def variant_name(B: int, Hq: int, S: int, D: int, causal: bool, in_dtype: int, out_dtype: int):
    r = lib().naut_attn_variant_name(B, Hq, S, D, int(bool(causal)), in_dtype, out_dtype)
    return r.decode() if r is not None else None


def naut_attn_fwd_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, S, D, causal, scale, stream_ptr,
                      in_dtype=None, out_dtype=None) -> int:
    """Direct call with integer device addresses; returns the status code."""
    L = lib()
    if in_dtype is None and out_dtype is None:
        return int(L.naut_attn_fwd(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, S, D, int(causal),
                                   float(scale), stream_ptr))
    return int(L.naut_attn_fwd_dt(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, S, D, int(causal),
                                  float(scale), stream_ptr, int(in_dtype), int(out_dtype)))


def _torch_dtype_code(t):
    import torch
    return {torch.bfloat16: NAUT_BF16, torch.float16: NAUT_F16, torch.float32: NAUT_F32}[t.dtype]


def naut_attn_fwd(q, k, v, o, lse, causal: bool, scale: float, stream=None):
    """Fused attention forward on torch device tensors (used for memory and streams only).

    q,o [B,Hq,S,D]; k,v [B,Hkv,S,D]; lse [B,Hq,S] fp32 or None; all contiguous, on one GPU.
    Enqueues on `stream` (a torch.cuda.Stream; default: the current stream) and returns.
    """
    import torch
    for t in (q, k, v, o):
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError("q, k, v, o must be contiguous device tensors")
    B, Hq, S, D = q.shape
    Hkv = k.shape[1]
    if tuple(k.shape) != (B, Hkv, S, D) or tuple(v.shape) != (B, Hkv, S, D) or tuple(o.shape) != (B, Hq, S, D):
        raise ValueError("shape mismatch between q, k, v, o")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v must share one dtype")
    lse_ptr = None
    if lse is not None:
        if not (lse.is_cuda and lse.is_contiguous() and lse.dtype == torch.float32 and tuple(lse.shape) == (B, Hq, S)):
            raise ValueError("lse must be a contiguous fp32 device tensor [B,Hq,S]")
        lse_ptr = lse.data_ptr()
    if stream is None:
        stream = torch.cuda.current_stream(q.device)
    in_dt, out_dt = _torch_dtype_code(q), _torch_dtype_code(o)
    if in_dt == NAUT_BF16 and out_dt == NAUT_BF16:
        rc = naut_attn_fwd_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse_ptr, B, Hq, Hkv, S, D,
                               causal, scale, stream.cuda_stream)
    else:
        rc = naut_attn_fwd_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse_ptr, B, Hq, Hkv, S, D,
                               causal, scale, stream.cuda_stream, in_dt, out_dt)
    if rc != NAUT_OK:
        raise NautError(rc, last_error_string())


def decode_workspace_bytes(B: int, Hq: int, Hkv: int, Sq: int, Sk: int, D: int) -> int:
    """Bytes of device workspace naut_attn_decode needs for these sizes (0: unsupported)."""
    return int(lib().naut_attn_decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D))


def naut_attn_decode_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, Sq, Sk, D, causal, scale, ws_ptr, ws_bytes,
                         stream_ptr, in_dtype=None, out_dtype=None) -> int:
    """Direct call with integer device addresses; returns the status code."""
    L = lib()
    if in_dtype is None and out_dtype is None:
        return int(L.naut_attn_decode(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, Sq, Sk, D, int(causal),
                                      float(scale), ws_ptr, ws_bytes, stream_ptr))
    return int(L.naut_attn_decode_dt(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, Sq, Sk, D, int(causal),
                                     float(scale), ws_ptr, ws_bytes, stream_ptr, int(in_dtype), int(out_dtype)))


def naut_attn_decode(q, k, v, o, lse, causal: bool, scale: float, workspace, stream=None):
    """Decode-time attention on torch device tensors (used for memory and streams only).

    q,o [B,Hq,Sq,D] (the last Sq positions); k,v [B,Hkv,Sk,D]; lse [B,Hq,Sq] fp32 or None; workspace: a
    contiguous device tensor of at least decode_workspace_bytes(...) bytes.  Enqueues on `stream`.
    """
    import torch
    for t in (q, k, v, o, workspace):
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError("q, k, v, o and workspace must be contiguous device tensors")
    B, Hq, Sq, D = q.shape
    Hkv, Sk = k.shape[1], k.shape[2]
    if tuple(k.shape) != (B, Hkv, Sk, D) or tuple(v.shape) != (B, Hkv, Sk, D) or tuple(o.shape) != (B, Hq, Sq, D):
        raise ValueError("shape mismatch between q, k, v, o")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v must share one dtype")
    lse_ptr = None
    if lse is not None:
        if not (lse.is_cuda and lse.is_contiguous() and lse.dtype == torch.float32 and tuple(lse.shape) == (B, Hq, Sq)):
            raise ValueError("lse must be a contiguous fp32 device tensor [B,Hq,Sq]")
        lse_ptr = lse.data_ptr()
    if stream is None:
        stream = torch.cuda.current_stream(q.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    in_dt, out_dt = _torch_dtype_code(q), _torch_dtype_code(o)
    if in_dt == NAUT_BF16 and out_dt == NAUT_BF16:
        rc = naut_attn_decode_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse_ptr, B, Hq, Hkv, Sq, Sk,
                                  D, causal, scale, workspace.data_ptr(), ws_bytes, stream.cuda_stream)
    else:
        rc = naut_attn_decode_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse_ptr, B, Hq, Hkv, Sq, Sk,
                                  D, causal, scale, workspace.data_ptr(), ws_bytes, stream.cuda_stream, in_dt, out_dt)
    if rc != NAUT_OK:
        raise NautError(rc, last_error_string())


def naut_attn_decode_static_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, Sq, Sk, D, causal, scale,
                                stream_ptr) -> int:
    """Direct call with integer device addresses; returns the status code."""
    return int(lib().naut_attn_decode_static(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, Sq, Sk, D, int(causal),
                                             float(scale), stream_ptr))


def naut_attn_decode_static(q, k, v, o, lse, causal: bool, scale: float, stream=None):
    """naut_attn_decode without a workspace argument (bf16 tensors; the library's static scratch holds the partials)."""
    import torch
    for t in (q, k, v, o):
        if not (t.is_cuda and t.is_contiguous() and t.dtype == torch.bfloat16):
            raise ValueError("q, k, v, o must be contiguous bf16 device tensors")
    B, Hq, Sq, D = q.shape
    Hkv, Sk = k.shape[1], k.shape[2]
    if tuple(k.shape) != (B, Hkv, Sk, D) or tuple(v.shape) != (B, Hkv, Sk, D) or tuple(o.shape) != (B, Hq, Sq, D):
        raise ValueError("shape mismatch between q, k, v, o")
    lse_ptr = None
    if lse is not None:
        if not (lse.is_cuda and lse.is_contiguous() and lse.dtype == torch.float32 and tuple(lse.shape) == (B, Hq, Sq)):
            raise ValueError("lse must be a contiguous fp32 device tensor [B,Hq,Sq]")
        lse_ptr = lse.data_ptr()
    if stream is None:
        stream = torch.cuda.current_stream(q.device)
    rc = naut_attn_decode_static_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse_ptr, B, Hq, Hkv, Sq,
                                     Sk, D, causal, scale, stream.cuda_stream)
    if rc != NAUT_OK:
        raise NautError(rc, last_error_string())


def naut_attn_decode_strided_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, Sq, Sk, D, causal, scale, ws_ptr,
                                 ws_bytes, stream_ptr, in_dtype, out_dtype, strides) -> int:
    """Direct call with integer device addresses; `strides` is a NautStrides, a 12-tuple or None."""
    if strides is not None and not isinstance(strides, NautStrides):
        strides = NautStrides(*[int(x) for x in strides])
    ref = ctypes.byref(strides) if strides is not None else None
    return int(lib().naut_attn_decode_strided(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, Sq, Sk, D, int(causal),
                                              float(scale), ws_ptr, ws_bytes, stream_ptr, int(in_dtype),
                                              int(out_dtype), ref))


def naut_attn_decode_strided(q, k, v, o, lse, causal: bool, scale: float, workspace, stream=None):
    """Decode-time attention on torch device tensors indexed q,o [B,Hq,Sq,D] and k,v [B,Hkv,Sk,D] with arbitrary
    batch/head/sequence strides (e.g. `cache.transpose(1, 2)` of a [B,Sk,Hkv,D] cache); the D axis contiguous.
    lse: contiguous fp32 [B,Hq,Sq] or None; workspace: contiguous, at least decode_workspace_bytes(...) bytes."""
    import torch
    for t in (q, k, v, o):
        if not (t.is_cuda and t.dim() == 4 and t.stride(3) == 1):
            raise ValueError("q, k, v, o must be 4-d device tensors with a contiguous last axis")
    if not (workspace.is_cuda and workspace.is_contiguous()):
        raise ValueError("workspace must be a contiguous device tensor")
    B, Hq, Sq, D = q.shape
    Hkv, Sk = k.shape[1], k.shape[2]
    if tuple(k.shape) != (B, Hkv, Sk, D) or tuple(v.shape) != (B, Hkv, Sk, D) or tuple(o.shape) != (B, Hq, Sq, D):
        raise ValueError("shape mismatch between q, k, v, o")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v must share one dtype")
    lse_ptr = None
    if lse is not None:
        if not (lse.is_cuda and lse.is_contiguous() and lse.dtype == torch.float32 and tuple(lse.shape) == (B, Hq, Sq)):
            raise ValueError("lse must be a contiguous fp32 device tensor [B,Hq,Sq]")
        lse_ptr = lse.data_ptr()
    if stream is None:
        stream = torch.cuda.current_stream(q.device)
    st = NautStrides(*[t.stride(a) for t in (q, k, v, o) for a in (0, 1, 2)])
    rc = naut_attn_decode_strided_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse_ptr, B, Hq, Hkv, Sq,
                                      Sk, D, causal, scale, workspace.data_ptr(),
                                      workspace.numel() * workspace.element_size(), stream.cuda_stream,
                                      _torch_dtype_code(q), _torch_dtype_code(o), st)
    if rc != NAUT_OK:
        raise NautError(rc, last_error_string())


def naut_attn_fwd_strided_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, S, D, causal, scale, stream_ptr,
                              in_dtype, out_dtype, strides) -> int:
    """Direct call with integer device addresses; `strides` is a NautStrides, a 12-tuple or None."""
    if strides is not None and not isinstance(strides, NautStrides):
        strides = NautStrides(*[int(x) for x in strides])
    ref = ctypes.byref(strides) if strides is not None else None
    return int(lib().naut_attn_fwd_strided(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, S, D, int(causal),
                                           float(scale), stream_ptr, int(in_dtype), int(out_dtype), ref))


def naut_attn_fwd_strided(q, k, v, o, lse, causal: bool, scale: float, stream=None):
    """Attention forward on torch device tensors indexed [B,H,S,D] with arbitrary batch/head/sequence strides
    (e.g. `x.transpose(1, 2)` of a [B,S,H,D] tensor); the D axis must be contiguous, D any multiple of 8 <= 256.
    lse: contiguous fp32 [B,Hq,S] or None."""
    import torch
    for t in (q, k, v, o):
        if not (t.is_cuda and t.dim() == 4 and t.stride(3) == 1):
            raise ValueError("q, k, v, o must be 4-d device tensors with a contiguous last axis")
    B, Hq, S, D = q.shape
    Hkv = k.shape[1]
    if tuple(k.shape) != (B, Hkv, S, D) or tuple(v.shape) != (B, Hkv, S, D) or tuple(o.shape) != (B, Hq, S, D):
        raise ValueError("shape mismatch between q, k, v, o")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v must share one dtype")
    lse_ptr = None
    if lse is not None:
        if not (lse.is_cuda and lse.is_contiguous() and lse.dtype == torch.float32 and tuple(lse.shape) == (B, Hq, S)):
            raise ValueError("lse must be a contiguous fp32 device tensor [B,Hq,S]")
        lse_ptr = lse.data_ptr()
    if stream is None:
        stream = torch.cuda.current_stream(q.device)
    st = NautStrides(*[t.stride(a) for t in (q, k, v, o) for a in (0, 1, 2)])
    rc = naut_attn_fwd_strided_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse_ptr, B, Hq, Hkv, S, D,
                                   causal, scale, stream.cuda_stream, _torch_dtype_code(q), _torch_dtype_code(o), st)
    if rc != NAUT_OK:
        raise NautError(rc, last_error_string())


def naut_attn_fwd_fp8_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, S, D, causal, scale, dq, dk, dv,
                          stream_ptr) -> int:
    """Direct call with integer device addresses; returns the status code."""
    return int(lib().naut_attn_fwd_fp8(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, S, D, int(causal), float(scale),
                                       float(dq), float(dk), float(dv), stream_ptr))


def naut_attn_fwd_fp8(q, k, v, o, lse, causal: bool, scale: float, descale_q: float, descale_k: float,
                      descale_v: float, stream=None):
    """Attention forward on FP8 E4M3 inputs: q,k,v uint8 (or float8_e4m3fn) device tensors [B,H,S,D], contiguous;
    o bf16 [B,Hq,S,D]; lse fp32 [B,Hq,S] or None; real tensors are descale_* times the decoded bytes."""
    import torch
    for t in (q, k, v, o):
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError("q, k, v, o must be contiguous device tensors")
    if any(t.element_size() != 1 for t in (q, k, v)) or o.dtype != torch.bfloat16:
        raise ValueError("q, k, v must be 1-byte tensors (E4M3) and o bf16")
    B, Hq, S, D = q.shape
    Hkv = k.shape[1]
    if tuple(k.shape) != (B, Hkv, S, D) or tuple(v.shape) != (B, Hkv, S, D) or tuple(o.shape) != (B, Hq, S, D):
        raise ValueError("shape mismatch between q, k, v, o")
    lse_ptr = None
    if lse is not None:
        if not (lse.is_cuda and lse.is_contiguous() and lse.dtype == torch.float32 and tuple(lse.shape) == (B, Hq, S)):
            raise ValueError("lse must be a contiguous fp32 device tensor [B,Hq,S]")
        lse_ptr = lse.data_ptr()
    if stream is None:
        stream = torch.cuda.current_stream(q.device)
    rc = naut_attn_fwd_fp8_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse_ptr, B, Hq, Hkv, S, D, causal,
                               scale, descale_q, descale_k, descale_v, stream.cuda_stream)
    if rc != NAUT_OK:
        raise NautError(rc, last_error_string())


def naut_attn_fwd_fp8_strided_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, S, D, causal, scale, dq, dk, dv,
                                  stream_ptr, strides) -> int:
    """Direct call with integer device addresses; `strides` is a NautStrides, a 12-tuple or None."""
    if strides is not None and not isinstance(strides, NautStrides):
        strides = NautStrides(*[int(x) for x in strides])
    ref = ctypes.byref(strides) if strides is not None else None
    return int(lib().naut_attn_fwd_fp8_strided(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, S, D, int(causal),
                                               float(scale), float(dq), float(dk), float(dv), stream_ptr, ref))


def naut_attn_fwd_fp8_strided(q, k, v, o, lse, causal: bool, scale: float, descale_q: float, descale_k: float,
                              descale_v: float, stream=None):
    """FP8 attention forward on torch device tensors indexed [B,H,S,D] with arbitrary batch/head/sequence strides
    (the D axis contiguous): q,k,v 1-byte tensors (E4M3), o bf16; lse contiguous fp32 [B,Hq,S] or None."""
    import torch
    for t in (q, k, v, o):
        if not (t.is_cuda and t.dim() == 4 and t.stride(3) == 1):
            raise ValueError("q, k, v, o must be 4-d device tensors with a contiguous last axis")
    if any(t.element_size() != 1 for t in (q, k, v)) or o.dtype != torch.bfloat16:
        raise ValueError("q, k, v must be 1-byte tensors (E4M3) and o bf16")
    B, Hq, S, D = q.shape
    Hkv = k.shape[1]
    if tuple(k.shape) != (B, Hkv, S, D) or tuple(v.shape) != (B, Hkv, S, D) or tuple(o.shape) != (B, Hq, S, D):
        raise ValueError("shape mismatch between q, k, v, o")
    lse_ptr = None
    if lse is not None:
        if not (lse.is_cuda and lse.is_contiguous() and lse.dtype == torch.float32 and tuple(lse.shape) == (B, Hq, S)):
            raise ValueError("lse must be a contiguous fp32 device tensor [B,Hq,S]")
        lse_ptr = lse.data_ptr()
    if stream is None:
        stream = torch.cuda.current_stream(q.device)
    st = NautStrides(*[t.stride(a) for t in (q, k, v, o) for a in (0, 1, 2)])
    rc = naut_attn_fwd_fp8_strided_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse_ptr, B, Hq, Hkv, S, D,
                                       causal, scale, descale_q, descale_k, descale_v, stream.cuda_stream, st)
    if rc != NAUT_OK:
        raise NautError(rc, last_error_string())


def naut_attn_decode_fp8_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, Sq, Sk, D, causal, scale, dq, dk, dv,
                             ws_ptr, ws_bytes, stream_ptr) -> int:
    """Direct call with integer device addresses; returns the status code."""
    return int(lib().naut_attn_decode_fp8(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, Sq, Sk, D, int(causal),
                                          float(scale), float(dq), float(dk), float(dv), ws_ptr, ws_bytes, stream_ptr))


def naut_attn_decode_fp8(q, k, v, o, lse, causal: bool, scale: float, descale_q: float, descale_k: float,
                         descale_v: float, workspace, stream=None):
    """Decode-time attention on FP8 E4M3 tensors: q [B,Hq,Sq,D], k,v [B,Hkv,Sk,D] 1-byte, contiguous; o bf16
    [B,Hq,Sq,D]; lse fp32 [B,Hq,Sq] or None; workspace as for naut_attn_decode."""
    import torch
    for t in (q, k, v, o, workspace):
        if not (t.is_cuda and t.is_contiguous()):
            raise ValueError("q, k, v, o and workspace must be contiguous device tensors")
    if any(t.element_size() != 1 for t in (q, k, v)) or o.dtype != torch.bfloat16:
        raise ValueError("q, k, v must be 1-byte tensors (E4M3) and o bf16")
    B, Hq, Sq, D = q.shape
    Hkv, Sk = k.shape[1], k.shape[2]
    if tuple(k.shape) != (B, Hkv, Sk, D) or tuple(v.shape) != (B, Hkv, Sk, D) or tuple(o.shape) != (B, Hq, Sq, D):
        raise ValueError("shape mismatch between q, k, v, o")
    lse_ptr = None
    if lse is not None:
        if not (lse.is_cuda and lse.is_contiguous() and lse.dtype == torch.float32 and tuple(lse.shape) == (B, Hq, Sq)):
            raise ValueError("lse must be a contiguous fp32 device tensor [B,Hq,Sq]")
        lse_ptr = lse.data_ptr()
    if stream is None:
        stream = torch.cuda.current_stream(q.device)
    rc = naut_attn_decode_fp8_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse_ptr, B, Hq, Hkv, Sq, Sk, D,
                                  causal, scale, descale_q, descale_k, descale_v, workspace.data_ptr(),
                                  workspace.numel() * workspace.element_size(), stream.cuda_stream)
    if rc != NAUT_OK:
        raise NautError(rc, last_error_string())


def naut_attn_decode_fp8_strided_raw(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, Sq, Sk, D, causal, scale, dq, dk,
                                     dv, ws_ptr, ws_bytes, stream_ptr, strides) -> int:
    """Direct call with integer device addresses; `strides` is a NautStrides, a 12-tuple or None."""
    if strides is not None and not isinstance(strides, NautStrides):
        strides = NautStrides(*[int(x) for x in strides])
    ref = ctypes.byref(strides) if strides is not None else None
    return int(lib().naut_attn_decode_fp8_strided(q_ptr, k_ptr, v_ptr, o_ptr, lse_ptr, B, Hq, Hkv, Sq, Sk, D,
                                                  int(causal), float(scale), float(dq), float(dk), float(dv), ws_ptr,
                                                  ws_bytes, stream_ptr, ref))


def naut_attn_decode_fp8_strided(q, k, v, o, lse, causal: bool, scale: float, descale_q: float, descale_k: float,
                                 descale_v: float, workspace, stream=None):
    """FP8 decode-time attention on torch device tensors indexed q,o [B,Hq,Sq,D] and k,v [B,Hkv,Sk,D] with arbitrary
    batch/head/sequence strides (the D axis contiguous): q,k,v 1-byte tensors (E4M3), o bf16; lse contiguous fp32
    [B,Hq,Sq] or None; workspace contiguous, as for naut_attn_decode."""
    import torch
    for t in (q, k, v, o):
        if not (t.is_cuda and t.dim() == 4 and t.stride(3) == 1):
            raise ValueError("q, k, v, o must be 4-d device tensors with a contiguous last axis")
    if not (workspace.is_cuda and workspace.is_contiguous()):
        raise ValueError("workspace must be a contiguous device tensor")
    if any(t.element_size() != 1 for t in (q, k, v)) or o.dtype != torch.bfloat16:
        raise ValueError("q, k, v must be 1-byte tensors (E4M3) and o bf16")
    B, Hq, Sq, D = q.shape
    Hkv, Sk = k.shape[1], k.shape[2]
    if tuple(k.shape) != (B, Hkv, Sk, D) or tuple(v.shape) != (B, Hkv, Sk, D) or tuple(o.shape) != (B, Hq, Sq, D):
        raise ValueError("shape mismatch between q, k, v, o")
    lse_ptr = None
    if lse is not None:
        if not (lse.is_cuda and lse.is_contiguous() and lse.dtype == torch.float32 and tuple(lse.shape) == (B, Hq, Sq)):
            raise ValueError("lse must be a contiguous fp32 device tensor [B,Hq,Sq]")
        lse_ptr = lse.data_ptr()
    if stream is None:
        stream = torch.cuda.current_stream(q.device)
    st = NautStrides(*[t.stride(a) for t in (q, k, v, o) for a in (0, 1, 2)])
    rc = naut_attn_decode_fp8_strided_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse_ptr, B, Hq, Hkv,
                                          Sq, Sk, D, causal, scale, descale_q, descale_k, descale_v,
                                          workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                          stream.cuda_stream, st)
    if rc != NAUT_OK:
        raise NautError(rc, last_error_string())


def naut_probe_mfma(out, work_groups: int, trips: int, kind: int, stream=None) -> float:
    """Enqueue the register-only MFMA loop (see naut_probe_mfma in the header); returns the FLOPs it performs."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(out.device)
    rc = int(lib().naut_probe_mfma(out.data_ptr(), out.numel(), work_groups, trips, kind, stream.cuda_stream))
    if rc != NAUT_OK:
        raise NautError(rc, last_error_string())
    return float(work_groups) * 8 * trips * 16 * 32768
