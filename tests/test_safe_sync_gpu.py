"""Race check of the hand-made synchronisation: the library built with -DNAUT_SAFE_SYNC=1 (every bare barrier a
full fence behind a wait for all memory operations, every counted wait a wait for all loads, tile loads issued,
awaited and published before their step computes, every owed wait state paid several times over) must agree
BIT FOR BIT with the shipped library.  The arithmetic and its order are the same in both; a difference is a
race or a missing wait in the fast build."""
import math
import os

import numpy as np
import pytest
import torch

from paper_2604_14825_amd import binding as nb
from paper_2604_14825_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu

_libs = None


def libs():
    global _libs
    if _libs is None:
        assert os.path.exists(nb.LIB_SAFE_PATH), "libnaut_attn_safe.so is missing: python -m paper_2604_14825_amd.build"
        _libs = (nb.lib(), nb.load(nb.LIB_SAFE_PATH))
    return _libs


def both_prefill(q, k, v, idt, odt, causal, scale, what):
    B, Hq, S, D = q.shape
    Hkv = k.shape[1]
    qd, kd, vd = (gu.to_device(a, idt) for a in (q, k, v))
    outs = []
    for L in libs():
        o = torch.full((B, Hq, S, D), float("nan"), dtype=gu.TORCH_DT[odt], device="cuda")
        lse = torch.full((B, Hq, S), float("nan"), dtype=torch.float32, device="cuda")
        rc = L.naut_attn_fwd_dt(qd.data_ptr(), kd.data_ptr(), vd.data_ptr(), o.data_ptr(), lse.data_ptr(), B, Hq, Hkv, S, D,
                                int(causal), scale, None, idt, odt)
        assert rc == 0, L.naut_last_error_string()
        torch.cuda.synchronize()
        outs.append((o.view(torch.int32 if odt == synth.F32 else torch.int16).cpu().numpy(), lse.view(torch.int32).cpu().numpy()))
    assert np.array_equal(outs[0][0], outs[1][0]), what + ": O differs between the fast and the conservative build"
    assert np.array_equal(outs[0][1], outs[1][1]), what + ": LSE differs between the fast and the conservative build"


def make(B, Hq, Hkv, S, D, idt, seed):
    q = synth.fill(B, Hq, S, D, seed, synth.TAG_Q, idt)
    k = synth.fill(B, Hkv, S, D, seed, synth.TAG_K, idt, S // 50, 8.0)
    v = synth.fill(B, Hkv, S, D, seed, synth.TAG_V, idt)
    return q, k, v


SMALL = [
    (1, 1, 1, 1, 64, False, synth.BF16, synth.BF16), (1, 2, 1, 63, 128, True, synth.BF16, synth.BF16),
    (2, 4, 2, 129, 128, True, synth.F16, synth.F16), (1, 3, 1, 200, 64, True, synth.BF16, synth.F32),
    (1, 2, 2, 257, 128, False, synth.BF16, synth.BF16), (1, 8, 2, 511, 64, False, synth.F16, synth.F32),
    (1, 4, 4, 777, 128, True, synth.BF16, synth.BF16), (2, 2, 2, 1024, 64, True, synth.BF16, synth.BF16),
]


@pytest.mark.parametrize("variant", ["w8q32", "w4q64", "bm128"])
@pytest.mark.parametrize("B,Hq,Hkv,S,D,causal,idt,odt", SMALL)
def test_small_shapes_bit_identical(B, Hq, Hkv, S, D, causal, idt, odt, variant, monkeypatch):
    monkeypatch.setenv("NAUT_ATTN_VARIANT", variant)
    q, k, v = make(B, Hq, Hkv, S, D, idt, 21000 + S + D)
    print("safe-sync small", variant, B, Hq, Hkv, S, D, causal, flush=True)
    both_prefill(q, k, v, idt, odt, causal, 1.0 / math.sqrt(D), "small/%s" % variant)


@pytest.mark.parametrize("variant", ["w8q32", "bm128"])
@pytest.mark.parametrize("causal", [True, False])
def test_every_tile_count_bit_identical(variant, causal, monkeypatch):
    """S = 64 t - 1, 64 t and 64 t + 1 for t = 1 .. 9: every phase of the four-buffer rotation, with and without a ragged tail."""
    monkeypatch.setenv("NAUT_ATTN_VARIANT", variant)
    for t in range(1, 10):
        for S in (64 * t - 1, 64 * t, 64 * t + 1):
            q, k, v = make(1, 2, 1, S, 128, synth.BF16, 22000 + S)
            print("safe-sync tiles", variant, causal, S, flush=True)
            both_prefill(q, k, v, synth.BF16, synth.BF16, causal, 1.0 / math.sqrt(128), "tiles S=%d/%s" % (S, variant))


@pytest.mark.parametrize("variant", ["w8q32", "w4q64", "bm128"])
@pytest.mark.parametrize("kind", ["ascending", "descending", "late_spike"])
def test_moving_reference_bit_identical(kind, variant, monkeypatch):
    """The score profiles that drive the rare blocks (reference moves, heavy blocks) of the online softmax."""
    monkeypatch.setenv("NAUT_ATTN_VARIANT", variant)
    B, Hq, Hkv, S, D, idt = 1, 4, 2, 700, 128, synth.BF16
    q = synth.fill(B, Hq, S, D, 4242, synth.TAG_Q, idt)
    k = synth.fill(B, Hkv, S, D, 4242, synth.TAG_K, idt)
    v = synth.fill(B, Hkv, S, D, 4242, synth.TAG_V, idt)
    j = np.arange(S, dtype=np.float32)
    prof = {"ascending": 0.25 + 12.0 * j / max(S - 1, 1), "descending": 12.25 - 12.0 * j / max(S - 1, 1),
            "late_spike": np.where(j == (3 * S) // 4, 60.0, 1.0).astype(np.float32)}[kind]
    kf = (k.astype(np.uint32) << 16).view(np.float32) * prof[None, None, :, None]
    k = synth.round16(kf, idt)
    print("safe-sync profile", kind, variant, flush=True)
    for causal, sc in ((True, 1.0), (False, 4.0)):
        both_prefill(q, k, v, idt, synth.F32, causal, sc / math.sqrt(D), "%s/%s" % (kind, variant))


@pytest.mark.parametrize("D,S,causal,idt,odt", [(256, 333, True, synth.BF16, synth.F32), (256, 500, False, synth.F16, synth.F16),
                                             (256, 1000, True, synth.BF16, synth.BF16), (256, 97, True, synth.BF16, synth.BF16)])
def test_wide_head_bit_identical(D, S, causal, idt, odt):
    """D = 256: direct loads over four buffers, one wavefront per SIMD, asm MFMAs with hand-owed wait states."""
    q, k, v = make(2, 4, 2, S, D, idt, 23000 + S)
    print("safe-sync wide", D, S, causal, flush=True)
    both_prefill(q, k, v, idt, odt, causal, 1.0 / math.sqrt(D), "wide D=%d S=%d" % (D, S))


def test_long_sequence_bit_identical():
    """One long causal head group on the pipelined kernel: hundreds of iterations per work-group."""
    q, k, v = make(1, 8, 8, 8192, 128, synth.BF16, 24000)
    both_prefill(q, k, v, synth.BF16, synth.BF16, True, 1.0 / math.sqrt(128), "long")


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D", [(1, 4, 4, 1, 100, 128), (2, 8, 2, 1, 777, 128), (1, 8, 1, 3, 500, 64),
                                            (1, 16, 2, 5, 300, 128), (2, 32, 8, 1, 16384, 128)])
def test_decode_bit_identical(B, Hq, Hkv, Sq, Sk, D):
    """The decode split kernel counts its own loads over a private double buffer per wavefront."""
    q = synth.fill(B, Hq, Sq, D, 25000 + Sk, synth.TAG_Q, synth.BF16)
    k = synth.fill(B, Hkv, Sk, D, 25000 + Sk, synth.TAG_K, synth.BF16, Sk // 50, 8.0)
    v = synth.fill(B, Hkv, Sk, D, 25000 + Sk, synth.TAG_V, synth.BF16)
    qd, kd, vd = (gu.to_device(a, synth.BF16) for a in (q, k, v))
    outs = []
    print("safe-sync decode", B, Hq, Hkv, Sq, Sk, D, flush=True)
    for L in libs():
        o = torch.full((B, Hq, Sq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        lse = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
        nbytes = L.naut_attn_decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D)
        ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")
        rc = L.naut_attn_decode(qd.data_ptr(), kd.data_ptr(), vd.data_ptr(), o.data_ptr(), lse.data_ptr(), B, Hq, Hkv, Sq, Sk, D,
                                1, 1.0 / math.sqrt(D), ws.data_ptr(), nbytes, None)
        assert rc == 0, L.naut_last_error_string()
        torch.cuda.synchronize()
        outs.append((o.view(torch.int16).cpu().numpy(), lse.view(torch.int32).cpu().numpy()))
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1]), "decode differs"


F8_SCALES = (1.0 / 64, 1.0 / 8, 1.0 / 64)


@pytest.mark.parametrize("B,Hq,Hkv,S,D,causal", [(1, 1, 1, 1, 64, False), (1, 2, 1, 63, 128, True), (2, 2, 2, 64, 64, False),
                                               (1, 2, 2, 65, 128, False), (2, 4, 2, 129, 128, True), (1, 3, 1, 200, 64, True),
                                               (1, 2, 2, 257, 128, False), (1, 8, 2, 400, 96, True), (1, 4, 4, 1024, 128, True),
                                               (1, 4, 2, 777, 48, False)])
def test_fp8_prefill_bit_identical(B, Hq, Hkv, S, D, causal):
    """The FP8 prefill kernel: direct loads a ring of buffers ahead, each wavefront counting its own; S from one
    tile to sixteen covers every phase of the ring and the ragged last tile."""
    dq, dk, dv = F8_SCALES
    q = synth.fill_e4m3(B, Hq, S, D, 26000 + S, synth.TAG_Q, dq)
    k = synth.fill_e4m3(B, Hkv, S, D, 26000 + S, synth.TAG_K, dk, S // 50, 8.0)
    v = synth.fill_e4m3(B, Hkv, S, D, 26000 + S, synth.TAG_V, dv)
    qd, kd, vd = (torch.from_numpy(a).cuda() for a in (q, k, v))
    outs = []
    print("safe-sync fp8", B, Hq, Hkv, S, D, causal, flush=True)
    for L in libs():
        o = torch.full((B, Hq, S, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        lse = torch.full((B, Hq, S), float("nan"), dtype=torch.float32, device="cuda")
        rc = L.naut_attn_fwd_fp8(qd.data_ptr(), kd.data_ptr(), vd.data_ptr(), o.data_ptr(), lse.data_ptr(), B, Hq, Hkv, S, D,
                                 int(causal), 1.0 / math.sqrt(D), dq, dk, dv, None)
        assert rc == 0, L.naut_last_error_string()
        torch.cuda.synchronize()
        outs.append((o.view(torch.int16).cpu().numpy(), lse.view(torch.int32).cpu().numpy()))
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1]), "fp8 prefill differs"


def test_fp8_every_tile_count_bit_identical():
    dq, dk, dv = F8_SCALES
    for t in range(1, 9):
        for S in (64 * t - 1, 64 * t, 64 * t + 1):
            q = synth.fill_e4m3(1, 2, S, 128, 27000 + S, synth.TAG_Q, dq)
            k = synth.fill_e4m3(1, 1, S, 128, 27000 + S, synth.TAG_K, dk)
            v = synth.fill_e4m3(1, 1, S, 128, 27000 + S, synth.TAG_V, dv)
            qd, kd, vd = (torch.from_numpy(a).cuda() for a in (q, k, v))
            outs = []
            print("safe-sync fp8 tiles", S, flush=True)
            for L in libs():
                o = torch.full((1, 2, S, 128), float("nan"), dtype=torch.bfloat16, device="cuda")
                rc = L.naut_attn_fwd_fp8(qd.data_ptr(), kd.data_ptr(), vd.data_ptr(), o.data_ptr(), None, 1, 2, 1, S, 128, 1,
                                         1.0 / math.sqrt(128), dq, dk, dv, None)
                assert rc == 0, L.naut_last_error_string()
                torch.cuda.synchronize()
                outs.append(o.view(torch.int16).cpu().numpy())
            assert np.array_equal(outs[0], outs[1]), "fp8 prefill differs at S = %d" % S


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D", [(1, 4, 4, 1, 100, 128), (2, 8, 2, 1, 777, 128), (1, 8, 1, 3, 500, 64),
                                            (2, 32, 8, 1, 16384, 128)])
def test_fp8_decode_bit_identical(B, Hq, Hkv, Sq, Sk, D):
    dq, dk, dv = F8_SCALES
    q = synth.fill_e4m3(B, Hq, Sq, D, 28000 + Sk, synth.TAG_Q, dq)
    k = synth.fill_e4m3(B, Hkv, Sk, D, 28000 + Sk, synth.TAG_K, dk, Sk // 50, 8.0)
    v = synth.fill_e4m3(B, Hkv, Sk, D, 28000 + Sk, synth.TAG_V, dv)
    qd, kd, vd = (torch.from_numpy(a).cuda() for a in (q, k, v))
    outs = []
    print("safe-sync fp8 decode", B, Hq, Hkv, Sq, Sk, D, flush=True)
    for L in libs():
        o = torch.full((B, Hq, Sq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        lse = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
        nbytes = L.naut_attn_decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D)
        ws = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")
        rc = L.naut_attn_decode_fp8(qd.data_ptr(), kd.data_ptr(), vd.data_ptr(), o.data_ptr(), lse.data_ptr(), B, Hq, Hkv, Sq, Sk,
                                    D, 1, 1.0 / math.sqrt(D), dq, dk, dv, ws.data_ptr(), nbytes, None)
        assert rc == 0, L.naut_last_error_string()
        torch.cuda.synchronize()
        outs.append((o.view(torch.int16).cpu().numpy(), lse.view(torch.int32).cpu().numpy()))
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1]), "fp8 decode differs"
