"""GPU parity of decode-time attention (through the C ABI) against the fp64 oracle on identical seeded inputs."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2604_14825_amd import binding as nb
from paper_2604_14825_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu

CASES = [
    # B, Hq, Hkv, Sq, Sk, D, causal, in, out   (R = Hq/Hkv*Sq rows share a K/V head; 32 rows per work-group)
    (1, 1, 1, 1, 1, 64, False, synth.BF16, synth.BF16),        # one key
    (1, 2, 2, 1, 31, 128, True, synth.BF16, synth.BF16),       # less than one block
    (1, 4, 4, 1, 100, 128, True, synth.BF16, synth.BF16),      # ragged last block
    (2, 8, 2, 1, 777, 128, True, synth.BF16, synth.F32),       # grouped-query, R = 4
    (1, 8, 1, 3, 500, 64, True, synth.F16, synth.F16),         # R = 24, three positions, D = 64
    (1, 16, 2, 5, 300, 128, True, synth.BF16, synth.BF16),     # R = 40: two row chunks
    (1, 2, 2, 1, 4096, 128, False, synth.BF16, synth.BF16),    # many splits
    (1, 2, 1, 64, 64, 64, True, synth.BF16, synth.F32),        # Sq == Sk: plain causal self-attention, R = 128
    (2, 4, 4, 7, 1000, 64, False, synth.F16, synth.F32),       # no mask, several positions
    (3, 6, 3, 2, 2049, 128, True, synth.BF16, synth.BF16),     # odd sizes everywhere
]


def make(B, Hq, Hkv, Sq, Sk, D, idt, seed, n_outlier=0):
    q = synth.fill(B, Hq, Sq, D, seed, synth.TAG_Q, idt)
    k = synth.fill(B, Hkv, Sk, D, seed, synth.TAG_K, idt, n_outlier, 8.0)
    v = synth.fill(B, Hkv, Sk, D, seed, synth.TAG_V, idt)
    return q, k, v


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D,causal,idt,odt", CASES)
def test_decode_elementwise(B, Hq, Hkv, Sq, Sk, D, causal, idt, odt):
    q, k, v = make(B, Hq, Hkv, Sq, Sk, D, idt, 7000 + Sk + D + Sq, Sk // 50)
    scale = 1.0 / math.sqrt(D)
    print("decode case", B, Hq, Hkv, Sq, Sk, D, causal, idt, odt, flush=True)
    o, lse = gu.run_hip_decode(q, k, v, idt, odt, causal, scale)
    o_ref, lse_ref = oracle.attn_cross16(q, k, v, idt, causal, scale)
    gu.check(o, lse, o_ref, lse_ref, "decode")


def test_decode_long_cache_gqa():
    """A cache of the benchmark's length: B=2, 32 query heads on 8 K/V heads, one new position, Sk = 16384."""
    B, Hq, Hkv, Sq, Sk, D = 2, 32, 8, 1, 16384, 128
    q, k, v = make(B, Hq, Hkv, Sq, Sk, D, synth.BF16, 7777, Sk // 100)
    scale = 1.0 / math.sqrt(D)
    o, lse = gu.run_hip_decode(q, k, v, synth.BF16, synth.BF16, True, scale)
    o_ref, lse_ref = oracle.attn_cross16(q, k, v, synth.BF16, True, scale)
    gu.check(o, lse, o_ref, lse_ref, "decode long")


def test_decode_matches_prefill_tail():
    """The last Sq rows of the prefill kernel's causal self-attention and the decode path agree with the
    oracle (and hence with each other to twice the tolerance)."""
    B, Hq, Hkv, S, D, Sq = 1, 4, 2, 640, 128, 4
    q, k, v = make(B, Hq, Hkv, S, S, D, synth.BF16, 7100)
    scale = 1.0 / math.sqrt(D)
    o_full, lse_full = gu.run_hip(q, k, v, synth.BF16, synth.F32, True, scale)
    o_dec, lse_dec = gu.run_hip_decode(np.ascontiguousarray(q[:, :, S - Sq:]), k, v, synth.BF16, synth.F32, True, scale)
    assert np.abs(o_dec - o_full[:, :, S - Sq:]).max() <= 2 * gu.TOL_MAX
    assert np.abs(lse_dec - lse_full[:, :, S - Sq:]).max() <= 2e-3 * np.maximum(1.0, np.abs(lse_dec)).max()
    o_ref, lse_ref = oracle.attn_cross16(np.ascontiguousarray(q[:, :, S - Sq:]), k, v, synth.BF16, True, scale)
    gu.check(o_dec, lse_dec, o_ref, lse_ref, "decode tail")


def test_decode_moving_maximum_and_hot_softmax():
    """Keys that grow along the cache (the reference maximum keeps moving inside every split, and differs
    wildly between splits) at four times the usual softmax temperature."""
    B, Hq, Hkv, Sq, Sk, D = 1, 8, 2, 2, 3000, 128
    q, k, v = make(B, Hq, Hkv, Sq, Sk, D, synth.BF16, 7200)
    kf = (k.astype(np.uint32) << 16).view(np.float32) * (0.25 + 12.0 * np.arange(Sk, dtype=np.float32) / (Sk - 1))[None, None, :, None]
    k = synth.round16(kf, synth.BF16)
    scale = 4.0 / math.sqrt(D)
    o, lse = gu.run_hip_decode(q, k, v, synth.BF16, synth.F32, True, scale)
    o_ref, lse_ref = oracle.attn_cross16(q, k, v, synth.BF16, True, scale)
    gu.check(o, lse, o_ref, lse_ref, "decode ascending")


def test_decode_bit_identical_and_lse_optional():
    B, Hq, Hkv, Sq, Sk, D = 2, 8, 4, 1, 5000, 128
    q, k, v = make(B, Hq, Hkv, Sq, Sk, D, synth.BF16, 7300)
    scale = 1.0 / math.sqrt(D)
    o1, l1 = gu.run_hip_decode(q, k, v, synth.BF16, synth.BF16, True, scale)
    o2, _ = gu.run_hip_decode(q, k, v, synth.BF16, synth.BF16, True, scale, want_lse=False, poison_workspace=False)
    assert np.array_equal(o1, o2)


def test_decode_rejects_short_workspace():
    B, Hq, Hkv, Sq, Sk, D = 1, 2, 2, 1, 1024, 128
    q = torch.zeros((B, Hq, Sq, D), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((B, Hkv, Sk, D), dtype=torch.bfloat16, device="cuda")
    o = torch.zeros_like(q)
    need = nb.decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D)
    ws = torch.empty(need - 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(nb.NautError) as e:
        nb.naut_attn_decode(q, k, k, o, None, True, 0.1, ws)
    assert e.value.code == nb.NAUT_ERR_SHAPE


def _bshd(a, dt):
    """Device copy stored [B][S][H][D], returned as the logical [B,H,S,D] view."""
    return gu.to_device(np.ascontiguousarray(a.transpose(0, 2, 1, 3)), dt).transpose(1, 2)


@pytest.mark.parametrize("B,Hq,Hkv,Sq,Sk,D,causal,idt,odt", [
    (2, 8, 2, 1, 777, 128, True, synth.BF16, synth.BF16),
    (1, 16, 2, 5, 300, 128, True, synth.BF16, synth.F32),
    (3, 6, 3, 2, 2049, 64, True, synth.F16, synth.F16),
    (2, 4, 4, 7, 1000, 64, False, synth.BF16, synth.BF16),
    (2, 8, 2, 1, 1500, 256, True, synth.BF16, synth.BF16),
    (1, 6, 3, 2, 700, 192, True, synth.F16, synth.F32),
])
def test_decode_sequence_major_cache(B, Hq, Hkv, Sq, Sk, D, causal, idt, odt):
    """K/V cache and queries stored [B][S][H][D]; O written in the same layout; the gaps of a padded O untouched."""
    q, k, v = make(B, Hq, Hkv, Sq, Sk, D, idt, 7500 + Sk + D + Sq, Sk // 50)
    scale = 1.0 / math.sqrt(D)
    qd, kd, vd = _bshd(q, idt), _bshd(k, idt), _bshd(v, idt)
    assert not kd.is_contiguous()
    P = D + 16                                                            # O rows padded to a wider pitch
    o_mem = torch.full((B, Sq, Hq, P), 7.0, dtype=gu.TORCH_DT[odt], device="cuda")
    od = o_mem[..., :D].transpose(1, 2)
    lse = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(nb.decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    print("decode bshd", B, Hq, Hkv, Sq, Sk, D, flush=True)
    nb.naut_attn_decode_strided(qd, kd, vd, od, lse, causal, scale, ws)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attn_cross16(q, k, v, idt, causal, scale)
    gu.check(od.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, "decode bshd")
    assert torch.all(o_mem[..., D:] == 7.0).item(), "the gaps between O rows were written"


def test_decode_shared_cache_and_padded_rows():
    """One K/V cache shared by every batch entry (batch stride 0), rows padded to a wider pitch with NaN gaps."""
    B, Hq, Hkv, Sq, Sk, D, idt = 3, 8, 2, 1, 1200, 128, synth.BF16
    q, k, v = make(B, Hq, Hkv, Sq, Sk, D, idt, 7600, Sk // 50)
    k[1:], v[1:] = k[0], v[0]
    scale = 1.0 / math.sqrt(D)

    def padded_shared(a):
        buf = np.full((1, Hkv, Sk, D + 64), 0x7FC0, dtype=np.uint16)     # bf16 NaN in the gaps
        buf[..., :D] = a[:1]
        return gu.to_device(buf, idt)[..., :D].expand(B, Hkv, Sk, D)
    kd, vd = padded_shared(k), padded_shared(v)
    assert kd.stride(0) == 0 and kd.stride(2) == D + 64
    qd = gu.to_device(q, idt)
    od = torch.full((B, Hq, Sq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(nb.decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D), dtype=torch.uint8, device="cuda")
    nb.naut_attn_decode_strided(qd, kd, vd, od, lse, True, scale, ws)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attn_cross16(q, k, v, idt, True, scale)
    gu.check(od.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, "decode shared cache")


@pytest.mark.parametrize("D,B,Hq,Hkv,Sq,Sk,causal,idt,odt", [
    (8, 1, 4, 2, 1, 300, True, synth.BF16, synth.F32),
    (40, 2, 8, 2, 3, 777, True, synth.BF16, synth.BF16),
    (80, 1, 16, 2, 5, 500, False, synth.F16, synth.F16),
    (96, 2, 4, 4, 1, 2049, True, synth.BF16, synth.BF16),
    (112, 1, 8, 1, 2, 1000, True, synth.F16, synth.F32),
    (256, 1, 1, 1, 1, 1, False, synth.BF16, synth.BF16),       # the 256-wide kernel: one key
    (256, 1, 2, 2, 1, 31, True, synth.BF16, synth.F32),        # less than one block
    (256, 2, 8, 2, 1, 777, True, synth.BF16, synth.BF16),      # grouped-query, ragged last block
    (256, 1, 16, 2, 5, 300, True, synth.F16, synth.F16),       # R = 40: two row chunks
    (256, 1, 2, 2, 1, 4096, False, synth.BF16, synth.BF16),    # many splits
    (256, 1, 2, 1, 64, 64, True, synth.F16, synth.F32),        # Sq == Sk, R = 128
    (256, 3, 6, 3, 2, 2049, True, synth.BF16, synth.BF16),     # odd sizes everywhere
    (136, 2, 4, 2, 1, 500, True, synth.BF16, synth.BF16),      # narrower heads on the 256-wide kernel
    (192, 1, 8, 2, 3, 1000, True, synth.BF16, synth.F32),
    (248, 1, 4, 4, 2, 333, False, synth.F16, synth.F16),
])
def test_decode_other_head_dimensions(D, B, Hq, Hkv, Sq, Sk, causal, idt, odt):
    """Multiples of 8 other than 64 and 128, up to 256, run on the next wider decode kernel (strided entry point,
    contiguous tensors: a chunk read past a row's end would show up as the next row's data)."""
    q, k, v = make(B, Hq, Hkv, Sq, Sk, D, idt, 7700 + Sk + D, Sk // 50)
    scale = 1.0 / math.sqrt(D)
    qd, kd, vd = (gu.to_device(a, idt) for a in (q, k, v))
    od = torch.full((B, Hq, Sq, D), float("nan"), dtype=gu.TORCH_DT[odt], device="cuda")
    lse = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(nb.decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    print("decode head dim", D, flush=True)
    nb.naut_attn_decode_strided(qd, kd, vd, od, lse, causal, scale, ws)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attn_cross16(q, k, v, idt, causal, scale)
    gu.check(od.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, "decode D=%d" % D)


def test_decode_long_cache_wide_heads():
    """The benchmark's cache length at the widest head: B=2, 16 query heads on 4 K/V heads of D = 256, Sk = 16384."""
    B, Hq, Hkv, Sq, Sk, D = 2, 16, 4, 1, 16384, 256
    q, k, v = make(B, Hq, Hkv, Sq, Sk, D, synth.BF16, 7878, Sk // 100)
    scale = 1.0 / math.sqrt(D)
    qd, kd, vd = (gu.to_device(a, synth.BF16) for a in (q, k, v))
    od = torch.full((B, Hq, Sq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(nb.decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D), dtype=torch.uint8, device="cuda")
    ws.fill_(0xFF)
    nb.naut_attn_decode_strided(qd, kd, vd, od, lse, True, scale, ws)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attn_cross16(q, k, v, synth.BF16, True, scale)
    gu.check(od.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, "decode long D=256")


@pytest.mark.parametrize("D", [64, 128, 256])
def test_decode_cache_rows_16_mib_apart(D):
    """K and V rows at the largest row stride the entry point admits (2^23 elements): Sk times the stride passes
    2^32 bytes, so block addresses must be formed in 64 bits, and 31 rows of it must fit the 32-bit offsets."""
    B, Hq, Hkv, Sq, Sk, idt = 1, 4, 1, 1, 300, synth.BF16
    stride = 1 << 23
    q, k, v = make(B, Hq, Hkv, Sq, Sk, D, idt, 7900 + D)
    scale = 1.0 / math.sqrt(D)

    def spread(a):
        buf = torch.empty(Sk * stride, dtype=torch.bfloat16, device="cuda")  # 4.7 GiB, rows at the start of each pitch
        rows = buf.view(Sk, stride)[:, :D]
        rows.copy_(gu.to_device(a, idt)[0, 0])
        return rows.unsqueeze(0).unsqueeze(0)  # logical [1,1,Sk,D]
    kd, vd = spread(k), spread(v)
    assert kd.stride(2) * 2 * Sk > 1 << 32
    od = torch.full((B, Hq, Sq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(nb.decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D), dtype=torch.uint8, device="cuda")
    print("decode, 16 MiB row stride", D, flush=True)
    nb.naut_attn_decode_strided(gu.to_device(q, idt), kd, vd, od, lse, True, scale, ws)
    torch.cuda.synchronize()
    o_ref, lse_ref = oracle.attn_cross16(q, k, v, idt, True, scale)
    gu.check(od.double().cpu().numpy(), lse.double().cpu().numpy(), o_ref, lse_ref, "decode D=%d, row stride 2^23" % D)


@pytest.mark.parametrize("Sk,Sq", [(131072, 1), (100003, 3)])
def test_decode_very_long_cache(Sk, Sq):
    """Caches well beyond the benchmark's 16k positions (many splits per head, ragged last block)."""
    B, Hq, Hkv, D, idt = 1, 8, 2, 128, synth.BF16
    q, k, v = make(B, Hq, Hkv, Sq, Sk, D, idt, 7950 + Sq, Sk // 100)
    scale = 1.0 / math.sqrt(D)
    print("decode very long cache", Sk, Sq, flush=True)
    o, lse = gu.run_hip_decode(q, k, v, idt, idt, True, scale)
    o_ref, lse_ref = oracle.attn_cross16(q, k, v, idt, True, scale)
    gu.check(o, lse, o_ref, lse_ref, "decode Sk=%d" % Sk)
