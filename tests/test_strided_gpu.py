"""GPU parity of the strided / any-head-dimension entry point (through the C ABI) against the fp64 oracle."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2604_14825_amd import binding as nb
from paper_2604_14825_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu


def make(B, Hq, Hkv, S, D, idt, seed):
    q = synth.fill(B, Hq, S, D, seed, synth.TAG_Q, idt)
    k = synth.fill(B, Hkv, S, D, seed, synth.TAG_K, idt, S // 50, 8.0)
    v = synth.fill(B, Hkv, S, D, seed, synth.TAG_V, idt)
    return q, k, v


def run_strided(qd, kd, vd, od, causal, scale, want_lse=True):
    B, Hq, S, D = qd.shape
    lse = torch.full((B, Hq, S), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    nb.naut_attn_fwd_strided(qd, kd, vd, od, lse, causal, scale)
    torch.cuda.synchronize()
    return od.double().cpu().numpy(), (lse.double().cpu().numpy() if want_lse else None)


@pytest.mark.parametrize("variant", ["w8q32", "w4q64", "bm128"])
@pytest.mark.parametrize("D", [8, 32, 40, 64, 80, 96, 112, 128])
def test_head_dimensions(D, variant, monkeypatch):
    """Every multiple of 8 runs on the 64- or 128-wide kernels; contiguous layout."""
    monkeypatch.setenv("NAUT_ATTN_VARIANT", variant)
    B, Hq, Hkv, S, causal, idt, odt = 1, 4, 2, 333, True, synth.BF16, synth.F32
    q, k, v = make(B, Hq, Hkv, S, D, idt, 9000 + D)
    scale = 1.0 / math.sqrt(D)
    print("head dim", D, variant, flush=True)
    qd, kd, vd = (gu.to_device(a, idt) for a in (q, k, v))
    od = torch.full((B, Hq, S, D), float("nan"), dtype=gu.TORCH_DT[odt], device="cuda")
    o, lse = run_strided(qd, kd, vd, od, causal, scale)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, causal, scale)
    gu.check(o, lse, o_ref, lse_ref, "D=%d %s" % (D, variant))


@pytest.mark.parametrize("variant", ["w8q32", "w4q64", "bm128"])
@pytest.mark.parametrize("D,causal,idt,odt", [(128, True, synth.BF16, synth.BF16), (64, False, synth.F16, synth.F16),
                                             (96, True, synth.BF16, synth.BF16)])
def test_bshd_layout(D, causal, idt, odt, variant, monkeypatch):
    """Tensors stored [B][S][H][D] (sequence-major), passed as transposed views; O written in the same layout."""
    monkeypatch.setenv("NAUT_ATTN_VARIANT", variant)
    B, Hq, Hkv, S = 2, 6, 2, 300
    q, k, v = make(B, Hq, Hkv, S, D, idt, 9100 + D)
    scale = 1.0 / math.sqrt(D)
    bshd = lambda a: gu.to_device(np.ascontiguousarray(a.transpose(0, 2, 1, 3)), idt)   # memory [B][S][H][D]
    qd, kd, vd = bshd(q).transpose(1, 2), bshd(k).transpose(1, 2), bshd(v).transpose(1, 2)  # logical [B,H,S,D]
    assert not qd.is_contiguous()
    o_mem = torch.full((B, S, Hq, D), float("nan"), dtype=gu.TORCH_DT[odt], device="cuda")
    print("bshd", D, variant, flush=True)
    o, lse = run_strided(qd, kd, vd, o_mem.transpose(1, 2), causal, scale)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, causal, scale)
    gu.check(o, lse, o_ref, lse_ref, "bshd D=%d %s" % (D, variant))


def test_padded_rows_and_untouched_gaps():
    """Rows padded to a wider pitch (D = 80 in rows of 128): nothing is read as data from the gaps (they hold
    NaN patterns) and nothing is written into the gaps of O."""
    B, Hq, Hkv, S, D, P = 1, 2, 1, 260, 80, 128
    idt = synth.BF16
    q, k, v = make(B, Hq, Hkv, S, D, idt, 9200)
    scale = 1.0 / math.sqrt(D)

    def padded(a):
        H = a.shape[1]
        buf = np.full((B, H, S, P), 0x7FC0, dtype=np.uint16)  # bf16 NaN in the gaps
        buf[..., :D] = a
        return gu.to_device(buf, idt)[..., :D]
    qd, kd, vd = padded(q), padded(k), padded(v)
    o_buf = torch.full((B, Hq, S, P), 7.0, dtype=torch.float32, device="cuda")
    o, lse = run_strided(qd, kd, vd, o_buf[..., :D], True, scale)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, True, scale)
    gu.check(o, lse, o_ref, lse_ref, "padded rows")
    assert torch.all(o_buf[..., D:] == 7.0).item(), "the gaps between O rows were written"


@pytest.mark.parametrize("variant", ["w8q32", "w4q64", "bm128"])
@pytest.mark.parametrize("D,odt", [(128, synth.BF16), (64, synth.F16), (80, synth.BF16)])
def test_o_rows_aligned_to_8_bytes_only(D, odt, variant, monkeypatch):
    """16-bit O with a row pitch of D + 4 elements: rows start on 8-byte, not 16-byte, boundaries (the least the
    entry point accepts), the S = 333 rows end in a ragged tile, and the 4-element gaps must stay untouched.
    The pipelined kernels write O in 16-byte pieces of whole rows, so this is their unaligned-store case."""
    monkeypatch.setenv("NAUT_ATTN_VARIANT", variant)
    B, Hq, Hkv, S = 2, 4, 2, 333
    idt = odt
    q, k, v = make(B, Hq, Hkv, S, D, idt, 9300 + D)
    scale = 1.0 / math.sqrt(D)
    qd, kd, vd = (gu.to_device(a, idt) for a in (q, k, v))
    o_buf = torch.full((B, Hq, S, D + 4), 7.0, dtype=gu.TORCH_DT[odt], device="cuda")
    print("8-byte O rows", D, variant, flush=True)
    o, lse = run_strided(qd, kd, vd, o_buf[..., :D], True, scale)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, True, scale)
    gu.check(o, lse, o_ref, lse_ref, "8-byte O rows D=%d %s" % (D, variant))
    assert torch.all(o_buf[..., D:] == 7.0).item(), "the gaps between O rows were written"


@pytest.mark.parametrize("D,odt", [(256, synth.BF16), (200, synth.F16), (136, synth.BF16)])
def test_o_rows_aligned_to_8_bytes_only_wide(D, odt):
    """The same on the 256-wide kernel (two O rows per store instruction, 25 or 17 of the 32 chunks real at
    D = 200 and 136)."""
    B, Hq, Hkv, S = 1, 4, 2, 333
    idt = odt
    q, k, v = make(B, Hq, Hkv, S, D, idt, 9400 + D)
    scale = 1.0 / math.sqrt(D)
    qd, kd, vd = (gu.to_device(a, idt) for a in (q, k, v))
    o_buf = torch.full((B, Hq, S, D + 4), 7.0, dtype=gu.TORCH_DT[odt], device="cuda")
    print("8-byte O rows, wide kernel", D, flush=True)
    o, lse = run_strided(qd, kd, vd, o_buf[..., :D], True, scale)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, True, scale)
    gu.check(o, lse, o_ref, lse_ref, "8-byte O rows D=%d" % D)
    assert torch.all(o_buf[..., D:] == 7.0).item(), "the gaps between O rows were written"


def test_broadcast_kv_over_batch():
    """Stride 0 on the batch axis of K and V: one cache shared by every batch entry."""
    B, Hq, Hkv, S, D = 3, 4, 4, 200, 64
    idt = synth.BF16
    q, k, v = make(B, Hq, Hkv, S, D, idt, 9300)
    k[1:], v[1:] = k[0], v[0]
    scale = 1.0 / math.sqrt(D)
    qd = gu.to_device(q, idt)
    kd = gu.to_device(k[:1], idt).expand(B, Hkv, S, D)
    vd = gu.to_device(v[:1], idt).expand(B, Hkv, S, D)
    assert kd.stride(0) == 0
    od = torch.full((B, Hq, S, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    o, lse = run_strided(qd, kd, vd, od, False, scale)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, False, scale)
    gu.check(o, lse, o_ref, lse_ref, "broadcast kv")


def test_bshd_prefill_size_sampled_rows():
    """The prefill workload's shape in sequence-major layout, on the default variant, sampled rows."""
    w = synth.WORKLOADS["prefill"]
    q, k, v = synth.make_inputs(w)
    bshd = lambda a: gu.to_device(np.ascontiguousarray(a.transpose(0, 2, 1, 3)), w.in_dtype)
    qd, kd, vd = bshd(q).transpose(1, 2), bshd(k).transpose(1, 2), bshd(v).transpose(1, 2)
    o_mem = torch.full((w.B, w.S, w.Hq, w.D), float("nan"), dtype=torch.bfloat16, device="cuda")
    o, lse = run_strided(qd, kd, vd, o_mem.transpose(1, 2), w.causal, w.scale)
    rows = gu.sample_rows(w, 1500, 77)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, w.in_dtype, w.causal, w.scale, rows=rows)
    gu.check(o.reshape(-1, w.D)[rows], lse.reshape(-1)[rows], o_ref, lse_ref, "bshd prefill")


@pytest.mark.parametrize("D,S,causal,idt,odt", [
    (256, 333, True, synth.BF16, synth.F32),
    (256, 500, False, synth.F16, synth.F16),
    (136, 260, True, synth.BF16, synth.BF16),
    (160, 129, False, synth.BF16, synth.F32),
    (192, 1000, True, synth.F16, synth.F32),
    (248, 97, True, synth.BF16, synth.BF16),
    (256, 1, True, synth.BF16, synth.F32),
])
def test_wide_head_dimensions(D, S, causal, idt, odt):
    """Head dimensions above 128 run on the 256-wide instantiation of the 128-query kernel (32 keys per step)."""
    B, Hq, Hkv = 2, 4, 2
    q, k, v = make(B, Hq, Hkv, S, D, idt, 9400 + D + S)
    scale = 1.0 / math.sqrt(D)
    print("wide head dim", D, S, flush=True)
    qd, kd, vd = (gu.to_device(a, idt) for a in (q, k, v))
    od = torch.full((B, Hq, S, D), float("nan"), dtype=gu.TORCH_DT[odt], device="cuda")
    o, lse = run_strided(qd, kd, vd, od, causal, scale)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, causal, scale)
    gu.check(o, lse, o_ref, lse_ref, "D=%d S=%d" % (D, S))


def test_wide_head_bshd_long_sampled_rows():
    """D = 256 at a prefill-sized sequence in sequence-major layout: many key steps, sampled rows."""
    B, Hq, Hkv, S, D, idt = 1, 8, 2, 4096, 256, synth.BF16
    q, k, v = make(B, Hq, Hkv, S, D, idt, 9500)
    scale = 1.0 / math.sqrt(D)
    bshd = lambda a: gu.to_device(np.ascontiguousarray(a.transpose(0, 2, 1, 3)), idt)
    qd, kd, vd = bshd(q).transpose(1, 2), bshd(k).transpose(1, 2), bshd(v).transpose(1, 2)
    o_mem = torch.full((B, S, Hq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    o, lse = run_strided(qd, kd, vd, o_mem.transpose(1, 2), True, scale)
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([rng.integers(0, B * Hq * S, 600), [0, S - 1, B * Hq * S - 1]]))
    o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, True, scale, rows=rows)
    gu.check(o.reshape(-1, D)[rows], lse.reshape(-1)[rows], o_ref, lse_ref, "bshd D=256")


def test_wide_head_24_heads_groups_of_two():
    """D = 256 with B*Hq = 24: every XCD gets three heads and works on two at a time, so its last group is
    smaller than the others (the multi-group branch of the 128-query kernel's tile scheduler)."""
    B, Hq, Hkv, S, D, idt = 3, 8, 4, 1024, 256, synth.BF16
    q, k, v = make(B, Hq, Hkv, S, D, idt, 9600)
    scale = 1.0 / math.sqrt(D)
    qd, kd, vd = (gu.to_device(a, idt) for a in (q, k, v))
    od = torch.full((B, Hq, S, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    print("wide head, 24 heads", flush=True)
    o, lse = run_strided(qd, kd, vd, od, True, scale)
    assert np.isfinite(o).all(), "an output tile was never written"
    rng = np.random.default_rng(6)
    rows = np.unique(np.concatenate([rng.integers(0, B * Hq * S, 3000),
                                     [bh * S + i for bh in range(B * Hq) for i in (0, 127, 128, S - 1)]]))
    o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, True, scale, rows=rows)
    gu.check(o.reshape(-1, D)[rows], lse.reshape(-1)[rows], o_ref, lse_ref, "D=256, 24 heads")


@pytest.mark.parametrize("D,variant", [(256, None), (128, "bm128"), (128, "w8q32"), (128, "w4q64"), (64, "bm128")])
def test_wide_head_row_stride_beyond_32_bits(D, variant, monkeypatch):
    """K and V rows 16 MiB apart (the largest row stride the entry point admits), on every kernel: S times the
    stride passes 2^32 bytes, so the tile addresses must be formed in 64 bits, and 63 rows of it must fit the
    32-bit offsets inside a tile."""
    if variant is not None:
        monkeypatch.setenv("NAUT_ATTN_VARIANT", variant)
    B, H, S, idt = 1, 1, 300, synth.BF16
    stride = 1 << 23  # elements
    q, k, v = make(B, H, H, S, D, idt, 9700)
    scale = 1.0 / math.sqrt(D)
    qd = gu.to_device(q, idt)

    def spread(a):
        buf = torch.empty(S * stride, dtype=torch.bfloat16, device="cuda")  # 4.7 GiB, rows at the start of each pitch
        rows = buf.view(S, stride)[:, :D]
        rows.copy_(gu.to_device(a, idt)[0, 0])
        return rows.unsqueeze(0).unsqueeze(0)  # logical [1,1,S,D]
    kd, vd = spread(k), spread(v)
    assert kd.stride(2) == stride and kd.stride(2) * 2 * S > 1 << 32
    od = torch.full((B, H, S, D), float("nan"), dtype=torch.float32, device="cuda")
    print("16 MiB row stride", D, variant, flush=True)
    o, lse = run_strided(qd, kd, vd, od, True, scale)
    o_ref, lse_ref = oracle.attn_rows(q, k, v, idt, True, scale)
    gu.check(o, lse, o_ref, lse_ref, "D=%d %s, row stride 2^23" % (D, variant))
