"""naut_attn_decode_static (no workspace argument, static device scratch) against naut_attn_decode on the same
inputs: bit-identical O and LSE, both within the parity bar of the oracle; two calls in a row, the second
with a smaller input, so that what the first call left in the shared scratch is seen to do no harm."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2604_14825_amd import binding as nb
from paper_2604_14825_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu


def _both(B, Hq, Hkv, Sq, Sk, D, seed):
    q = synth.fill(B, Hq, Sq, D, seed, synth.TAG_Q, synth.BF16)
    k = synth.fill(B, Hkv, Sk, D, seed, synth.TAG_K, synth.BF16, Sk // 100, 8.0)
    v = synth.fill(B, Hkv, Sk, D, seed, synth.TAG_V, synth.BF16)
    scale = 1.0 / math.sqrt(D)
    qd, kd, vd = (gu.to_device(a, synth.BF16) for a in (q, k, v))
    outs = []
    for static in (True, False):
        o = torch.full((B, Hq, Sq, D), float("nan"), dtype=torch.bfloat16, device="cuda")
        lse = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device="cuda")
        print("no-alloc case", B, Hq, Hkv, Sq, Sk, D, "static" if static else "workspace", flush=True)
        if static:
            nb.naut_attn_decode_static(qd, kd, vd, o, lse, True, scale)
        else:
            ws = torch.empty(nb.decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D), dtype=torch.uint8, device="cuda")
            ws.fill_(0xFF)
            nb.naut_attn_decode(qd, kd, vd, o, lse, True, scale, ws)
        torch.cuda.synchronize()
        outs.append((o.view(torch.int16).cpu().numpy(), lse.cpu().numpy(), o.double().cpu().numpy()))
    (o_s, lse_s, of_s), (o_w, lse_w, _) = outs
    assert np.array_equal(o_s, o_w), "O of the static-scratch entry point differs from naut_attn_decode"
    assert np.array_equal(lse_s.view(np.int32), lse_w.view(np.int32)), "LSE differs"
    o_ref, lse_ref = oracle.attn_cross16(q, k, v, synth.BF16, True, scale)
    gu.check(of_s, lse_s.astype(np.float64), o_ref, lse_ref, "decode_static")


def test_static_scratch_two_calls_second_smaller():
    _both(2, 32, 8, 2, 8192, 128, 9100)   # many splits: several MiB of partials
    _both(1, 8, 2, 1, 700, 64, 9101)      # smaller in every size; most of the scratch keeps the first call's partials


def test_static_scratch_rejects_oversize():
    """Partials beyond the 16 MiB scratch: a clear error, nothing launched."""
    B, Hq, Hkv, Sq, Sk, D = 64, 64, 64, 1, 4096, 128
    assert nb.decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D) > 16 << 20
    z = torch.zeros(16, dtype=torch.uint8, device="cuda")
    rc = nb.naut_attn_decode_static_raw(z.data_ptr(), z.data_ptr(), z.data_ptr(), z.data_ptr(), None, B, Hq, Hkv, Sq, Sk,
                                        D, True, 0.1, None)
    assert rc == nb.NAUT_ERR_UNSUPPORTED
    assert "static scratch" in nb.last_error_string()
