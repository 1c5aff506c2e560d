"""The entry points enqueue kernels and nothing else (no allocation, no memset, no synchronisation), so a
caller may record them into a HIP graph.  One graph holds a prefill launch, a strided launch and a decode
launch (two kernels and a caller-provided workspace); it is replayed several times on fresh inputs, with eager
work and synchronisations in between, and every replay is compared with the eager result of the same inputs
and, once, with the fp64 oracle."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2604_14825_amd import binding as nb
from paper_2604_14825_amd import synth

import gpu_util as gu

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager():
    idt = synth.BF16
    B, Hq, Hkv, S, D = 2, 4, 2, 700, 128
    Sq, Sk = 2, 1500
    scale = 1.0 / math.sqrt(D)

    def inputs(seed):
        q = synth.fill(B, Hq, S, D, seed, synth.TAG_Q, idt)
        k = synth.fill(B, Hkv, S, D, seed, synth.TAG_K, idt, S // 50, 8.0)
        v = synth.fill(B, Hkv, S, D, seed, synth.TAG_V, idt)
        qd = synth.fill(B, Hq, Sq, D, seed + 1, synth.TAG_Q, idt)
        kd = synth.fill(B, Hkv, Sk, D, seed + 1, synth.TAG_K, idt)
        vd = synth.fill(B, Hkv, Sk, D, seed + 1, synth.TAG_V, idt)
        return [q, k, v, qd, kd, vd]

    host = inputs(100)
    bufs = [gu.to_device(a, idt) for a in host]             # static input buffers of the graph
    q, k, v, qd, kd, vd = bufs
    o = torch.zeros((B, Hq, S, D), dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros((B, Hq, S), dtype=torch.float32, device="cuda")
    o_s = torch.zeros((B, S, Hq, D), dtype=torch.float32, device="cuda")   # sequence-major output of the strided call
    od = torch.zeros((B, Hq, Sq, D), dtype=torch.bfloat16, device="cuda")
    lsed = torch.zeros((B, Hq, Sq), dtype=torch.float32, device="cuda")
    ws = torch.empty(nb.decode_workspace_bytes(B, Hq, Hkv, Sq, Sk, D), dtype=torch.uint8, device="cuda")

    def enqueue():
        nb.naut_attn_fwd(q, k, v, o, lse, True, scale)
        nb.naut_attn_fwd_strided(q, k, v, o_s.transpose(1, 2), None, False, scale)
        nb.naut_attn_decode(qd, kd, vd, od, lsed, True, scale, ws)

    outs = (o, lse, o_s, od, lsed)
    snapshot = lambda: [t.clone() for t in outs]

    enqueue()                                                  # eager: warm-up and the first expectation
    torch.cuda.synchronize()
    want = snapshot()
    o_ref, lse_ref = oracle.attn_rows(host[0], host[1], host[2], idt, True, scale)
    gu.check(want[0].double().cpu().numpy(), want[1].double().cpu().numpy(), o_ref, lse_ref, "eager prefill")

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            enqueue()
    torch.cuda.synchronize()

    for rep, seed in enumerate((100, 200, 300, 200)):
        print("graph replay", rep, "seed", seed, flush=True)
        host = inputs(seed)
        for dst, src in zip(bufs, host):
            dst.copy_(gu.to_device(src, idt))
        for t in outs:
            t.fill_(7.0)                                      # a replay must rewrite every output
        ws.fill_(0xFF)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = snapshot()
        for t in outs:
            t.fill_(7.0)
        ws.fill_(0xFF)
        enqueue()                                              # eager on the same inputs
        torch.cuda.synchronize()
        for a, b_, name in zip(got, outs, ("o", "lse", "o strided", "o decode", "lse decode")):
            assert torch.equal(a, b_), "replay %d: %s differs from the eager result" % (rep, name)
