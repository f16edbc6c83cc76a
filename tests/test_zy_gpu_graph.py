"""The whole step (mask, forward, backward) captured into a HIP graph and replayed: the library
allocates nothing, clears nothing with memset nodes and keeps no state, so a captured step must
reproduce the eager results bit for bit on every replay, also after the inputs have changed."""

import numpy as np
import pytest
import torch

from paper_2508_10774_amd import binding, synth
from tests import util

pytestmark = pytest.mark.gpu


def test_captured_step_replays_bit_identically():
    w = synth.Workload("graph", 1, 2, 128, (4, 12, 20), 0, 128, 16)      # L = 960, ragged last block
    p = binding.Params(B=w.B, H=w.H, L=w.L, d=w.d, block=w.block, k_samples=w.k_samples, tau=0.9)
    inputs = []
    for seed in (1, 2, 3):
        qb, kb, vb = synth.make_qkv(w, seed)
        inputs.append([util.dev_bf16(x) for x in (qb, kb, vb, synth.make_do(w, seed))])
    q, k, v, g = (torch.empty_like(t) for t in inputs[0])
    bufs = binding.alloc_index_lists(p)
    ws_m = binding.alloc_workspace(binding.asa_mask_workspace_bytes(p))
    ws_f = binding.alloc_workspace(binding.asa_fwd_workspace_bytes(p))
    ws_b = binding.alloc_workspace(binding.asa_bwd_workspace_bytes(p))
    o, o_lo = torch.empty_like(q), torch.empty_like(q)
    lse = torch.empty((p.B * p.H, p.L), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)

    def step():
        binding.asa_build_mask(p, q, k, bufs["mask"], bufs["row_ptr"], bufs["col_idx"], bufs["col_ptr"],
                               bufs["row_idx"], None, ws_m)
        binding.asa_attn_fwd(p, q, k, v, bufs["row_ptr"], bufs["col_idx"], o, lse, ws_f, o_lo=o_lo)
        binding.asa_attn_bwd(p, q, k, v, o, g, lse, bufs["row_ptr"], bufs["col_idx"], bufs["col_ptr"],
                             bufs["row_idx"], dq, dk, dv, ws_b, o_lo=o_lo)

    def load(i):
        for dst, src in zip((q, k, v, g), inputs[i]):
            dst.copy_(src)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (bufs["mask"], bufs["row_ptr"], o, lse, dq, dk, dv)]

    eager = []
    for i in range(3):
        load(i)
        step()
        eager.append(snapshot())
    assert not torch.equal(eager[0][2], eager[1][2])         # the inputs really differ

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    load(0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(2):
        for i in (2, 0, 1):
            load(i)
            for t in (o, dq, dk, dv):
                t.fill_(float("nan"))                        # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            got = snapshot()
            for a, b, what in zip(got, eager[i], ("mask", "row_ptr", "O", "LSE", "dQ", "dK", "dV")):
                assert torch.equal(a.view(torch.uint8) if a.dtype == torch.bfloat16 else a,
                                   b.view(torch.uint8) if b.dtype == torch.bfloat16 else b), (rep, i, what)
