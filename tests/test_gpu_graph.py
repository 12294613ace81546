"""The library's launches under HIP graph capture: a decode step and a forward + backward are
captured once and replayed several times, with eager work and synchronisations between the
replays; every replay must reproduce the eager result bit for bit.  (The calls enqueue kernels only:
no allocation, no memset, no synchronisation inside the library.)"""

import numpy as np
import pytest
import torch

from paper_2407_17678_amd import binding as B
from paper_2407_17678_amd import synth

pytestmark = pytest.mark.gpu


def _rand(shape, seed):
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    return torch.randn(shape, device="cuda", generator=gen).to(torch.bfloat16)


def test_decode_step_in_a_graph():
    w = synth.WORKLOADS["7b_decode"]
    nseq, H, D, S, max_len = 8, 8, w.head_dim, w.block_size, 4096
    params = B.layout_params(H, 1, S, w.local_blocks, w.stride, 0, w.window_blocks, 0)
    q = _rand((nseq, H, D), 1)
    kc, vc = _rand((nseq, H, max_len, D), 2), _rand((nseq, H, max_len, D), 3)
    lens = torch.tensor([1, 64, 65, 1000, 2048, 4095, 4096, 3000], dtype=torch.int32, device="cuda")
    o = torch.empty_like(q)
    lse = torch.empty((nseq, H), dtype=torch.float32, device="cuda")
    splits = 4
    ws = torch.empty(B.s2_attn_decode_workspace_bytes(nseq, H, D, max_len, splits), dtype=torch.uint8, device="cuda")
    step = lambda: B.s2_attn_decode(params, q, kc, vc, lens, o, lse, w.scale, ws, max_len, num_splits=splits)
    step()
    torch.cuda.synchronize()
    want_o, want_lse = o.clone(), lse.clone()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        o.zero_()
        lse.zero_()
        ws.random_(0, 255)                       # eager work between replays; partials are overwritten
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o, want_o) and torch.equal(lse, want_lse), rep
    # new inputs in the same buffers: the replay follows them
    q.copy_(_rand((nseq, H, D), 9))
    lens.copy_(torch.tensor([7, 100, 640, 4096, 1, 333, 2049, 64], dtype=torch.int32, device="cuda"))
    step()
    torch.cuda.synchronize()
    want_o, want_lse = o.clone(), lse.clone()
    o.zero_()
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(o, want_o) and torch.equal(lse, want_lse)


@pytest.mark.parametrize("keep_ds", [False, True])
def test_forward_backward_in_a_graph(keep_ds):
    """Both forms of the backward: the small workspace, and the one that holds dS between the launches."""
    w = synth.WORKLOADS["1p3b_8k"]
    Bt, H, N, D, S = 1, 4, 2048, w.head_dim, w.block_size
    lay = B.s2_layout_build(B.layout_params(H, N // S, S, w.local_blocks, w.stride))
    q, k, v, g = (_rand((Bt, H, N, D), 20 + i) for i in range(4))
    o = torch.empty_like(q)
    lse = torch.empty((Bt, H, N), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    nbytes = B.s2_attn_bwd_layout_workspace_bytes(lay, Bt, H, N, D) if keep_ds else B.s2_attn_bwd_workspace_bytes(Bt, H, N, D)
    assert not keep_ds or nbytes > B.s2_attn_bwd_workspace_bytes(Bt, H, N, D)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")

    def step():
        B.s2_attn_fwd(lay, q, k, v, o, lse, w.scale)
        B.s2_attn_bwd(lay, q, k, v, o, lse, g, dq, dk, dv, w.scale, ws)

    step()   # also sets the kernels' dynamic LDS limits, which is not a stream operation
    torch.cuda.synchronize()
    want = [t.clone() for t in (o, lse, dq, dk, dv)]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for t in (o, lse, dq, dk, dv):
            t.zero_()
        ws.random_(0, 255)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, ref in zip((o, lse, dq, dk, dv), want):
            assert torch.equal(t, ref), rep
