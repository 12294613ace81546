"""The hand-scheduled forward and dQ kernels (head_dim 128, mask blocks of 64 or 128 tokens, whole
128-row tiles) against the fp64 oracle on shapes picked to reach their corners: head counts that do
not fill the eight XCDs evenly, one-tile sequences, windows shorter than a tile, mask rows of a
tile that keep almost disjoint blocks (a wavefront idle for many steps in a row, then active
again), strided tensors, the dense instantiation, and repeatability bit for bit."""

import dataclasses

import numpy as np
import pytest
import torch

from oracle import s2_oracle as orc
from paper_2407_17678_amd import binding as B
from paper_2407_17678_amd import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

LSE_TOL, GRAD_TOL = 1e-3, 2e-2
W = synth.WORKLOADS["1p3b_8k"]   # head_dim 128, scale 1/sqrt(128)


def _check_all(bits, M, S, scale, o, lse, dq, dk, dv):
    qb, kb, vb, gb = bits
    dQ, dK, dV, O, LSE = orc.attention_backward(G.bits_f64(qb), G.bits_f64(kb), G.bits_f64(vb), G.bits_f64(gb), M, S, scale)
    assert G.o_excess(G.to_f64(o), O) <= 0
    assert np.abs(G.to_f64(lse) - LSE).max() <= LSE_TOL
    for n, t, ref in (("dq", dq, dQ), ("dk", dk, dK), ("dv", dv, dV)):
        e = G.rel_l2(G.to_f64(t), ref)
        assert e <= GRAD_TOL, (n, e)


def _run(lay, q, k, v, g, scale):
    Bt, H, N, D = q.shape
    o = torch.empty((Bt, H, N, D), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty((Bt, H, N), dtype=torch.float32, device="cuda")
    dq, dk, dv = (torch.empty((Bt, H, N, D), dtype=torch.bfloat16, device="cuda") for _ in range(3))
    ws = torch.full((B.s2_attn_bwd_workspace_bytes(Bt, H, N, D),), 0xFF, dtype=torch.uint8, device="cuda")
    B.s2_attn_fwd(lay, q, k, v, o, lse, scale)
    B.s2_attn_bwd(lay, q, k, v, o, lse, g, dq, dk, dv, scale, ws)
    torch.cuda.synchronize()
    return o, lse, dq, dk, dv


CASES = [
    # S, heads, batch, blocks, local, stride, base, window
    (64, 1, 1, 2, 1, 0, 0, 0),      # one tile, diagonal blocks only
    (64, 3, 2, 2, 4, 1, 0, 0),      # one tile, window longer than the sequence
    (64, 9, 1, 6, 1, 2, 3, 0),      # nine heads: the ninth alone on its XCD slot; one local block
    (64, 5, 1, 10, 2, 3, 1, 0),
    (64, 2, 3, 16, 4, 8, 0, 0),     # the 1.3B rule
    (64, 4, 1, 24, 16, 16, 5, 0),   # the 7B rule, stripes not yet reached by most rows
    (64, 2, 1, 12, 3, 5, 0, 7),     # a stripe window
    (128, 1, 1, 1, 1, 0, 0, 0),     # a single 128-token block
    (128, 7, 1, 5, 2, 2, 0, 0),
    (128, 3, 2, 8, 8, 32, 4, 0),    # the 128K rule cut short
    (128, 2, 1, 9, 1, 3, 1, 4),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "S%d_H%d_b%d_B%d_L%d_V%d_o%d_w%d" % c)
def test_rule_patterns(case):
    S, H, batch, Bk, B_l, stride, base, window = case
    print("fast-path case", case, flush=True)
    N = Bk * S
    assert N % 128 == 0
    bits = synth.train_inputs(W, heads=H, batch=batch, seqlen=N)
    lay = B.s2_layout_build(B.layout_params(H, Bk, S, B_l, stride, base, window, 0))
    M = orc.block_mask(H, Bk, B_l, stride, base, window)
    out = _run(lay, *(G.to_dev(x) for x in bits), W.scale)
    _check_all(bits, M, S, W.scale, *out)


def _csr(M):
    row_ptr, col_idx, _, _ = orc.compressed_layout(M)
    return row_ptr, col_idx


def test_mask_rows_of_a_tile_that_share_little():
    # 64-token blocks: the two mask rows of a 128-row tile keep almost disjoint blocks (even rows the
    # even columns, odd rows the odd ones, plus each row's diagonal), so each half of the workgroup
    # idles through the other's blocks: runs of steps that are not a wavefront's, then its own again
    H, Bk, S = 2, 12, 64
    M = np.zeros((H, Bk, Bk), dtype=bool)
    for i in range(Bk):
        for j in range(i + 1):
            M[0, i, j] = (i == j) or (j % 2 == i % 2)
            M[1, i, j] = (i == j) or (j % 3 == 0 and i % 2 == 0) or (j == i - 1 and i % 2 == 1)
    assert orc.valid_custom_mask(M)
    bits = synth.train_inputs(W, heads=H, batch=2, seqlen=Bk * S)
    lay = B.s2_layout_from_csr(H, Bk, S, *_csr(M))
    out = _run(lay, *(G.to_dev(x) for x in bits), W.scale)
    _check_all(bits, M, S, W.scale, *out)


def test_random_patterns():
    rng = np.random.default_rng(5)
    for S, Bk, H in ((64, 10, 3), (128, 6, 2), (64, 4, 1)):
        M = np.tril(rng.random((H, Bk, Bk)) < 0.35)
        i = np.arange(Bk)
        M[:, i, i] = True
        bits = synth.train_inputs(W, heads=H, batch=1, seqlen=Bk * S)
        lay = B.s2_layout_from_csr(H, Bk, S, *_csr(M))
        out = _run(lay, *(G.to_dev(x) for x in bits), W.scale)
        _check_all(bits, M, S, W.scale, *out)


def test_strided_tensors():
    # q, k, v, dO and the outputs are slices of wider tensors: token stride 192, head and batch strides to match
    H, Bk, S, batch = 3, 8, 64, 2
    N, D, Dw = Bk * S, 128, 192
    bits = synth.train_inputs(W, heads=H, batch=batch, seqlen=N)
    wide = [torch.zeros((batch, H, N, Dw), dtype=torch.bfloat16, device="cuda") for _ in range(4)]
    views = []
    for t, x in zip(wide, bits):
        t[..., 32:32 + D] = G.to_dev(x)
        views.append(t[..., 32:32 + D])
    q, k, v, g = views
    outs = [torch.zeros((batch, H, N, Dw), dtype=torch.bfloat16, device="cuda") for _ in range(4)]
    o, dq, dk, dv = (t[..., 16:16 + D] for t in outs)
    lse = torch.empty((batch, H, N), dtype=torch.float32, device="cuda")
    ws = torch.empty(B.s2_attn_bwd_workspace_bytes(batch, H, N, D), dtype=torch.uint8, device="cuda")
    lay = B.s2_layout_build(B.layout_params(H, Bk, S, 2, 3))
    B.s2_attn_fwd(lay, q, k, v, o, lse, W.scale)
    B.s2_attn_bwd(lay, q, k, v, o, lse, g, dq, dk, dv, W.scale, ws)
    torch.cuda.synchronize()
    M = orc.block_mask(H, Bk, 2, 3)
    _check_all(bits, M, S, W.scale, o.contiguous(), lse, dq.contiguous(), dk.contiguous(), dv.contiguous())
    for t in outs:   # nothing written outside the 128 features of the outputs
        assert float(t[..., :16].abs().max()) == 0 and float(t[..., 16 + D:].abs().max()) == 0


def test_dense_instantiation_and_repeatability():
    H, N, batch = 5, 640, 1
    bits = synth.train_inputs(W, heads=H, batch=batch, seqlen=N)
    q, k, v, g = (G.to_dev(x) for x in bits)
    o = torch.empty_like(q)
    lse = torch.empty((batch, H, N), dtype=torch.float32, device="cuda")
    d = [torch.empty_like(q) for _ in range(3)]
    ws = torch.empty(B.s2_attn_bwd_workspace_bytes(batch, H, N, 128), dtype=torch.uint8, device="cuda")
    B.s2_dense_causal_fwd(q, k, v, o, lse, W.scale)
    B.s2_dense_causal_bwd(q, k, v, o, lse, g, d[0], d[1], d[2], W.scale, ws)
    torch.cuda.synchronize()
    M = orc.block_mask(H, N // 64, 1, 0, dense=True)
    _check_all(bits, M, 64, W.scale, o, lse, *d)
    # a second run of the sparse path gives the same bits (no atomics, fixed order of accumulation)
    lay = B.s2_layout_build(B.layout_params(H, N // 64, 64, 2, 4))
    a = _run(lay, q, k, v, g, W.scale)
    b = _run(lay, q, k, v, g, W.scale)
    for x, y in zip(a, b):
        assert torch.equal(x, y)
