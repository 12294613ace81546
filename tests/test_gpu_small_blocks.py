"""GPU parity with 32- and 16-token mask blocks (section 3.2: fine-grained shards inside a large
query tile): forward, backward, decode, paged decode and a caller-supplied pattern, all against the
fp64 oracle run with the same block size."""

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


def _small(name, S, local_blocks, stride):
    return dataclasses.replace(synth.WORKLOADS[name], block_size=S, local_blocks=local_blocks, stride=stride)


@pytest.mark.parametrize("S", [32, 16])
@pytest.mark.parametrize("name,heads,batch,seqlen,B_l,s", [
    ("1p3b_8k", 4, 2, 1024, 4, 8),     # D=128
    ("7b_32k", 3, 1, 2048, 9, 16),     # longer rows, more stripes than heads
    ("tiny", 4, 1, 640, 3, 4),         # D=64, five 128-row tiles
    ("1p3b_8k", 2, 1, 128, 1, 0),      # one tile, diagonal blocks only
    ("1p3b_8k", 5, 1, 768, 1, 3),      # odd stride: stripes fall on either block of a 32-token unit
    ("tiny", 3, 1, 512, 2, 5),
])
def test_small_blocks_fwd_bwd(name, heads, batch, seqlen, B_l, s, S):
    w = _small(name, S, B_l, s)
    qb, kb, vb, gb = synth.train_inputs(w, heads=heads, batch=batch, seqlen=seqlen)
    print("small-block case", name, qb.shape, "S", S, "B_l", B_l, "stride", s, flush=True)
    out = G.run_fwd_bwd(w, qb, kb, vb, gb)
    M = G.oracle_mask(w, heads, seqlen)
    assert M.shape[1] == seqlen // S
    dQ, dK, dV, O, LSE = orc.attention_backward(G.bits_f64(qb), G.bits_f64(kb), G.bits_f64(vb), G.bits_f64(gb),
                                                M, S, w.scale)
    assert G.o_excess(G.to_f64(out["o"]), O) <= 0
    assert np.abs(G.to_f64(out["lse"]) - LSE).max() <= LSE_TOL
    for n, ref in (("dq", dQ), ("dk", dK), ("dv", dV)):
        assert G.rel_l2(G.to_f64(out[n]), ref) <= GRAD_TOL, n


@pytest.mark.parametrize("S,B_l,s", [(32, 2, 4), (16, 2, 4), (16, 1, 3), (16, 3, 7)])
def test_small_blocks_zero_queries_count_keys(S, B_l, s):
    # Q = 0: LSE = ln(#kept keys), which checks every row's kept set through the kernel
    w = _small("tiny", S, B_l, s)
    H, N = 4, 512
    qb, kb, vb, _ = synth.train_inputs(w, heads=H, batch=1, seqlen=N)
    qb = np.zeros_like(qb)
    o, lse, lay, _ = G.run_fwd(w, qb, kb, vb)
    M = G.oracle_mask(w, H, N)
    t = np.arange(N)
    want = np.log(float(S) * (M[:, t // S].sum(axis=2) - 1) + (t % S) + 1)
    assert np.abs(G.to_f64(lse)[0] - want).max() <= 1e-5


@pytest.mark.parametrize("S,Bk,density", [(32, 24, 0.35), (16, 48, 0.35), (16, 40, 0.08), (16, 24, 0.9)])
def test_small_blocks_custom_pattern(S, Bk, density):
    # random rows: with 16-token blocks every 2 x 2 keep pattern of a (query pair, key pair) occurs
    rng = np.random.default_rng(8)
    H = 3
    M = np.tril(rng.random((H, Bk, Bk)) < density)
    i = np.arange(Bk)
    M[:, i, i] = True
    w = _small("1p3b_8k", S, 1, 0)
    N = Bk * S
    qb, kb, vb, gb = synth.train_inputs(w, heads=H, batch=1, seqlen=N)
    row_ptr, col_idx, _, _ = orc.compressed_layout(M)
    lay = B.s2_layout_from_csr(H, Bk, S, row_ptr, col_idx)
    q, k, v, g = G.to_dev(qb), G.to_dev(kb), G.to_dev(vb), G.to_dev(gb)
    o = torch.empty_like(q)
    lse = torch.empty((1, H, N), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ws = torch.empty(B.s2_attn_bwd_workspace_bytes(1, H, N, w.head_dim), dtype=torch.uint8, device="cuda")
    B.s2_attn_fwd(lay, q, k, v, o, lse, w.scale)
    B.s2_attn_bwd(lay, q, k, v, o, lse, g, dq, dk, dv, w.scale, ws)
    torch.cuda.synchronize()
    dQ, dK, dV, O, LSE = orc.attention_backward(G.bits_f64(qb), G.bits_f64(kb), G.bits_f64(vb), G.bits_f64(gb),
                                                M, S, w.scale)
    assert G.o_excess(G.to_f64(o), O) <= 0
    assert np.abs(G.to_f64(lse) - LSE).max() <= LSE_TOL
    for n, got, ref in (("dq", dq, dQ), ("dk", dk, dK), ("dv", dv, dV)):
        assert G.rel_l2(G.to_f64(got), ref) <= GRAD_TOL, n


@pytest.mark.parametrize("S", [32, 16])
@pytest.mark.parametrize("paged", [False, True])
def test_small_blocks_decode(paged, S):
    w = _small("7b_decode", S, 5, 8)
    heads, max_len = 6, 1000
    lens = np.array([1, 15, 16, 17, 31, 32, 33, 1000, 777], dtype=np.int32)
    nseq = len(lens)
    qb, kcb, vcb, lens = synth.decode_inputs_small(w, nseq, heads, max_len, lengths=lens)
    params = B.layout_params(heads, 1, S, w.local_blocks, w.stride, 0, w.window_blocks, 0)
    q = G.to_dev(qb)
    sl = torch.from_numpy(lens).cuda()
    o = torch.empty_like(q)
    lse = torch.empty((nseq, heads), dtype=torch.float32, device="cuda")
    max_blocks = -(-max_len // S)
    ws = torch.empty(B.s2_attn_decode_workspace_bytes(nseq, heads, w.head_dim, max_blocks * S, 3),
                     dtype=torch.uint8, device="cuda")
    f = G.bits_f64
    if paged:
        resident = [[orc.resident_blocks(int(L), h, S, w.local_blocks, w.stride) for h in range(heads)] for L in lens]
        table, num_pages = synth.page_table(resident, max_blocks, index=w.index)
        pad = max_blocks * S - max_len
        kcb = np.concatenate([kcb, np.zeros((nseq, heads, pad, w.head_dim), np.uint16)], axis=2)
        vcb = np.concatenate([vcb, np.zeros((nseq, heads, pad, w.head_dim), np.uint16)], axis=2)
        kpool = synth.pages_from_cache(kcb, table, num_pages, S)
        vpool = synth.pages_from_cache(vcb, table, num_pages, S)
        missing = torch.zeros(1, dtype=torch.int32, device="cuda")
        B.s2_attn_decode_paged(params, q, G.to_dev(kpool), G.to_dev(vpool), torch.from_numpy(table).cuda(), sl, o,
                               lse, w.scale, ws, missing=missing, num_splits=3)
        torch.cuda.synchronize()
        assert int(missing.item()) == 0
    else:
        B.s2_attn_decode(params, q, G.to_dev(kcb), G.to_dev(vcb), sl, o, lse, w.scale, ws, max_len, num_splits=3)
        torch.cuda.synchronize()
    for b in range(nseq):
        for h in range(heads):
            if paged:
                ref, ref_lse = orc.paged_decode_row(f(qb)[b, h], f(kpool), f(vpool), table[b, h], int(lens[b]), h, S,
                                                    w.local_blocks, w.stride, w.scale)
            else:
                ref, ref_lse = orc.decode_row(f(qb)[b, h], f(kcb)[b, h], f(vcb)[b, h], int(lens[b]), h, S,
                                              w.local_blocks, w.stride, w.scale)
            assert G.o_excess(G.to_f64(o[b, h]), ref) <= 0, (b, h)
            assert abs(float(lse[b, h]) - ref_lse) <= LSE_TOL, (b, h)


@pytest.mark.parametrize("S,seqlen", [(64, 576), (64, 64), (32, 160), (32, 32), (32, 96), (16, 160), (16, 32),
                                      (16, 96)])
def test_sequences_that_end_inside_a_128_row_tile(S, seqlen):
    # the last tile of queries (and of keys) is partly empty: wavefronts beyond the sequence idle
    w = dataclasses.replace(synth.WORKLOADS["1p3b_8k"], block_size=S, local_blocks=2, stride=3)
    H = 3
    qb, kb, vb, gb = synth.train_inputs(w, heads=H, batch=2, seqlen=seqlen)
    out = G.run_fwd_bwd(w, qb, kb, vb, gb)
    M = G.oracle_mask(w, H, seqlen)
    dQ, dK, dV, O, LSE = orc.attention_backward(G.bits_f64(qb), G.bits_f64(kb), G.bits_f64(vb), G.bits_f64(gb),
                                                M, S, w.scale)
    assert G.o_excess(G.to_f64(out["o"]), O) <= 0
    assert np.abs(G.to_f64(out["lse"]) - LSE).max() <= LSE_TOL
    for n, ref in (("dq", dQ), ("dk", dK), ("dv", dV)):
        assert G.rel_l2(G.to_f64(out[n]), ref) <= GRAD_TOL, n


@pytest.mark.parametrize("S", [32, 16])
def test_all_blocks_kept_with_small_blocks_is_dense_causal_attention(S):
    # a layout that keeps every causal block (dense = 1) walked in small blocks must give plain
    # causal attention, which the library's dense kernel also computes
    w = dataclasses.replace(synth.WORKLOADS["tiny"], block_size=S)
    H, N = 2, 384
    qb, kb, vb, gb = synth.train_inputs(w, heads=H, batch=1, seqlen=N)
    lay = B.s2_layout_build(B.layout_params(H, N // S, S, 1, 0, dense=1))
    q, k, v, g = G.to_dev(qb), G.to_dev(kb), G.to_dev(vb), G.to_dev(gb)
    o = torch.empty_like(q)
    lse = torch.empty((1, H, N), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ws = torch.empty(B.s2_attn_bwd_workspace_bytes(1, H, N, w.head_dim), dtype=torch.uint8, device="cuda")
    B.s2_attn_fwd(lay, q, k, v, o, lse, w.scale)
    B.s2_attn_bwd(lay, q, k, v, o, lse, g, dq, dk, dv, w.scale, ws)
    torch.cuda.synchronize()
    M = np.tril(np.ones((H, N // S, N // S), dtype=bool))
    dQ, dK, dV, O, LSE = orc.attention_backward(G.bits_f64(qb), G.bits_f64(kb), G.bits_f64(vb), G.bits_f64(gb),
                                                M, S, w.scale)
    assert G.o_excess(G.to_f64(o), O) <= 0
    assert np.abs(G.to_f64(lse) - LSE).max() <= LSE_TOL
    for n, got, ref in (("dq", dq, dQ), ("dk", dk, dK), ("dv", dv, dV)):
        assert G.rel_l2(G.to_f64(got), ref) <= GRAD_TOL, n
