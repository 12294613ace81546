"""GPU parity of forward, backward and decode under caller-supplied per-head patterns (s2_layout_from_csr):
attention sink, the same shards for all heads, per-context-range and random patterns (sections 3
and 5.1) against the fp64 oracle evaluated on the same block mask."""

import numpy as np
import pytest
import torch

from oracle import s2_oracle as orc
from paper_2407_17678_amd import binding as B
from paper_2407_17678_amd import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

LSE_TOL, GRAD_TOL = 1e-3, 2e-2


def _per_range_mask(H, Bk):
    """Per head AND per context range: early rows dense, middle rows window 3 + stripes of stride 4
    with the head's offset, late rows window 2 + sink 1 + stripes of stride 8."""
    M = np.zeros((H, Bk, Bk), dtype=bool)
    for h in range(H):
        for i in range(Bk):
            for j in range(i + 1):
                d = i - j
                if i < Bk // 4:
                    keep = True
                elif i < Bk // 2:
                    keep = d < 3 or (j % 4 == h % 4)
                else:
                    keep = d < 2 or j == 0 or (j % 8 == (3 * h) % 8)
                M[h, i, j] = keep
    return M


def _random_mask(seed, H, Bk, density):
    rng = np.random.default_rng(seed)
    M = np.tril(rng.random((H, Bk, Bk)) < density)
    i = np.arange(Bk)
    M[:, i, i] = True
    return M


CASES = {
    # name: (workload for shapes/seed, heads, seqlen, mask builder)
    "sink_S64_D128": ("1p3b_8k", 3, 1536, lambda H, Bk: orc.with_sink(orc.block_mask(H, Bk, 4, 8), 2)),
    "homogeneous_S64_D128": ("1p3b_8k", 3, 1024, lambda H, Bk: orc.homogeneous_mask(H, Bk, 3, 4, offset=2)),
    "per_range_S64_D64": ("tiny", 4, 1280, _per_range_mask),
    "random_sparse_S128_D128": ("7b_128k", 2, 2048, lambda H, Bk: _random_mask(1, H, Bk, 0.3)),
    "random_dense_S64_D64": ("tiny", 2, 768, lambda H, Bk: _random_mask(2, H, Bk, 0.8)),
    "diagonal_only_S64_D128": ("1p3b_8k", 2, 512, lambda H, Bk: _random_mask(3, H, Bk, 0.0)),
}


@pytest.mark.parametrize("case", sorted(CASES))
def test_custom_layout_fwd_bwd(case):
    wname, H, N, build = CASES[case]
    w = synth.WORKLOADS[wname]
    S = w.block_size
    Bk = N // S
    M = build(H, Bk)
    assert orc.valid_custom_mask(M)
    print("custom layout case", case, "H", H, "N", N, "S", S, "nnz", int(M.sum()), flush=True)
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
    for name, got, want in (("dq", dq, dQ), ("dk", dk, dK), ("dv", dv, dV)):
        assert G.rel_l2(G.to_f64(got), want) <= GRAD_TOL, name


def test_custom_layout_equal_to_the_rule_gives_identical_bits():
    # the section 4.2 pattern passed in as lists must run exactly like the built-in builder
    w = synth.WORKLOADS["tiny"]
    H, N, S = w.heads, w.seqlen, w.block_size
    qb, kb, vb, gb = synth.train_inputs(w)
    M = orc.block_mask(H, N // S, w.local_blocks, w.stride)
    row_ptr, col_idx, _, _ = orc.compressed_layout(M)
    q, k, v = G.to_dev(qb), G.to_dev(kb), G.to_dev(vb)
    outs = []
    for lay in (B.s2_layout_from_csr(H, N // S, S, row_ptr, col_idx),
                B.s2_layout_build(B.layout_params(H, N // S, S, w.local_blocks, w.stride))):
        o = torch.empty_like(q)
        lse = torch.empty((1, H, N), dtype=torch.float32, device="cuda")
        B.s2_attn_fwd(lay, q, k, v, o, lse, w.scale)
        torch.cuda.synchronize()
        outs.append((o.clone(), lse.clone()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])


DECODE_CASES = {
    # name: (workload, heads, block size, layout blocks, mask builder)
    "sink_S64": ("7b_decode", 4, 64, 20, lambda H, Bk: orc.with_sink(orc.block_mask(H, Bk, 3, 5), 2)),
    "random_S64": ("7b_decode", 3, 64, 18, lambda H, Bk: _random_mask(11, H, Bk, 0.4)),
    "per_range_S128": ("7b_decode", 4, 128, 12, _per_range_mask),
    "random_S16": ("7b_decode", 3, 16, 64, lambda H, Bk: _random_mask(12, H, Bk, 0.15)),
    "random_S32_D64": ("tiny", 2, 32, 30, lambda H, Bk: _random_mask(13, H, Bk, 0.5)),
}


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("case", sorted(DECODE_CASES))
def test_custom_layout_decode(case, paged):
    wname, H, S, Bk, build = DECODE_CASES[case]
    w = synth.WORKLOADS[wname]
    M = build(H, Bk)
    max_len = Bk * S
    lens = np.array([1, S - 1, S, S + 1, max_len // 2 + 3, max_len - 1, max_len], dtype=np.int32)
    nseq = len(lens)
    print("custom decode case", case, "paged", paged, "H", H, "S", S, "B", Bk, flush=True)
    qb, kcb, vcb, lens = synth.decode_inputs_small(w, nseq, H, max_len, lengths=lens)
    row_ptr, col_idx, _, _ = orc.compressed_layout(M)
    lay = B.s2_layout_from_csr(H, Bk, S, row_ptr, col_idx)
    q = G.to_dev(qb)
    sl = torch.from_numpy(lens).cuda()
    o = torch.empty_like(q)
    lse = torch.empty((nseq, H), dtype=torch.float32, device="cuda")
    ws = torch.empty(B.s2_attn_decode_workspace_bytes(nseq, H, w.head_dim, max_len, 3), dtype=torch.uint8,
                     device="cuda")
    f = G.bits_f64
    if paged:
        # hold exactly what the layout says must stay: blocks kept by later rows only are resident
        # too, blocks nobody will read again are gone
        resident = [[B.s2_layout_resident_blocks(lay, h, int(L)) for h in range(H)] for L in lens]
        for b, L in enumerate(lens):
            for h in range(H):
                assert resident[b][h] == orc.resident_blocks_mask(M[h], int(L), S)
        table, num_pages = synth.page_table(resident, Bk, index=w.index)
        kpool = synth.pages_from_cache(kcb, table, num_pages, S)
        vpool = synth.pages_from_cache(vcb, table, num_pages, S)
        missing = torch.zeros(1, dtype=torch.int32, device="cuda")
        B.s2_attn_decode_paged_layout(lay, q, G.to_dev(kpool), G.to_dev(vpool), torch.from_numpy(table).cuda(), sl,
                                      o, lse, w.scale, ws, missing=missing, num_splits=3)
        torch.cuda.synchronize()
        assert int(missing.item()) == 0
    else:
        B.s2_attn_decode_layout(lay, q, G.to_dev(kcb), G.to_dev(vcb), sl, o, lse, w.scale, ws, max_len, num_splits=3)
        torch.cuda.synchronize()
    for b in range(nseq):
        for h in range(H):
            if paged:
                ref, ref_lse = orc.paged_decode_row_mask(f(qb)[b, h], f(kpool), f(vpool), table[b, h], int(lens[b]),
                                                         M[h], S, w.scale)
            else:
                ref, ref_lse = orc.decode_row_mask(f(qb)[b, h], f(kcb)[b, h], f(vcb)[b, h], int(lens[b]), M[h], S,
                                                   w.scale)
            assert G.o_excess(G.to_f64(o[b, h]), ref) <= 0, (b, h)
            assert abs(float(lse[b, h]) - ref_lse) <= LSE_TOL, (b, h)


def test_layout_decode_of_the_rule_gives_the_closed_form_bits():
    # a layout built from section 4.2's rule must decode exactly like the closed-form entry point
    w = synth.WORKLOADS["7b_decode"]
    H, S, Bk = 5, 64, 24
    max_len = Bk * S
    lens = np.array([1, 64, 65, 1000, max_len], dtype=np.int32)
    qb, kcb, vcb, lens = synth.decode_inputs_small(w, len(lens), H, max_len, lengths=lens)
    params = B.layout_params(H, Bk, S, 3, 6)
    lay = B.s2_layout_build(params)
    q, kc, vc = G.to_dev(qb), G.to_dev(kcb), G.to_dev(vcb)
    sl = torch.from_numpy(lens).cuda()
    ws = torch.empty(B.s2_attn_decode_workspace_bytes(len(lens), H, w.head_dim, max_len, 4), dtype=torch.uint8,
                     device="cuda")
    outs = []
    for use_layout in (False, True):
        o = torch.empty_like(q)
        lse = torch.empty((len(lens), H), dtype=torch.float32, device="cuda")
        if use_layout:
            B.s2_attn_decode_layout(lay, q, kc, vc, sl, o, lse, w.scale, ws, max_len, num_splits=4)
        else:
            B.s2_attn_decode(params, q, kc, vc, sl, o, lse, w.scale, ws, max_len, num_splits=4)
        torch.cuda.synchronize()
        outs.append((o.clone(), lse.clone()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
