"""A seeded sweep over valid shapes and patterns: block size, head dimension, heads, batch, length,
window, stride, head index base and stripe window all drawn at random, forward and backward against
the fp64 oracle each time.  The cases are fixed by the seed; they widen coverage beyond the
hand-picked ones (odd combinations such as stride 1, windows longer than the sequence, a single
block, strides above the head count)."""

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


def _cases(n, seed=20240717):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        S = int(rng.choice([16, 32, 64, 128]))
        D = int(rng.choice([64, 128]))
        H = int(rng.integers(1, 6))
        batch = int(rng.integers(1, 3))
        max_blocks = {16: 40, 32: 24, 64: 14, 128: 8}[S]
        Bk = int(rng.integers(1, max_blocks + 1))
        if S == 16:
            Bk += Bk & 1
        B_l = int(rng.integers(1, min(Bk, 6) + 2))          # may exceed the number of blocks
        stride = int(rng.choice([0, 1, 2, 3, 5, 8, 11]))
        base = int(rng.integers(0, 9))
        window = int(rng.choice([0, 0, 0, 4, 9]))
        out.append((S, D, H, batch, Bk, B_l, stride, base, window))
    return out


@pytest.mark.parametrize("case", _cases(24), ids=lambda c: "S%d_D%d_H%d_b%d_B%d_L%d_V%d_o%d_w%d" % c)
def test_random_case(case):
    S, D, H, batch, Bk, B_l, stride, base, window = case
    N = Bk * S
    w = dataclasses.replace(synth.WORKLOADS["tiny" if D == 64 else "1p3b_8k"], block_size=S, local_blocks=B_l,
                            stride=stride, window_blocks=window)
    print("sweep case", case, flush=True)
    qb, kb, vb, gb = synth.train_inputs(w, heads=H, batch=batch, seqlen=N)
    params = B.layout_params(H, Bk, S, B_l, stride, base, window, 0)
    lay = B.s2_layout_build(params)
    M = orc.block_mask(H, Bk, B_l, stride, base, window)
    got = B.s2_layout_get(lay)
    row_ptr, col_idx, _, _ = orc.compressed_layout(M)
    assert np.array_equal(got["row_ptr"], row_ptr) and np.array_equal(got["col_idx"], col_idx)
    q, k, v, g = G.to_dev(qb), G.to_dev(kb), G.to_dev(vb), G.to_dev(gb)
    o = torch.empty_like(q)
    lse = torch.empty((batch, H, N), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ws = torch.empty(B.s2_attn_bwd_workspace_bytes(batch, H, N, D), dtype=torch.uint8, device="cuda")
    B.s2_attn_fwd(lay, q, k, v, o, lse, w.scale)
    B.s2_attn_bwd(lay, q, k, v, o, lse, g, dq, dk, dv, w.scale, ws)
    torch.cuda.synchronize()
    dQ, dK, dV, O, LSE = orc.attention_backward(G.bits_f64(qb), G.bits_f64(kb), G.bits_f64(vb), G.bits_f64(gb),
                                                M, S, w.scale)
    assert G.o_excess(G.to_f64(o), O) <= 0
    assert np.abs(G.to_f64(lse) - LSE).max() <= LSE_TOL
    for n, got_t, ref in (("dq", dq, dQ), ("dk", dk, dK), ("dv", dv, dV)):
        assert G.rel_l2(G.to_f64(got_t), ref) <= GRAD_TOL, n


def _decode_cases(n, seed=20240718):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        S = int(rng.choice([16, 32, 64, 128]))
        D = int(rng.choice([64, 128]))
        H = int(rng.integers(1, 7))
        nseq = int(rng.integers(1, 6))
        max_len = int(rng.integers(1, 1500))
        B_l = int(rng.integers(1, 8))
        stride = int(rng.choice([0, 1, 2, 3, 5, 8, 11]))
        base = int(rng.integers(0, 9))
        window = int(rng.choice([0, 0, 5]))
        splits = int(rng.choice([0, 1, 2, 5, 16]))
        paged = bool(rng.integers(0, 2))
        out.append((S, D, H, nseq, max_len, B_l, stride, base, window, splits, paged))
    return out


@pytest.mark.parametrize("case", _decode_cases(16), ids=lambda c: "S%d_D%d_H%d_n%d_len%d_L%d_V%d_o%d_w%d_sp%d_pg%d" % c)
def test_random_decode_case(case):
    S, D, H, nseq, max_len, B_l, stride, base, window, splits, paged = case
    w = dataclasses.replace(synth.WORKLOADS["tiny" if D == 64 else "7b_decode"], block_size=S, local_blocks=B_l,
                            stride=stride, window_blocks=window)
    print("decode sweep case", case, flush=True)
    rng = np.random.default_rng(sum(case))
    lens = rng.integers(1, max_len + 1, size=nseq).astype(np.int32)
    lens[0] = max_len
    qb, kcb, vcb, lens = synth.decode_inputs_small(w, nseq, H, max_len, lengths=lens)
    params = B.layout_params(H, 1, S, B_l, stride, base, window, 0)
    q = G.to_dev(qb)
    sl = torch.from_numpy(lens).cuda()
    o = torch.empty_like(q)
    lse = torch.empty((nseq, H), dtype=torch.float32, device="cuda")
    max_blocks = -(-max_len // S)
    ws = torch.empty(B.s2_attn_decode_workspace_bytes(nseq, H, D, max_blocks * S, splits), dtype=torch.uint8,
                     device="cuda")
    f = G.bits_f64
    if paged:
        resident = [[B.s2_kv_resident_blocks(params, h, int(L)) for h in range(H)] for L in lens]
        for b, L in enumerate(lens):
            for h in range(H):
                assert resident[b][h] == orc.resident_blocks(int(L), base + h, S, B_l, stride, window)
        table, num_pages = synth.page_table(resident, max_blocks, index=w.index)
        pad = max_blocks * S - max_len
        kcb = np.concatenate([kcb, np.zeros((nseq, H, pad, D), np.uint16)], axis=2)
        vcb = np.concatenate([vcb, np.zeros((nseq, H, pad, D), np.uint16)], axis=2)
        kpool = synth.pages_from_cache(kcb, table, num_pages, S)
        vpool = synth.pages_from_cache(vcb, table, num_pages, S)
        missing = torch.zeros(1, dtype=torch.int32, device="cuda")
        B.s2_attn_decode_paged(params, q, G.to_dev(kpool), G.to_dev(vpool), torch.from_numpy(table).cuda(), sl, o,
                               lse, w.scale, ws, missing=missing, num_splits=splits)
        torch.cuda.synchronize()
        assert int(missing.item()) == 0
    else:
        B.s2_attn_decode(params, q, G.to_dev(kcb), G.to_dev(vcb), sl, o, lse, w.scale, ws, max_len, num_splits=splits)
        torch.cuda.synchronize()
    for b in range(nseq):
        for h in range(H):
            ref, ref_lse = orc.decode_row(f(qb)[b, h], f(kcb)[b, h], f(vcb)[b, h], int(lens[b]), base + h, S, B_l,
                                          stride, w.scale, window)
            assert G.o_excess(G.to_f64(o[b, h]), ref) <= 0, (b, h)
            assert abs(float(lse[b, h]) - ref_lse) <= LSE_TOL, (b, h)
