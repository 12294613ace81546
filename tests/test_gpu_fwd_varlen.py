"""GPU parity of the forward on packed variable-length batches (s2_attn_fwd_varlen; serving prefill
batches of section 5.3) against the fp64 oracle: ragged lengths, empty sequences, rows owned by no
sequence, every block size, and bit-identity with the fixed-length forward."""

import dataclasses

import numpy as np
import pytest
import torch

from oracle import s2_oracle as orc
from paper_2407_17678_amd import binding as B
from paper_2407_17678_amd import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

LSE_TOL = 1e-3
SENTINEL = 0x4248  # bf16 50.0: what o holds where the kernel must not write


def _run(w, H, lens, Bk, M=None, extra_rows=0, max_seqlen=None):
    S = w.block_size
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(cu[-1]) + extra_rows
    qb, kb, vb, _ = synth.train_inputs(w, heads=H, batch=1, seqlen=total)
    if M is None:
        M = orc.block_mask(H, Bk, w.local_blocks, w.stride)
        lay = B.s2_layout_build(B.layout_params(H, Bk, S, w.local_blocks, w.stride))
    else:
        row_ptr, col_idx, _, _ = orc.compressed_layout(M)
        lay = B.s2_layout_from_csr(H, Bk, S, row_ptr, col_idx)
    q, k, v = G.to_dev(qb), G.to_dev(kb), G.to_dev(vb)
    o = torch.full_like(q.view(torch.int16), SENTINEL).view(q.dtype)
    lse = torch.full((H, total), 77.0, dtype=torch.float32, device="cuda")
    B.s2_attn_fwd_varlen(lay, q, k, v, o, lse, torch.from_numpy(cu).cuda(),
                         max_seqlen if max_seqlen is not None else Bk * S, w.scale)
    torch.cuda.synchronize()
    return qb, kb, vb, cu, M, o, lse


CASES = {
    # name: (workload for D / seed, S, heads, layout blocks, B_l, stride, lengths)
    "S64_D128": ("1p3b_8k", 64, 3, 16, 2, 3, [1, 127, 128, 129, 700, 64, 0, 333, 1024]),
    "S16_D64": ("tiny", 16, 4, 16, 2, 5, [5, 16, 17, 31, 100, 250, 256, 33]),
    "S128_D128": ("7b_128k", 128, 2, 8, 2, 3, [130, 384, 1, 1000, 257]),
    "S32_D128": ("1p3b_8k", 32, 3, 20, 3, 4, [31, 32, 33, 95, 640, 2, 161]),
    "S64_D64_many_short": ("tiny", 64, 2, 4, 1, 2, [3, 9, 1, 64, 65, 12, 200, 7, 130, 256, 40, 99, 128, 5]),
}


@pytest.mark.parametrize("case", sorted(CASES))
def test_varlen_forward_against_the_oracle(case):
    wname, S, H, Bk, B_l, s, lens = CASES[case]
    w = dataclasses.replace(synth.WORKLOADS[wname], block_size=S, local_blocks=B_l, stride=s)
    print("varlen case", case, "H", H, "S", S, "B", Bk, "lens", lens, flush=True)
    qb, kb, vb, cu, M, o, lse = _run(w, H, lens, Bk, extra_rows=70)
    f = G.bits_f64
    O, LSE = orc.attention_forward_varlen(f(qb)[0], f(kb)[0], f(vb)[0], cu, M, S, w.scale)
    end = int(cu[-1])
    assert G.o_excess(G.to_f64(o)[0, :, :end], O[:, :end]) <= 0
    assert np.abs(G.to_f64(lse)[:, :end] - LSE[:, :end]).max() <= LSE_TOL
    # rows after the last sequence belong to nobody (the oracle says NaN there): untouched
    assert np.isnan(O[:, end:]).all()
    assert (o.view(torch.int16)[0, :, end:] == SENTINEL).all()
    assert (lse[:, end:] == 77.0).all()


def test_varlen_custom_pattern():
    w = dataclasses.replace(synth.WORKLOADS["1p3b_8k"], block_size=32)
    H, Bk, S = 2, 24, 32
    rng = np.random.default_rng(17)
    M = np.tril(rng.random((H, Bk, Bk)) < 0.3)
    i = np.arange(Bk)
    M[:, i, i] = True
    lens = [700, 45, 768, 129]
    qb, kb, vb, cu, M, o, lse = _run(w, H, lens, Bk, M=M)
    f = G.bits_f64
    O, LSE = orc.attention_forward_varlen(f(qb)[0], f(kb)[0], f(vb)[0], cu, M, S, w.scale)
    assert G.o_excess(G.to_f64(o)[0], O) <= 0
    assert np.abs(G.to_f64(lse) - LSE).max() <= LSE_TOL


def test_varlen_rows_agree_with_the_fixed_length_forward():
    # The two entry points may run differently scheduled kernels (the fixed-length one has a fast
    # path for whole 128-row tiles), so they agree to rounding, not bit for bit: O within one bf16
    # ulp of each other (and 1e-2), LSE within 1e-5.
    # each sequence on its own through s2_attn_fwd (lengths it accepts: whole blocks)
    w = dataclasses.replace(synth.WORKLOADS["1p3b_8k"], block_size=64, local_blocks=2, stride=3)
    H, Bk, S = 3, 12, 64
    lens = [768, 64, 320, 128]
    qb, kb, vb, cu, M, o, lse = _run(w, H, lens, Bk)
    q, k, v = G.to_dev(qb), G.to_dev(kb), G.to_dev(vb)
    for sq, L in enumerate(lens):
        lo = int(cu[sq])
        lay = B.s2_layout_build(B.layout_params(H, L // S, S, w.local_blocks, w.stride))
        qs, ks, vs = (x[:, :, lo:lo + L].contiguous() for x in (q, k, v))
        o1 = torch.empty_like(qs)
        lse1 = torch.empty((1, H, L), dtype=torch.float32, device="cuda")
        B.s2_attn_fwd(lay, qs, ks, vs, o1, lse1, w.scale)
        torch.cuda.synchronize()
        a, b = G.to_f64(o1), G.to_f64(o[:, :, lo:lo + L])
        assert (np.abs(a - b) <= np.maximum(1e-2, 2.0 ** -7 * np.abs(b))).all(), sq
        assert np.abs(G.to_f64(lse1[0]) - G.to_f64(lse[:, lo:lo + L])).max() <= 1e-5, sq


def test_varlen_length_above_the_stated_maximum_is_cut_there():
    # the kernel trusts no entry of cu_seqlens further than max_seqlen and the tensors' rows
    w = dataclasses.replace(synth.WORKLOADS["tiny"], block_size=64, local_blocks=2, stride=3)
    H, Bk, S = 2, 8, 64
    lens = [100, 300, 50]
    qb, kb, vb, cu, M, o, lse = _run(w, H, lens, Bk, max_seqlen=200)
    f = G.bits_f64
    cut = [100, 200, 50]
    for sq, L in enumerate(cut):
        lo = int(cu[sq])
        for h in range(H):
            O, LSE = orc.attention_forward_head(f(qb)[0, h, lo:lo + L], f(kb)[0, h, lo:lo + L], f(vb)[0, h, lo:lo + L],
                                                M[h], S, w.scale)
            assert G.o_excess(G.to_f64(o)[0, h, lo:lo + L], O) <= 0
            assert np.abs(G.to_f64(lse)[h, lo:lo + L] - LSE).max() <= LSE_TOL
    lo = int(cu[1])
    assert (o.view(torch.int16)[0, :, lo + 200:lo + 300] == SENTINEL).all()


def test_varlen_strided_tensors():
    # q / o and k / v as slices of wider buffers (token stride above head_dim, heads interleaved)
    w = dataclasses.replace(synth.WORKLOADS["1p3b_8k"], block_size=64, local_blocks=2, stride=3)
    H, Bk, S, D = 3, 8, 64, 128
    lens = [200, 17, 512, 90]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(cu[-1])
    qb, kb, vb, _ = synth.train_inputs(w, heads=H, batch=1, seqlen=total)
    lay = B.s2_layout_build(B.layout_params(H, Bk, S, w.local_blocks, w.stride))
    # [1, total, H, 3*D] buffer: q, k, v of a token side by side, heads next to each other
    buf = torch.zeros((1, total, H, 3 * D), dtype=torch.bfloat16, device="cuda")
    buf[..., 0:D] = G.to_dev(qb).permute(0, 2, 1, 3)
    buf[..., D:2 * D] = G.to_dev(kb).permute(0, 2, 1, 3)
    buf[..., 2 * D:] = G.to_dev(vb).permute(0, 2, 1, 3)
    q, k, v = (buf[..., i * D:(i + 1) * D].permute(0, 2, 1, 3) for i in range(3))
    obuf = torch.zeros((1, total, H, 3 * D), dtype=torch.bfloat16, device="cuda")
    o = obuf[..., 0:D].permute(0, 2, 1, 3)
    assert q.stride() == o.stride() and q.stride(2) == 3 * D * H
    lse = torch.empty((H, total), dtype=torch.float32, device="cuda")
    B.s2_attn_fwd_varlen(lay, q, k, v, o, lse, torch.from_numpy(cu).cuda(), Bk * S, w.scale)
    torch.cuda.synchronize()
    M = orc.block_mask(H, Bk, w.local_blocks, w.stride)
    f = G.bits_f64
    O, LSE = orc.attention_forward_varlen(f(qb)[0], f(kb)[0], f(vb)[0], cu, M, S, w.scale)
    assert G.o_excess(G.to_f64(o.contiguous())[0], O) <= 0
    assert np.abs(G.to_f64(lse) - LSE).max() <= LSE_TOL
    assert (obuf[..., D:] == 0).all()   # nothing written outside o's columns
