"""GPU parity of the split-KV decode kernels against the fp64 oracle (through the C ABI)."""

import numpy as np
import pytest
import torch

from oracle import s2_oracle as orc
from paper_2407_17678_amd import binding as B
from paper_2407_17678_amd import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

O_TOL, LSE_TOL = 1e-2, 1e-3


def _run(w, qb, kcb, vcb, lens, max_len, splits, params=None):
    nseq, H, D = qb.shape
    q, kc, vc = G.to_dev(qb), G.to_dev(kcb), G.to_dev(vcb)
    sl = torch.from_numpy(lens).cuda()
    o = torch.empty_like(q)
    lse = torch.empty((nseq, H), dtype=torch.float32, device="cuda")
    p = params or B.layout_params(H, 1, w.block_size, w.local_blocks, w.stride, 0, w.window_blocks, 0)
    ws = torch.empty(B.s2_attn_decode_workspace_bytes(nseq, H, D, max_len, splits), dtype=torch.uint8,
                     device="cuda")
    B.s2_attn_decode(p, q, kc, vc, sl, o, lse, w.scale, ws, max_len, num_splits=splits)
    torch.cuda.synchronize()
    return G.to_f64(o), G.to_f64(lse)


def _oracle(w, qb, kcb, vcb, lens, base=0, dense=False):
    nseq, H, D = qb.shape
    q, kc, vc = G.bits_f64(qb), G.bits_f64(kcb), G.bits_f64(vcb)
    O = np.zeros((nseq, H, D))
    LSE = np.zeros((nseq, H))
    for b in range(nseq):
        for h in range(H):
            O[b, h], LSE[b, h] = orc.decode_row(q[b, h], kc[b, h], vc[b, h], int(lens[b]), base + h,
                                                w.block_size, w.local_blocks, w.stride, w.scale,
                                                w.window_blocks, dense)
    return O, LSE


@pytest.mark.parametrize("name,heads,max_len,splits", [
    ("7b_decode", 16, 2500, 0),     # S=64, 16 local + stride 16; library-chosen splits
    ("7b_decode", 16, 2500, 1),
    ("7b_decode", 5, 1500, 7),      # more splits than some sequences have units
    ("7b_128k", 4, 3000, 3),        # S=128, partial last block, half-empty last chunk
    ("tiny", 4, 700, 2),            # D=64
])
def test_decode_small(name, heads, max_len, splits):
    w = synth.WORKLOADS[name]
    nseq = 6
    lens = np.array([1, 63, 64, 65, max_len, max_len - 100], dtype=np.int32)
    if name == "7b_128k":
        lens = np.array([1, 127, 128, 129, 2048 + 17, max_len], dtype=np.int32)
    qb, kcb, vcb, lens = synth.decode_inputs_small(w, nseq, heads, max_len, lengths=lens)
    print("decode case", name, qb.shape, "max_len", max_len, "splits", splits, flush=True)
    o, lse = _run(w, qb, kcb, vcb, lens, max_len, splits)
    O, LSE = _oracle(w, qb, kcb, vcb, lens)
    eo, el = np.abs(o - O).max(), np.abs(lse - LSE).max()
    print("   max|dO| %.3e max|dLSE| %.3e" % (eo, el), flush=True)
    assert G.o_excess(o, O) <= 0 and el <= LSE_TOL


def test_decode_independent_of_split_count_and_head_base():
    w = synth.WORKLOADS["7b_decode"]
    qb, kcb, vcb, lens = synth.decode_inputs_small(w, 4, 8, 4096)
    outs = [_run(w, qb, kcb, vcb, lens, 4096, s) for s in (1, 2, 5, 16)]
    for o, lse in outs[1:]:
        assert np.abs(o - outs[0][0]).max() <= 2 ** -7      # one bf16 ulp of O(1) outputs
        assert np.abs(lse - outs[0][1]).max() <= 1e-5
    # a tensor-parallel shard: local head 0 is global head 8
    p = B.layout_params(8, 1, w.block_size, w.local_blocks, w.stride, 8, 0, 0)
    o, lse = _run(w, qb, kcb, vcb, lens, 4096, 3, params=p)
    O, LSE = _oracle(w, qb, kcb, vcb, lens, base=8)
    assert G.o_excess(o, O) <= 0 and np.abs(lse - LSE).max() <= LSE_TOL
    # dense decode
    p = B.layout_params(8, 1, 64, 1, 0, 0, 0, 1)
    o, lse = _run(w, qb, kcb, vcb, lens, 4096, 4, params=p)
    O, LSE = _oracle(w, qb, kcb, vcb, lens, dense=True)
    assert G.o_excess(o, O) <= 0 and np.abs(lse - LSE).max() <= LSE_TOL
