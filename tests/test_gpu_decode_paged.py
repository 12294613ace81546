"""GPU parity of decoding against a paged KV cache with evicted blocks (through the C ABI) against
the fp64 oracle; the pages and the block table are inputs that both sides receive."""

import numpy as np
import pytest
import torch

from oracle import s2_oracle as orc
from paper_2407_17678_amd import binding as B
from paper_2407_17678_amd import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

O_TOL, LSE_TOL = 1e-2, 1e-3


def _params(w, H, base=0, dense=0):
    return B.layout_params(H, 1, w.block_size, w.local_blocks, w.stride, base, w.window_blocks, dense)


def _run(w, qb, kpool, vpool, table, lens, splits, params, with_missing=True):
    nseq, H, D = qb.shape
    q, kp, vp = G.to_dev(qb), G.to_dev(kpool), G.to_dev(vpool)
    tb = torch.from_numpy(table).cuda()
    sl = torch.from_numpy(lens).cuda()
    o = torch.empty_like(q)
    lse = torch.empty((nseq, H), dtype=torch.float32, device="cuda")
    missing = torch.zeros(1, dtype=torch.int32, device="cuda") if with_missing else None
    max_len = table.shape[2] * w.block_size
    ws = torch.empty(B.s2_attn_decode_workspace_bytes(nseq, H, D, max_len, splits), dtype=torch.uint8,
                     device="cuda")
    B.s2_attn_decode_paged(params, q, kp, vp, tb, sl, o, lse, w.scale, ws, missing=missing, num_splits=splits)
    torch.cuda.synchronize()
    return G.to_f64(o), G.to_f64(lse), (int(missing.item()) if with_missing else None)


def _oracle(w, qb, kpool, vpool, table, lens, base=0, dense=False):
    nseq, H, D = qb.shape
    q, kp, vp = G.bits_f64(qb), G.bits_f64(kpool), G.bits_f64(vpool)
    O = np.zeros((nseq, H, D))
    LSE = np.zeros((nseq, H))
    for b in range(nseq):
        for h in range(H):
            O[b, h], LSE[b, h] = orc.paged_decode_row(q[b, h], kp, vp, table[b, h], int(lens[b]), base + h,
                                                      w.block_size, w.local_blocks, w.stride, w.scale,
                                                      w.window_blocks, dense)
    return O, LSE


def _resident(w, H, lens, base=0, dense=False):
    return [[orc.resident_blocks(int(L), base + h, w.block_size, w.local_blocks, w.stride, w.window_blocks, dense)
             for h in range(H)] for L in lens]


@pytest.mark.parametrize("name,heads,max_len,splits,base", [
    ("7b_decode", 16, 2500, 0, 0),   # S=64, 16 local + stride 16
    ("7b_decode", 5, 1500, 7, 9),    # more splits than some sequences have units; head index base
    ("7b_128k", 4, 3000, 3, 0),      # S=128, partial last block
    ("tiny", 4, 700, 2, 0),          # D=64
])
def test_paged_decode_with_evicted_blocks(name, heads, max_len, splits, base):
    w = synth.WORKLOADS[name]
    S = w.block_size
    lens = np.array([1, S - 1, S, S + 1, max_len, max_len - 100], dtype=np.int32)
    nseq = len(lens)
    qb, kcb, vcb, lens = synth.decode_inputs_small(w, nseq, heads, max_len, lengths=lens)
    max_blocks = -(-max_len // S)
    resident = _resident(w, heads, lens, base)
    table, num_pages = synth.page_table(resident, max_blocks, index=w.index)
    pad = max_blocks * S - max_len
    if pad:
        kcb = np.concatenate([kcb, np.zeros((nseq, heads, pad, w.head_dim), np.uint16)], axis=2)
        vcb = np.concatenate([vcb, np.zeros((nseq, heads, pad, w.head_dim), np.uint16)], axis=2)
    kpool = synth.pages_from_cache(kcb, table, num_pages, S)
    vpool = synth.pages_from_cache(vcb, table, num_pages, S)
    print("paged decode case", name, qb.shape, "pages", num_pages, "of", nseq * heads * max_blocks, flush=True)
    params = _params(w, heads, base)
    # the library's own eviction helper names the same blocks
    for b in range(nseq):
        for h in range(heads):
            assert B.s2_kv_resident_blocks(params, h, int(lens[b])) == resident[b][h]
    o, lse, missing = _run(w, qb, kpool, vpool, table, lens, splits, params)
    O, LSE = _oracle(w, qb, kpool, vpool, table, lens, base)
    assert missing == 0
    assert np.isfinite(O).all()
    assert G.o_excess(o, O) <= 0, np.abs(o - O).max()
    assert np.abs(lse - LSE).max() <= LSE_TOL
    # and it is what the contiguous cache gives (storage does not change the result)
    O2 = np.zeros_like(O)
    for b in range(nseq):
        for h in range(heads):
            O2[b, h], _ = orc.decode_row(G.bits_f64(qb[b, h]), G.bits_f64(kcb[b, h]), G.bits_f64(vcb[b, h]),
                                         int(lens[b]), base + h, S, w.local_blocks, w.stride, w.scale,
                                         w.window_blocks)
    assert np.array_equal(O, O2)


def test_paged_dense_layout_and_no_missing_pointer():
    w = synth.WORKLOADS["tiny"]
    S, heads, max_len = w.block_size, 3, 400
    lens = np.array([400, 77, 129], dtype=np.int32)
    qb, kcb, vcb, lens = synth.decode_inputs_small(w, 3, heads, max_len, lengths=lens)
    max_blocks = -(-max_len // S)
    resident = _resident(w, heads, lens, dense=True)
    table, num_pages = synth.page_table(resident, max_blocks, index=w.index)
    pad = max_blocks * S - max_len
    kcb = np.concatenate([kcb, np.zeros((3, heads, pad, w.head_dim), np.uint16)], axis=2)
    vcb = np.concatenate([vcb, np.zeros((3, heads, pad, w.head_dim), np.uint16)], axis=2)
    kpool = synth.pages_from_cache(kcb, table, num_pages, S)
    vpool = synth.pages_from_cache(vcb, table, num_pages, S)
    params = _params(w, heads, dense=1)
    o, lse, _ = _run(w, qb, kpool, vpool, table, lens, 0, params, with_missing=False)
    O, LSE = _oracle(w, qb, kpool, vpool, table, lens, dense=True)
    assert G.o_excess(o, O) <= 0
    assert np.abs(lse - LSE).max() <= LSE_TOL


def test_missing_blocks_are_counted_and_skipped():
    w = synth.WORKLOADS["7b_decode"]
    S, heads, max_len = w.block_size, 4, 2048
    lens = np.array([2048, 1000], dtype=np.int32)
    qb, kcb, vcb, lens = synth.decode_inputs_small(w, 2, heads, max_len, lengths=lens)
    max_blocks = max_len // S
    resident = _resident(w, heads, lens)
    table, num_pages = synth.page_table(resident, max_blocks, index=w.index)
    kpool = synth.pages_from_cache(kcb, table, num_pages, S)
    vpool = synth.pages_from_cache(vcb, table, num_pages, S)
    params = _params(w, heads)
    # drop two kept blocks of (0, 1), point one kept block of (1, 2) past the pool, and drop
    # everything of (1, 3)
    broken = table.copy()
    gone = resident[0][1][:2]
    for j in gone:
        broken[0, 1, j] = -1
    broken[1, 2, resident[1][2][-1]] = num_pages + 5
    broken[1, 3, :] = -1
    expect_missing = 2 + 1 + len(resident[1][3])
    o, lse, missing = _run(w, qb, kpool, vpool, broken, lens, 3, params)
    assert missing == expect_missing
    assert np.isfinite(o).all()
    assert (o[1, 3] == 0).all() and lse[1, 3] == -np.inf
    # untouched (sequence, head) pairs are unaffected
    O, LSE = _oracle(w, qb, kpool, vpool, table, lens)
    for b, h in ((0, 0), (0, 2), (0, 3), (1, 0), (1, 1)):
        assert G.o_excess(o[b, h], O[b, h]) <= 0
        assert abs(lse[b, h] - LSE[b, h]) <= LSE_TOL
    # (0, 1) without its two blocks equals the oracle on a cache where those blocks' keys cannot win:
    # checked as a property instead: the remaining softmax mass is smaller, so lse drops
    assert lse[0, 1] < LSE[0, 1] + LSE_TOL


def test_paged_argument_errors():
    w = synth.WORKLOADS["tiny"]
    heads = 2
    q = torch.zeros((1, heads, 64), dtype=torch.bfloat16, device="cuda")
    kp = torch.zeros((4, 64, 64), dtype=torch.bfloat16, device="cuda")
    tb = torch.zeros((1, heads, 2), dtype=torch.int32, device="cuda")
    sl = torch.ones(1, dtype=torch.int32, device="cuda")
    o = torch.empty_like(q)
    ws = torch.empty(B.s2_attn_decode_workspace_bytes(1, heads, 64, 128, 0), dtype=torch.uint8, device="cuda")
    with pytest.raises(B.S2Error) as e:
        B.s2_attn_decode_paged(_params(w, heads + 1), q, kp, kp, tb, sl, o, None, w.scale, ws)
    assert e.value.status == -3  # SHAPE: heads differ
    with pytest.raises(B.S2Error) as e:
        B.s2_attn_decode_paged(_params(w, heads), q, kp, kp, tb, sl, o, None, -1.0, ws)
    assert e.value.status == -2  # BAD_PARAM: scale
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.S2Error) as e:
        B.s2_attn_decode_paged(_params(w, heads), q, kp, kp, tb, sl, o, None, w.scale, small)
    assert e.value.status == -5  # WORKSPACE
