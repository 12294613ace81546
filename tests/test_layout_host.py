"""CPU tests of the library's host side: symbols, the closed-form layout builder (bit-exact
against the oracle's scan of the predicate), and every argument-error path.  No kernel runs."""

import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import s2_oracle as orc
from paper_2407_17678_amd import binding as B
from paper_2407_17678_amd.synth import WORKLOADS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "s2attn.h")).read()
    declared = set(re.findall(r"\b(s2_[a-z_0-9]+)\s*\(", header))
    assert declared, "no declarations found"
    lib = B.lib()
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(B.EXPORTS)
    assert lib.s2_version() >= 100
    assert lib.s2_status_string(0) == b"ok"
    for code in range(-8, 0):
        assert lib.s2_status_string(code) not in (b"ok", b"unknown status")


def _compare(H, Bk, S, B_l, s, base=0, win=0, dense=0):
    lay = B.s2_layout_build(B.layout_params(H, Bk, S, B_l, s, base, win, dense))
    got = B.s2_layout_get(lay)
    M = orc.block_mask(H, Bk, B_l, s, head_index_base=base, window_blocks=win, dense=bool(dense))
    row_ptr, col_idx, col_ptr, row_idx = orc.compressed_layout(M)
    assert got["nnz"] == int(M.sum())
    for name, want in (("row_ptr", row_ptr), ("col_idx", col_idx), ("col_ptr", col_ptr),
                       ("row_idx", row_idx)):
        assert got[name].dtype == np.int32
        assert np.array_equal(got[name], want), name
    assert got["covers_all"] == int(orc.covers_all(M))
    assert got["max_row_blocks"] == int(M.sum(axis=2).max())
    B.s2_layout_destroy(lay)
    return got


@pytest.mark.parametrize("name", ["tiny", "1p3b_8k", "7b_32k", "7b_128k"])
def test_layout_bit_exact_at_workloads(name):
    w = WORKLOADS[name]
    got = _compare(w.heads, w.num_blocks, w.block_size, w.local_blocks, w.stride)
    assert got["nnz"] == {"tiny": 81, "1p3b_8k": 23596, "7b_32k": 504816, "7b_128k": 777884}[name]
    assert got["covers_all"] == 1


def test_layout_bit_exact_random_parameters():
    rng = np.random.default_rng(11)
    for _ in range(120):
        H = int(rng.integers(1, 10))
        Bk = int(rng.integers(1, 70))
        S = int(rng.choice([32, 64, 128]))
        B_l = int(rng.integers(1, 9))
        s = int(rng.integers(0, 12))
        base = int(rng.integers(0, 20))
        win = int(rng.choice([0, 0, int(rng.integers(1, 70))]))
        dense = int(rng.random() < 0.1)
        _compare(H, Bk, S, B_l, s, base, win, dense)


def test_layout_variants():
    _compare(16, 128, 64, 1, 15)        # L1V15
    _compare(16, 128, 64, 9, 0)         # sliding window only
    _compare(16, 128, 64, 2, 18)        # stride above head count: union incomplete
    assert _compare(16, 128, 64, 2, 18)["covers_all"] == 0
    _compare(4, 33, 128, 200, 3)        # B_l >= B is dense
    _compare(8, 64, 64, 4, 8, base=8)   # second tensor-parallel shard of 16 heads
    _compare(6, 96, 16, 3, 5)           # 16-token blocks
    _compare(6, 96, 32, 3, 5)


@pytest.mark.parametrize("kw,code", [
    (dict(num_heads=0), -2), (dict(num_blocks=0), -2), (dict(block_size=8), -2), (dict(block_size=96), -2),
    (dict(block_size=16, num_blocks=5), -2),   # 16-token blocks come in pairs
    (dict(local_blocks=0), -2), (dict(stride=-1), -2), (dict(window_blocks=-1), -2),
    (dict(head_index_base=-1), -2), (dict(dense=2), -2),
])
def test_layout_bad_params(kw, code):
    args = dict(num_heads=2, num_blocks=4, block_size=64, local_blocks=1, stride=2, head_index_base=0,
                window_blocks=0, dense=0)
    args.update(kw)
    with pytest.raises(B.S2Error) as e:
        B.s2_layout_build(B.layout_params(**args))
    assert e.value.status == code


def test_null_and_overflow_paths():
    lib = B.lib()
    out = C.c_void_p()
    assert lib.s2_layout_build(None, C.byref(out)) == -1
    p = B.layout_params(1, 1, 64, 1, 0)
    assert lib.s2_layout_build(C.byref(p), None) == -1
    assert lib.s2_layout_destroy(None) == -1
    assert lib.s2_layout_get(None, None) == -1
    # dense layout whose block count would overflow int32
    big = B.layout_params(64, 70000, 64, 1, 0, dense=1)
    assert lib.s2_layout_build(C.byref(big), C.byref(out)) == -8


def _tensors(**kw):
    base = dict(q=256, k=256, v=256, o=256, lse=256, d_o=256, dq=256, dk=256, dv=256, batch=1, heads=2,
                seqlen=256, head_dim=128, q_stride_b=2 * 256 * 128, q_stride_h=256 * 128, q_stride_t=128,
                kv_stride_b=2 * 256 * 128, kv_stride_h=256 * 128, kv_stride_t=128)
    base.update(kw)
    return B.Tensors(**base)


def test_attention_argument_errors_without_device():
    """Validation happens before any launch, so these run (and fail cleanly) with no GPU.
    Pointers are fake non-null addresses that are never dereferenced on these paths."""
    lib = B.lib()
    lay = B.s2_layout_build(B.layout_params(2, 4, 64, 1, 2))
    h = lay.handle
    call = lambda t, scale=0.1: lib.s2_attn_fwd(h, C.byref(t), scale, None)
    assert lib.s2_attn_fwd(None, C.byref(_tensors()), 0.1, None) == -1
    assert lib.s2_attn_fwd(h, None, 0.1, None) == -1
    assert call(_tensors(q=None)) == -1
    assert call(_tensors(), scale=0.0) == -2
    assert call(_tensors(), scale=float("nan")) == -2
    assert call(_tensors(head_dim=96)) == -3
    assert call(_tensors(heads=3)) == -3
    assert call(_tensors(seqlen=192)) == -3
    assert call(_tensors(q=264)) == -4
    assert call(_tensors(q_stride_t=132)) == -4
    assert call(_tensors(kv_stride_t=64)) == -4
    ws = 1 << 20
    bwd = lambda t, wptr=256, wbytes=ws: lib.s2_attn_bwd(h, C.byref(t), 0.1, wptr, wbytes, None)
    assert bwd(_tensors(dq=None)) == -1
    assert bwd(_tensors(), wptr=None) == -5
    assert bwd(_tensors(), wbytes=16) == -5
    assert bwd(_tensors(), wptr=264) == -5
    need = lib.s2_attn_bwd_workspace_bytes(1, 2, 256, 128)
    assert need >= 1 * 2 * 256 * 4 and need % 256 == 0
    assert lib.s2_dense_causal_fwd(C.byref(_tensors(seqlen=192)), 0.1, None) == -3
    assert lib.s2_dense_causal_fwd(None, 0.1, None) == -1
    import torch
    if not torch.cuda.is_available():
        # a host-only layout refuses to launch
        assert B.s2_layout_get(lay)["on_device"] == 0
        assert call(_tensors()) == -7


def test_decode_argument_errors():
    lib = B.lib()
    p = B.layout_params(2, 1, 64, 2, 4)
    def args(**kw):
        base = dict(q=256, k_cache=256, v_cache=256, seq_lens=256, o=256, lse=None, nseq=3, heads=2,
                    head_dim=128, max_len=1000, num_splits=2, kv_stride_seq=2 * 1000 * 128,
                    kv_stride_head=1000 * 128, kv_stride_tok=128)
        base.update(kw)
        return B.DecodeArgs(**base)
    call = lambda a, scale=0.1, ws=256, wb=1 << 20, pp=p: lib.s2_attn_decode(
        C.byref(pp), C.byref(a), scale, ws, wb, None)
    assert lib.s2_attn_decode(None, C.byref(args()), 0.1, 256, 1 << 20, None) == -1
    assert call(args(q=None)) == -1
    assert call(args(), scale=-1.0) == -2
    assert call(args(heads=4)) == -3
    assert call(args(head_dim=32)) == -3
    assert call(args(num_splits=100)) == -2
    assert call(args(kv_stride_tok=100)) == -4
    assert call(args(k_cache=260)) == -4
    assert call(args(), ws=None) == -5
    assert call(args(), wb=8) == -5
    assert call(args(), pp=B.layout_params(2, 1, 64, 0, 4)) == -2
    need = lib.s2_attn_decode_workspace_bytes(3, 2, 128, 1000, 2)
    assert need >= 3 * 2 * 2 * 130 * 4
    assert 1 <= lib.s2_attn_decode_default_splits(64, 32, 32768) <= 64


def test_resident_blocks_bit_exact_against_the_oracle():
    # the cache manager's helper (which blocks a head may never evict) against the oracle's
    # definition-by-scan, at the decode workload and at random parameters incl. windows
    w = WORKLOADS["7b_decode"]
    p = B.layout_params(w.heads, 1, w.block_size, w.local_blocks, w.stride, 0, w.window_blocks, 0)
    for h in (0, 5, 15, 31):
        for L in (1, 64, 65, 1024, 8192, 20001, 32768):
            assert B.s2_kv_resident_blocks(p, h, L) == orc.resident_blocks(L, h, 64, w.local_blocks, w.stride)
    rng = np.random.default_rng(5)
    for _ in range(150):
        S = int(rng.choice([32, 64, 128]))
        H = int(rng.integers(1, 9))
        B_l = int(rng.integers(1, 7))
        s = int(rng.integers(0, 9))
        win = int(rng.choice([0, 0, rng.integers(B_l, 40)]))
        base = int(rng.integers(0, 20))
        dense = int(rng.integers(0, 8) == 0)
        h = int(rng.integers(0, H))
        L = int(rng.integers(1, 40 * S))
        p = B.layout_params(H, 1, S, B_l, s, base, win, dense)
        assert B.s2_kv_resident_blocks(p, h, L) == orc.resident_blocks(L, base + h, S, B_l, s, win, bool(dense))


def test_resident_blocks_errors():
    lib = B.lib()
    p = B.layout_params(4, 1, 64, 2, 4)
    n = C.c_int32(-1)
    buf = (C.c_int32 * 2)()
    assert lib.s2_kv_resident_blocks(None, 0, 10, buf, 2, C.byref(n)) == -1
    assert lib.s2_kv_resident_blocks(C.byref(p), 0, 10, buf, 2, None) == -1
    assert lib.s2_kv_resident_blocks(C.byref(p), 0, 10, None, 2, C.byref(n)) == -1
    assert lib.s2_kv_resident_blocks(C.byref(p), 4, 10, buf, 2, C.byref(n)) == -2   # head out of range
    assert lib.s2_kv_resident_blocks(C.byref(p), -1, 10, buf, 2, C.byref(n)) == -2
    assert lib.s2_kv_resident_blocks(C.byref(p), 0, 0, buf, 2, C.byref(n)) == -2    # length < 1
    bad = B.layout_params(4, 1, 8, 2, 4)
    assert lib.s2_kv_resident_blocks(C.byref(bad), 0, 10, buf, 2, C.byref(n)) == -2
    # capacity too small: count still reported, first entries written
    assert lib.s2_kv_resident_blocks(C.byref(p), 0, 64 * 8, buf, 2, C.byref(n)) == -8
    assert n.value == 4 and list(buf) == [0, 4]
    assert lib.s2_kv_resident_blocks(C.byref(p), 0, 64 * 8, None, 0, C.byref(n)) == -8 and n.value == 4


def test_paged_decode_argument_errors_without_launch():
    lib = B.lib()
    p = B.layout_params(2, 1, 64, 2, 4)
    a = B.PagedDecodeArgs()
    assert lib.s2_attn_decode_paged(None, C.byref(a), 1.0, None, 0, None) == -1
    assert lib.s2_attn_decode_paged(C.byref(p), C.byref(a), 1.0, None, 0, None) == -1   # NULL tensors
    for f in ("q", "k_pages", "v_pages", "block_table", "seq_lens", "o"):
        setattr(a, f, 4096)
    a.nseq, a.heads, a.head_dim, a.max_blocks, a.num_pages = 1, 2, 64, 4, 8
    a.page_stride, a.tok_stride = 64 * 64, 64
    assert lib.s2_attn_decode_paged(C.byref(p), C.byref(a), 0.0, None, 0, None) == -2   # scale
    a.heads = 3
    assert lib.s2_attn_decode_paged(C.byref(p), C.byref(a), 1.0, None, 0, None) == -3   # heads differ
    a.heads, a.head_dim = 2, 96
    assert lib.s2_attn_decode_paged(C.byref(p), C.byref(a), 1.0, None, 0, None) == -3
    a.head_dim, a.tok_stride = 64, 60
    assert lib.s2_attn_decode_paged(C.byref(p), C.byref(a), 1.0, None, 0, None) == -4   # stride
    a.tok_stride, a.q = 64, 4100
    assert lib.s2_attn_decode_paged(C.byref(p), C.byref(a), 1.0, None, 0, None) == -4   # alignment
    a.q, a.num_splits = 4096, 65
    assert lib.s2_attn_decode_paged(C.byref(p), C.byref(a), 1.0, None, 0, None) == -2
    a.num_splits = 0
    assert lib.s2_attn_decode_paged(C.byref(p), C.byref(a), 1.0, None, 0, None) == -5   # workspace


def _random_causal_mask(rng, H, Bk, density):
    M = np.tril(rng.random((H, Bk, Bk)) < density)
    i = np.arange(Bk)
    M[:, i, i] = True
    return M


def test_layout_from_csr_round_trip_and_transpose():
    # caller-supplied patterns: the library must hand back the same rows and the exact transpose
    rng = np.random.default_rng(21)
    masks = [orc.with_sink(orc.block_mask(4, 24, 3, 4), 2),
             orc.homogeneous_mask(3, 17, 2, 5, offset=3),
             orc.block_mask(2, 9, 4, 0)]
    masks += [_random_causal_mask(rng, int(rng.integers(1, 6)), int(rng.integers(1, 40)), float(rng.random()))
              for _ in range(40)]
    for M in masks:
        H, Bk, _ = M.shape
        assert orc.valid_custom_mask(M)
        row_ptr, col_idx, col_ptr, row_idx = orc.compressed_layout(M)
        for S in (32, 64, 128):
            lay = B.s2_layout_from_csr(H, Bk, S, row_ptr, col_idx)
            got = B.s2_layout_get(lay)
            assert got["nnz"] == int(M.sum()) and got["block_size"] == S
            for name, want in (("row_ptr", row_ptr), ("col_idx", col_idx), ("col_ptr", col_ptr),
                               ("row_idx", row_idx)):
                assert np.array_equal(got[name], want), name
            assert got["covers_all"] == int(orc.covers_all(M))
            assert got["max_row_blocks"] == int(M.sum(axis=2).max())
            B.s2_layout_destroy(lay)


def test_layout_from_csr_rejects_bad_rows():
    lib = B.lib()
    out = C.c_void_p()
    arr = lambda xs: (C.c_int32 * len(xs))(*xs)
    call = lambda H, Bk, S, rp, ci: lib.s2_layout_from_csr(H, Bk, S, arr(rp), arr(ci), C.byref(out))
    good_rp, good_ci = [0, 1, 3, 5], [0, 0, 1, 0, 2]      # 1 head, 3 blocks
    assert call(1, 3, 64, good_rp, good_ci) == 0
    lib.s2_layout_destroy(out)
    assert lib.s2_layout_from_csr(1, 3, 64, None, arr(good_ci), C.byref(out)) == -1
    assert lib.s2_layout_from_csr(1, 3, 64, arr(good_rp), None, C.byref(out)) == -1
    assert lib.s2_layout_from_csr(1, 3, 64, arr(good_rp), arr(good_ci), None) == -1
    assert call(0, 3, 64, good_rp, good_ci) == -2
    assert call(1, 0, 64, good_rp, good_ci) == -2
    assert call(1, 3, 48, good_rp, good_ci) == -2
    assert call(1, 3, 64, [1, 2, 4, 6], good_ci + [0]) == -2        # row_ptr[0] != 0
    assert call(1, 3, 64, [0, 1, 1, 3], [0, 0, 2]) == -2            # empty row
    assert call(1, 3, 64, [0, 1, 3, 5], [0, 1, 1, 0, 2]) == -2      # not strictly ascending
    assert call(1, 3, 64, [0, 1, 3, 5], [0, 0, 2, 0, 2]) == -2      # above the diagonal
    assert call(1, 3, 64, [0, 1, 3, 4], [0, 0, 1, 1]) == -2         # diagonal missing in row 2
    assert call(1, 3, 64, [0, 1, 3, 5], [0, 0, 1, -1, 2]) == -2     # negative column


def test_layout_resident_blocks_bit_exact_against_the_oracle():
    # the scan of the layout's later rows, for arbitrary patterns and for the section 4.2 rule
    rng = np.random.default_rng(33)
    masks = [_random_causal_mask(rng, 3, int(Bk), float(d)) for Bk, d in ((1, 0.5), (7, 0.3), (20, 0.1), (16, 0.9))]
    masks.append(orc.with_sink(orc.block_mask(4, 24, 3, 4), 2))
    for M in masks:
        H, Bk, _ = M.shape
        row_ptr, col_idx, _, _ = orc.compressed_layout(M)
        for S in (16, 64) if Bk % 2 == 0 else (64,):
            lay = B.s2_layout_from_csr(H, Bk, S, row_ptr, col_idx)
            for h in range(H):
                for L in sorted(x for x in {1, S - 1, S, S + 1, (Bk * S) // 2, Bk * S - 1, Bk * S} if 1 <= x <= Bk * S):
                    assert B.s2_layout_resident_blocks(lay, h, L) == orc.resident_blocks_mask(M[h], L, S), (h, L, S)
    # a layout built from the rule: same answer as the closed-form helper away from the layout's end
    p = B.layout_params(4, 64, 32, 3, 5)
    lay = B.s2_layout_build(p)
    for h in range(4):
        for L in (1, 32, 33, 500, 1024):
            assert B.s2_layout_resident_blocks(lay, h, L) == B.s2_kv_resident_blocks(p, h, L)


def test_layout_decode_errors_without_launch():
    lib = B.lib()
    lay = B.s2_layout_build(B.layout_params(2, 8, 64, 2, 4))
    n = C.c_int32(-1)
    buf = (C.c_int32 * 2)()
    assert lib.s2_layout_resident_blocks(None, 0, 10, buf, 2, C.byref(n)) == -1
    assert lib.s2_layout_resident_blocks(lay.handle, 0, 10, buf, 2, None) == -1
    assert lib.s2_layout_resident_blocks(lay.handle, 0, 10, None, 2, C.byref(n)) == -1
    assert lib.s2_layout_resident_blocks(lay.handle, 2, 10, buf, 2, C.byref(n)) == -2
    assert lib.s2_layout_resident_blocks(lay.handle, 0, 0, buf, 2, C.byref(n)) == -2
    assert lib.s2_layout_resident_blocks(lay.handle, 0, 8 * 64 + 1, buf, 2, C.byref(n)) == -2   # beyond the layout
    assert lib.s2_layout_resident_blocks(lay.handle, 0, 8 * 64, buf, 1, C.byref(n)) == -8 and n.value >= 2
    a = B.DecodeArgs(4096, 4096, 4096, 4096, 4096, None, 1, 2, 128, 8 * 64 + 1, 1, 1024, 512, 128)
    assert lib.s2_attn_decode_layout(None, C.byref(a), 1.0, None, 0, None) == -1
    assert lib.s2_attn_decode_layout(lay.handle, None, 1.0, None, 0, None) == -1
    assert lib.s2_attn_decode_layout(lay.handle, C.byref(a), 1.0, None, 0, None) == -3         # cache longer than layout
    a.heads = 3
    a.max_len = 64
    assert lib.s2_attn_decode_layout(lay.handle, C.byref(a), 1.0, None, 0, None) == -3         # head count
    pa = B.PagedDecodeArgs(4096, 4096, 4096, 4096, 4096, 4096, None, None, 1, 2, 128, 9, 4, 1, 64 * 128, 128)
    assert lib.s2_attn_decode_paged_layout(None, C.byref(pa), 1.0, None, 0, None) == -1
    assert lib.s2_attn_decode_paged_layout(lay.handle, C.byref(pa), 1.0, None, 0, None) == -3   # 9 blocks > 8


def test_varlen_forward_argument_errors_without_launch():
    lib = B.lib()
    lay = B.s2_layout_build(B.layout_params(2, 8, 64, 2, 4))
    t = _tensors(batch=1, heads=2, seqlen=700)
    call = lambda t, cu=4096, n=3, mx=512: lib.s2_attn_fwd_varlen(lay.handle, C.byref(t), cu, n, mx, 1.0, None)
    assert lib.s2_attn_fwd_varlen(None, C.byref(t), 4096, 3, 512, 1.0, None) == -1
    assert call(t, cu=None) == -1
    assert call(_tensors(batch=2, heads=2, seqlen=700)) == -3      # packed batches have batch 1
    assert call(_tensors(batch=1, heads=3, seqlen=700)) == -3      # head count
    assert call(t, n=0) == -3 and call(t, mx=0) == -3
    assert call(t, mx=8 * 64 + 1) == -3                            # longer than the layout
    assert call(t, cu=4098) == -4                                  # misaligned int32 pointer
    import torch
    if not torch.cuda.is_available():
        assert call(t) == -7                                       # a host-only layout refuses to launch


def test_block_count_limits_of_the_tile_lists():
    # tile-list entries keep the partner index in 15 bits: 32768 blocks, or 65536 16-token ones
    lib = B.lib()
    out = C.c_void_p()
    ok = B.layout_params(1, 32768, 64, 1, 0)
    assert lib.s2_layout_build(C.byref(ok), C.byref(out)) == 0
    lib.s2_layout_destroy(out)
    too_many = B.layout_params(1, 32769, 64, 1, 0)
    assert lib.s2_layout_build(C.byref(too_many), C.byref(out)) == -8
    ok16 = B.layout_params(1, 65536, 16, 1, 0)
    assert lib.s2_layout_build(C.byref(ok16), C.byref(out)) == 0
    lib.s2_layout_destroy(out)
    too_many16 = B.layout_params(1, 65538, 16, 1, 0)
    assert lib.s2_layout_build(C.byref(too_many16), C.byref(out)) == -8


def test_varlen_backward_argument_errors_without_launch():
    lib = B.lib()
    lay = B.s2_layout_build(B.layout_params(2, 8, 64, 2, 4))
    t = _tensors(batch=1, heads=2, seqlen=700)
    need = lib.s2_attn_bwd_varlen_workspace_bytes(2, 700, 128)
    assert need >= 2 * (2 * 700 + 64) * 4 and need % 256 == 0
    assert lib.s2_attn_bwd_varlen_workspace_bytes(0, 700, 128) == 0
    call = lambda t, cu=4096, n=3, mx=512, ws=256, nbytes=need: lib.s2_attn_bwd_varlen(
        lay.handle, C.byref(t), cu, n, mx, 1.0, ws, nbytes, None)
    assert lib.s2_attn_bwd_varlen(None, C.byref(t), 4096, 3, 512, 1.0, 256, need, None) == -1
    assert call(t, cu=None) == -1
    assert call(_tensors(batch=1, heads=2, seqlen=700, dq=None)) == -1
    assert call(_tensors(batch=2, heads=2, seqlen=700)) == -3
    assert call(t, mx=8 * 64 + 1) == -3
    assert call(t, ws=None) == -5 and call(t, nbytes=need - 1) == -5 and call(t, ws=264) == -5
    import torch
    if not torch.cuda.is_available():
        assert call(t) == -7


def _mask_from_tiles(lay, which, H, Bk):
    """Rebuilds the block mask from one of the kernels' work lists, checking its shape on the way."""
    t = B.s2_layout_get_tiles(lay, which)
    T, G, sub = t["tiles_per_head"], t["group"], t["blocks_per_unit"]
    cols = which == B.TILES_DKDV
    M = np.zeros((H, Bk, Bk), dtype=bool)
    seen_members = [set() for _ in range(H)]
    for h in range(H):
        lens = []
        for tile in range(T):
            lo, hi = int(t["ptr"][h * T + tile]), int(t["ptr"][h * T + tile + 1])
            lens.append(hi - lo)
            mem = t["members"][(h * T + tile) * G:(h * T + tile + 1) * G] if len(t["members"]) else None
            members = [int(m) for m in mem] if cols else [tile * G + r if tile * G + r < Bk else -1 for r in range(G)]
            if cols:
                seen_members[h].update(m for m in members if m >= 0)
                if sub > 1:    # a wavefront's 32 key rows span two members: they must be adjacent columns
                    real = [m for m in members if m >= 0]
                    assert real == list(range(real[0], real[0] + len(real)))
            units = [int(e) >> 16 for e in t["ent"][lo:hi]]
            if cols:
                # descending, or (an unbroken run of n rows shared by many equal tiles) descending from the
                # row that is a multiple of n, wrapping round to the run's last row
                want = sorted(set(units), reverse=True)
                n = len(units)
                if units != want:
                    assert n >= 2 and want[0] - want[-1] == n - 1, "only an unbroken run is rotated"
                    k = want[0] - (want[0] // n) * n
                    assert units == want[k:] + want[:k], "rotated to start at a multiple of its length"
                    assert lens.count(n) + sum(1 for tt in range(tile + 1, T) if int(t["ptr"][h * T + tt + 1]) - int(t["ptr"][h * T + tt]) == n) >= 8
            else:
                assert units == sorted(set(units)), "partners strictly ascending, none twice"
            for e in t["ent"][lo:hi]:
                unit, bits = int(e) >> 16, int(e) & 0xFFFF
                assert bits != 0 and bits < (1 << (G * sub))
                for r in range(G):
                    for c in range(sub):
                        if (bits >> (r * sub + c)) & 1:
                            assert members[r] >= 0
                            partner = unit * sub + c
                            i, j = (partner, members[r]) if cols else (members[r], partner)
                            assert not M[h, i, j], "a block listed twice"
                            M[h, i, j] = True
        order = [int(x) for x in t["order"][h * T:(h + 1) * T]]
        assert sorted(order) == list(range(T))
        assert [lens[x] for x in order] == sorted(lens, reverse=True), "longest tiles first"
        if cols:
            assert seen_members[h] == set(range(Bk)), "every column belongs to exactly one key tile"
    return M


@pytest.mark.parametrize("S", [16, 32, 64, 128])
def test_work_lists_hold_exactly_the_mask(S):
    # the lists the three kernels walk (merged query tiles, merged key tiles) against the oracle's
    # mask, for the rule and for arbitrary patterns, every block size
    rng = np.random.default_rng(40 + S)
    cases = [orc.block_mask(5, 24, 3, 4), orc.block_mask(3, 10, 1, 0), orc.with_sink(orc.block_mask(2, 18, 2, 7), 1),
             orc.block_mask(2, 64, 4, 8)]
    cases += [_random_causal_mask(rng, int(rng.integers(1, 5)), 2 * int(rng.integers(1, 20)), float(rng.random()))
              for _ in range(6)]
    for M in cases:
        H, Bk, _ = M.shape
        row_ptr, col_idx, _, _ = orc.compressed_layout(M)
        lay = B.s2_layout_from_csr(H, Bk, S, row_ptr, col_idx)
        for which in (B.TILES_FWD, B.TILES_DQ, B.TILES_DKDV):
            assert np.array_equal(_mask_from_tiles(lay, which, H, Bk), M), (S, which)
    lay = B.s2_layout_build(B.layout_params(4, 32, S, 3, 5, 2))
    want = orc.block_mask(4, 32, 3, 5, 2)
    for which in (B.TILES_FWD, B.TILES_DQ, B.TILES_DKDV):
        assert np.array_equal(_mask_from_tiles(lay, which, 4, 32), want)
    v = B.TileView()
    assert B.lib().s2_layout_get_tiles(lay.handle, 3, C.byref(v)) == -2
    assert B.lib().s2_layout_get_tiles(None, 0, C.byref(v)) == -1


@pytest.mark.parametrize("S", [64, 128])
def test_ds_unit_table(S):
    # the backward that keeps dS: every 64 x 64 piece of a kept block that holds a causal pair has one
    # unit of its own among the steps of the dK/dV lists, and the dQ lists find exactly those units
    rng = np.random.default_rng(70 + S)
    cases = [orc.block_mask(5, 24, 3, 4), orc.block_mask(2, 64, 4, 8), orc.block_mask(3, 11, 1, 0),
             orc.with_sink(orc.block_mask(2, 18, 2, 7), 1)]
    cases += [_random_causal_mask(rng, int(rng.integers(1, 5)), int(rng.integers(1, 40)), float(rng.random()))
              for _ in range(6)]
    sub = S // 64
    for M in cases:
        H, Bk, _ = M.shape
        row_ptr, col_idx, _, _ = orc.compressed_layout(M)
        lay = B.s2_layout_from_csr(H, Bk, S, row_ptr, col_idx)
        kv, dq = B.s2_layout_get_tiles(lay, B.TILES_DKDV), B.s2_layout_get_tiles(lay, B.TILES_DQ)
        view = B.s2_layout_get_ds_units(lay)
        assert view["ds_units"] == 2 * sub * len(kv["ent"])
        assert len(view["dq_units"]) == 2 * sub * len(dq["ent"])
        # the dK/dV walk, as the header describes it
        where = {}
        T, G = kv["tiles_per_head"], kv["group"]
        assert G == 128 // S and dq["group"] == 128 // S
        for h in range(H):
            for t in range(T):
                mem = kv["members"][(h * T + t) * G:(h * T + t + 1) * G]
                for e in range(int(kv["ptr"][h * T + t]), int(kv["ptr"][h * T + t + 1])):
                    ent = int(kv["ent"][e])
                    for c in range(sub):
                        q64 = (ent >> 16) * sub + (sub - 1 - c)
                        for r in range(2):
                            m = r if sub == 1 else 0
                            if mem[m] < 0 or not (ent >> m) & 1:
                                continue
                            k64 = int(mem[m]) if sub == 1 else int(mem[0]) * 2 + r
                            if k64 > q64:
                                continue
                            assert (h, q64, k64) not in where
                            where[(h, q64, k64)] = (e * sub + c) * 2 + r
        assert len(set(where.values())) == len(where) and max(where.values()) < view["ds_units"]
        # every piece of the mask that holds a causal pair, and nothing else
        want = {(h, i * sub + a, j * sub + b) for h, i, j in zip(*np.nonzero(M)) for a in range(sub)
                for b in range(sub) if j * sub + b <= i * sub + a}
        assert set(where) == want
        # the dQ walk finds them
        Tq = dq["tiles_per_head"]
        for h in range(H):
            for t in range(Tq):
                for e in range(int(dq["ptr"][h * Tq + t]), int(dq["ptr"][h * Tq + t + 1])):
                    ent = int(dq["ent"][e])
                    for c in range(sub):
                        k64 = (ent >> 16) * sub + c
                        for m in range(2):
                            q64 = 2 * t + m
                            got = int(view["dq_units"][(e * sub + c) * 2 + m])
                            kept = q64 // sub < Bk and bool(M[h, q64 // sub, k64 // sub]) and k64 <= q64
                            assert got == (where[(h, q64, k64)] if kept else -1), (h, t, e, c, m)
    for S_other in (16, 32):
        lay = B.s2_layout_build(B.layout_params(2, 16, S_other, 2, 4))
        view = B.s2_layout_get_ds_units(lay)
        assert view["ds_units"] == 0 and len(view["dq_units"]) == 0
    v = B.DsUnitsView()
    assert B.lib().s2_layout_get_ds_units(None, C.byref(v)) == -1
    # the workspace that selects the path: the small one plus 8 KiB per unit and batch element, and
    # only the small one where the path does not apply
    lay = B.s2_layout_build(B.layout_params(4, 8, S, 2, 3))
    units = B.s2_layout_get_ds_units(lay)["ds_units"]
    small = B.s2_attn_bwd_workspace_bytes(3, 4, 8 * S, 128)
    assert B.s2_attn_bwd_layout_workspace_bytes(lay, 3, 4, 8 * S, 128) == small + 3 * units * 8192
    assert B.s2_attn_bwd_layout_workspace_bytes(lay, 3, 4, 8 * S, 64) == B.s2_attn_bwd_workspace_bytes(3, 4, 8 * S, 64)
    assert B.s2_attn_bwd_layout_workspace_bytes(lay, 3, 5, 8 * S, 128) == B.s2_attn_bwd_workspace_bytes(3, 5, 8 * S, 128)
    assert B.s2_attn_bwd_layout_workspace_bytes(lay, 3, 4, 4 * S, 128) == B.s2_attn_bwd_workspace_bytes(3, 4, 4 * S, 128)
