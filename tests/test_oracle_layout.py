"""Pins for the oracle's integer layout (CPU only).

Every check here compares the oracle with something other than itself: rows
worked out by hand from section 4.2, a closed-form row count derived
separately from the predicate, the invariants the paper states (union of
heads covers the context; Eq. 1, KV-efficiency), and the loose figures the
paper prints.
"""

import os

import numpy as np
import pytest

from oracle import s2_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_rows():
    rows = {}
    with open(os.path.join(GOLDEN, "hhst_tiny_rows.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            left, right = line.split(":")
            h, i = (int(x) for x in left.split())
            rows[(h, i)] = [int(x) for x in right.split()]
    return rows


def _read_figures():
    out = {}
    with open(os.path.join(GOLDEN, "paper_figures.txt")) as f:
        for line in f:
            line = line.split("--")[0].strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split()
            out[k] = float(v)
    return out


def test_worked_example_rows():
    """Section 4.2's mask on B=8, B_l=2, s=4, o_h=h, against the hand-derived rows."""
    rows = _read_rows()
    M = orc.block_mask(4, 8, 2, 4)
    assert len(rows) == 32
    for (h, i), cols in rows.items():
        assert np.flatnonzero(M[h, i]).tolist() == cols, (h, i)
    assert int(M.sum()) == 81
    assert [int(M[h].sum()) for h in range(4)] == [23, 21, 19, 18]


def test_compressed_layout_matches_rows():
    rows = _read_rows()
    M = orc.block_mask(4, 8, 2, 4)
    row_ptr, col_idx, col_ptr, row_idx = orc.compressed_layout(M)
    assert row_ptr[0] == 0 and row_ptr[-1] == 81 and col_ptr[-1] == 81
    for (h, i), cols in rows.items():
        a, b = row_ptr[h * 8 + i], row_ptr[h * 8 + i + 1]
        assert col_idx[a:b].tolist() == cols
    # CSC is the transpose: rebuild the dense mask from it.
    M2 = np.zeros_like(M)
    for h in range(4):
        for j in range(8):
            a, b = col_ptr[h * 8 + j], col_ptr[h * 8 + j + 1]
            r = row_idx[a:b]
            assert np.all(np.diff(r) > 0)
            M2[h, r, j] = True
    assert np.array_equal(M, M2)


def _closed_form_count(i, o_h, B_l, s):
    """Blocks in row i: the local run plus the stripe columns at or before i-B_l."""
    n = min(i + 1, B_l)
    if s > 0 and i - B_l >= o_h:
        n += (i - B_l - o_h) // s + 1
    return n


@pytest.mark.parametrize("H,B,B_l,s,nnz", [
    (4, 8, 2, 4, 81),
    (16, 128, 4, 8, 23596),
    (32, 512, 16, 16, 504816),
    (32, 1024, 8, 32, 777884),
    (16, 128, 1, 15, 10779),
])
def test_row_counts_closed_form(H, B, B_l, s, nnz):
    """Row sums equal a count derived by reasoning about the pattern, not by the predicate."""
    M = orc.block_mask(H, B, B_l, s)
    total = 0
    for h in range(H):
        o_h = h % s
        got = M[h].sum(axis=1)
        want = [_closed_form_count(i, o_h, B_l, s) for i in range(B)]
        assert got.tolist() == want
        total += sum(want)
    assert total == nnz == int(M.sum())


def test_row_sets_closed_form_random():
    """Active set of row i = stripe columns {o_h + k s <= i - B_l} plus the local run."""
    rng = np.random.default_rng(7)
    for _ in range(40):
        H = int(rng.integers(1, 9))
        B = int(rng.integers(1, 40))
        B_l = int(rng.integers(1, 8))
        s = int(rng.integers(0, 10))
        base = int(rng.integers(0, 5))
        win = int(rng.choice([0, 0, rng.integers(1, 40)]))
        M = orc.block_mask(H, B, B_l, s, head_index_base=base, window_blocks=win)
        for h in range(H):
            o_h = (base + h) % s if s > 0 else 0
            for i in range(B):
                want = set(range(max(0, i - B_l + 1), i + 1))
                if s > 0:
                    j = o_h
                    while j <= i - B_l:
                        if win == 0 or i - j < win:
                            want.add(j)
                        j += s
                assert set(np.flatnonzero(M[h, i]).tolist()) == want
                for j in range(B):
                    assert bool(M[h, i, j]) == orc.block_predicate(i, j, o_h, B_l, s, win)


@pytest.mark.parametrize("H,s,expect", [(4, 4, True), (8, 4, True), (3, 4, False), (16, 18, False),
                                        (16, 8, True), (1, 1, True)])
def test_union_covers_context_iff_enough_heads(H, s, expect):
    """Section 4.2: heads jointly cover the whole context; section 5.1: not when stride > heads."""
    M = orc.block_mask(H, 48, 2, s)
    assert orc.covers_all(M) == expect


def test_kv_efficiency_eq1():
    """Eq. 1: a key block attended by query block i+1 (i >= j) is also attended by block i."""
    for (H, B, B_l, s) in [(4, 8, 2, 4), (16, 64, 4, 8), (5, 37, 3, 7), (2, 20, 1, 1)]:
        M = orc.block_mask(H, B, B_l, s)
        for h in range(H):
            for j in range(B):
                col = M[h, j:, j]                 # rows i = j .. B-1
                assert col[0]                     # diagonal always kept
                # once a column drops out it never comes back: "vertical lines"
                assert np.all(col[1:] <= col[:-1])
                for i in range(j, B - 1):
                    if M[h, i + 1, j]:
                        assert M[h, i, j], (h, i, j)


def test_heads_balanced():
    """Section 4.2: every head attends an (almost) equal number of blocks."""
    for (H, B, B_l, s, lo, hi) in [(16, 128, 4, 8, 1421, 1530), (32, 512, 16, 16, 15543, 16008)]:
        per_head = orc.block_mask(H, B, B_l, s).sum(axis=(1, 2))
        assert per_head.min() == lo and per_head.max() == hi
        assert (per_head.max() - per_head.min()) / per_head.mean() < 0.08


def test_dense_and_window_and_swa():
    B = 12
    tril = np.tril(np.ones((B, B), dtype=bool))
    assert np.array_equal(orc.block_mask(2, B, 3, 4, dense=True)[1], tril)
    assert np.array_equal(orc.block_mask(1, B, B, 4)[0], tril)          # B_l >= B is dense
    swa = orc.block_mask(1, B, 3, 0)[0]                                  # no stripes
    i, j = np.indices((B, B))
    assert np.array_equal(swa, (i - j >= 0) & (i - j < 3))
    win = orc.block_mask(1, B, 2, 1, window_blocks=5)[0]                 # every column a stripe
    assert np.array_equal(win, (i - j >= 0) & (i - j < 5))


def test_paper_printed_figures():
    fig = _read_figures()
    # nine local 64-token shards
    M = orc.block_mask(1, 32, 9, 0)
    assert int(M[0, 20].sum()) * 64 == fig["local9_tokens"]
    # 1.3B / 8K workload: block density relative to dense causal ~ 18 %
    M = orc.block_mask(16, 128, 4, 8)
    dens = M.sum() / (16 * 128 * 129 / 2)
    assert abs(dens - fig["table1_flop_fraction"]) < 0.01
    # 7B shape, 31 local + stride 32, 64-token shards, 128K: pair ratio near the measured speed-up
    H, B, S = 32, 2048, 64
    nnz = sum(_closed_form_count(i, h % 32, 31, 32) for h in range(H) for i in range(B))
    assert nnz == 4051889
    sparse_pairs = (nnz - H * B) * S * S + H * B * S * (S + 1) // 2
    dense_pairs = H * (B * S) * (B * S + 1) // 2
    ratio = dense_pairs / sparse_pairs
    assert 0.9 * fig["speedup_7b"] < ratio < 1.15 * fig["speedup_7b"]
    # Merge-Q example: 8 query shards attending KV_1, merged in pairs -> 4 loads
    assert fig["mergeq_loads_before"] / 2 == fig["mergeq_loads_after"]


def test_token_mask_and_pairs():
    M = orc.block_mask(4, 8, 2, 4)
    S, N = 4, 32
    for h in range(4):
        tm = orc.token_mask(M[h], S, N)
        for t in range(N):
            for u in range(N):
                assert tm[t, u] == (M[h, t // S, u // S] and u <= t)
    nnz = int(M.sum())
    assert orc.unmasked_pairs(M, S, N) == (nnz - 4 * 8) * S * S + 4 * 8 * S * (S + 1) // 2
    # partial last block
    tm = orc.token_mask(orc.block_mask(1, 3, 1, 0)[0], 4, 10)
    assert tm.shape == (10, 10) and tm[9].tolist() == [False] * 8 + [True, True]
