"""Pins for the oracle's paged-cache functions (section 4.1: KV-efficient sparsity, eviction of
blocks no later query attends, page-table storage).  CPU only."""
import os

import numpy as np
import pytest

from oracle import s2_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hhst_tiny_rows.txt")


def golden_rows():
    rows = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        key, cols = line.split(":")
        h, i = (int(x) for x in key.replace("h", "").replace("i", "").split())
        rows[(h, i)] = [int(c) for c in cols.split()]
    return rows


def test_golden_file_parses():
    rows = golden_rows()
    assert len(rows) == 32 and rows[(1, 7)] == [1, 5, 6, 7]


def test_resident_set_of_tiny_workload_is_the_hand_derived_row():
    # tiny workload: S=64, B_l=2, s=4, o_h=h.  With L tokens cached the blocks still needed are
    # those of block row (L-1) div S, which the golden file lists by hand.
    rows = golden_rows()
    for h in range(4):
        for i in range(8):
            for L in (64 * i + 1, 64 * i + 17, 64 * (i + 1)):
                assert O.resident_blocks(L, h, 64, 2, 4) == rows[(h, i)]


@pytest.mark.parametrize("seed", range(6))
def test_resident_set_against_a_long_scan_of_future_rows(seed):
    # the definition again with a horizon far beyond anything the parameters could need
    rng = np.random.default_rng(100 + seed)
    for _ in range(25):
        S = int(rng.choice([64, 128]))
        B_l = int(rng.integers(1, 7))
        s = int(rng.integers(0, 9))
        win = int(rng.choice([0, 0, rng.integers(B_l, 40)]))
        g = int(rng.integers(0, 40))
        L = int(rng.integers(1, 30 * S))
        B = -(-L // S)
        i = (L - 1) // S
        o = O.head_offset(g, s)
        want = [j for j in range(B)
                if any(O.block_predicate(ip, j, o, B_l, s, win) for ip in range(i, i + 400))]
        assert O.resident_blocks(L, g, S, B_l, s, win) == want


@pytest.mark.parametrize("seed", range(4))
def test_resident_set_is_the_current_row_when_the_window_is_unbounded(seed):
    # Eq. 1 (KV-efficiency): M[i+1][j] implies M[i][j] for j <= i, so nothing a later row needs is
    # missing from row i; and row i itself needs all of its own blocks.
    rng = np.random.default_rng(200 + seed)
    for _ in range(20):
        B_l = int(rng.integers(1, 9))
        s = int(rng.integers(1, 17))
        H = int(rng.integers(1, 9))
        B = int(rng.integers(1, 60))
        M = O.block_mask(H, B, B_l, s)
        h = int(rng.integers(0, H))
        i = int(rng.integers(0, B))
        L = 64 * i + int(rng.integers(1, 65))
        assert O.resident_blocks(L, h, 64, B_l, s) == [j for j in range(i + 1) if M[h, i, j]]


def test_resident_count_closed_form_and_memory_ratio():
    # local blocks + stripes at or before i - B_l; at the 7B decode shape a head keeps about 1/9
    # of a 32K cache (section 4.1's point)
    for g in (0, 5, 15, 31):
        for L in (8192, 20000, 32768):
            i = (L - 1) // 64
            o = g % 16
            cnt = min(i + 1, 16) + ((i - 16 - o) // 16 + 1 if i - 16 >= o else 0)
            assert len(O.resident_blocks(L, g, 64, 16, 16)) == cnt
    kept = len(O.resident_blocks(32768, 3, 64, 16, 16))
    assert 8.0 < 512 / kept < 11.0


def test_dense_keeps_everything():
    assert O.resident_blocks(1000, 0, 64, 1, 0, dense=True) == list(range(16))


def _case(seed, L, S=64, D=16):
    rng = np.random.default_rng(seed)
    B = -(-L // S)
    k = rng.standard_normal((B * S, D))
    v = rng.standard_normal((B * S, D))
    q = rng.standard_normal(D)
    return q, k, v, B


def _pages_from(cache, B, S, order):
    """Pool where logical block j sits in page order[j]."""
    pool = np.zeros((len(order) + 3, S, cache.shape[1]))
    for j in range(B):
        pool[order[j]] = cache[j * S:(j + 1) * S]
    return pool


@pytest.mark.parametrize("L", [1, 63, 64, 65, 700, 1024])
def test_identity_table_is_the_contiguous_cache(L):
    q, k, v, B = _case(L, L)
    ident = np.arange(B)
    kp, vp = _pages_from(k, B, 64, ident), _pages_from(v, B, 64, ident)
    for g in (0, 1, 3):
        o1, l1 = O.paged_decode_row(q, kp, vp, ident, L, g, 64, 2, 4, 0.25)
        o2, l2 = O.decode_row(q, k, v, L, g, 64, 2, 4, 0.25)
        assert np.array_equal(o1, o2) and l1 == l2


def test_result_does_not_depend_on_where_pages_sit_or_on_evicted_content():
    L, S, B_l, s, g = 1500, 64, 3, 4, 2
    q, k, v, B = _case(7, L)
    ref = O.decode_row(q, k, v, L, g, S, B_l, s, 0.3)
    rng = np.random.default_rng(1)
    order = rng.permutation(B + 3)[:B]
    kp, vp = _pages_from(k, B, S, order), _pages_from(v, B, S, order)
    got = O.paged_decode_row(q, kp, vp, order, L, g, S, B_l, s, 0.3)
    assert np.array_equal(got[0], ref[0]) and got[1] == ref[1]
    # evict everything the head no longer needs: same result
    keep = set(O.resident_blocks(L, g, S, B_l, s))
    table = np.array([order[j] if j in keep else -1 for j in range(B)])
    got = O.paged_decode_row(q, kp, vp, table, L, g, S, B_l, s, 0.3)
    assert np.array_equal(got[0], ref[0]) and got[1] == ref[1]
    assert len(keep) < B
    # blocks the mask drops may point at any page at all
    junk = np.array([order[j] if j in keep else order[0] for j in range(B)])
    got = O.paged_decode_row(q, kp, vp, junk, L, g, S, B_l, s, 0.3)
    assert np.array_equal(got[0], ref[0]) and got[1] == ref[1]


def test_evicting_a_block_that_is_still_needed_shows():
    L, S, B_l, s, g = 900, 64, 2, 4, 1
    q, k, v, B = _case(9, L)
    ident = np.arange(B)
    kp, vp = _pages_from(k, B, S, ident), _pages_from(v, B, S, ident)
    keep = O.resident_blocks(L, g, S, B_l, s)
    for j in keep:
        table = ident.copy()
        table[j] = -1
        o, lse = O.paged_decode_row(q, kp, vp, table, L, g, S, B_l, s, 0.3)
        assert np.isnan(o).all() or np.isnan(lse)


def test_later_steps_never_need_an_evicted_block():
    # decode 200 steps evicting after every step: each step's kept set is within what the
    # previous step left resident (plus the new block), for every head of a 4-head group
    S, B_l, s = 64, 2, 4
    for g in range(4):
        resident = set(O.resident_blocks(1, g, S, B_l, s))
        for L in range(2, 64 * 12):
            i = (L - 1) // S
            need = set(O.resident_blocks(L, g, S, B_l, s))
            assert need <= resident | {i}
            resident = need
