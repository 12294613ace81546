"""Pins for the oracle on masks other than the section 4.2 rule: attention sink, homogeneous heads,
arbitrary per-head patterns (sections 3 and 5.1).  CPU only."""
import numpy as np
import pytest

from oracle import s2_oracle as O


def rows_of(Mh):
    return [list(np.nonzero(r)[0]) for r in Mh]


def test_sink_rows_by_hand():
    # B=6, sliding window of 2 blocks (no stripes), sink of 1 block: worked out by hand
    M = O.with_sink(O.block_mask(1, 6, 2, 0), 1)
    assert rows_of(M[0]) == [[0], [0, 1], [0, 1, 2], [0, 2, 3], [0, 3, 4], [0, 4, 5]]
    # sink of 2 on the tiny workload's head 2 (rows from tests/golden: [2,3] -> [0,1,2,3] etc.)
    M = O.with_sink(O.block_mask(4, 8, 2, 4), 2)
    assert rows_of(M[2])[3:6] == [[0, 1, 2, 3], [0, 1, 2, 3, 4], [0, 1, 2, 4, 5]]
    assert O.valid_custom_mask(M)
    # sink never reaches above the diagonal
    assert rows_of(O.with_sink(O.block_mask(1, 3, 1, 0), 5)[0]) == [[0], [0, 1], [0, 1, 2]]


def test_homogeneous_heads_are_identical_and_incomplete():
    M = O.homogeneous_mask(4, 16, 2, 4, offset=1)
    for h in range(1, 4):
        assert np.array_equal(M[h], M[0])
    assert np.array_equal(M[0], O.block_mask(4, 16, 2, 4)[1])
    # same shards for all heads: the union cannot cover the context (section 5.1's point)
    assert not O.covers_all(M)
    assert O.covers_all(O.block_mask(4, 16, 2, 4))


def test_valid_custom_mask():
    M = O.block_mask(2, 5, 2, 2)
    assert O.valid_custom_mask(M)
    bad = M.copy(); bad[0, 1, 3] = True
    assert not O.valid_custom_mask(bad)
    bad = M.copy(); bad[1, 2, 2] = False
    assert not O.valid_custom_mask(bad)


def random_mask(rng, H, B, density):
    M = np.tril(rng.random((H, B, B)) < density)
    i = np.arange(B)
    M[:, i, i] = True
    return M


@pytest.mark.parametrize("seed", range(3))
def test_zero_queries_count_the_kept_keys_of_an_arbitrary_mask(seed):
    # Q = 0 makes every kept score 0: LSE = ln(#kept keys), O = mean of the kept V rows.  The count
    # comes from the mask alone: S per kept off-diagonal block, t mod S + 1 on the diagonal.
    rng = np.random.default_rng(seed)
    H, B, S, D = 3, 7, 4, 5
    M = random_mask(rng, H, B, 0.4)
    N = B * S
    q = np.zeros((1, H, N, D))
    k = rng.standard_normal((1, H, N, D))
    v = rng.standard_normal((1, H, N, D))
    o, lse = O.attention_forward(q, k, v, M, S, 0.7)
    for h in range(H):
        for t in range(N):
            i = t // S
            cnt = S * (int(M[h, i].sum()) - 1) + (t % S) + 1
            assert abs(lse[0, h, t] - np.log(cnt)) < 1e-12
            keys = [u for u in range(t + 1) if M[h, i, u // S]]
            assert len(keys) == cnt
            assert np.allclose(o[0, h, t], v[0, h, keys].mean(axis=0), atol=1e-12)


def test_arbitrary_mask_against_loops_and_finite_differences():
    rng = np.random.default_rng(5)
    H, B, S, D = 2, 4, 3, 4
    M = random_mask(rng, H, B, 0.5)
    N = B * S
    q, k, v, g = (rng.standard_normal((1, H, N, D)) for _ in range(4))
    scale = 0.6
    o, lse = O.attention_forward(q, k, v, M, S, scale)
    # brute force with Python loops
    for h in range(H):
        for t in range(N):
            keys = [u for u in range(t + 1) if M[h, t // S, u // S]]
            z = np.array([scale * float(q[0, h, t] @ k[0, h, u]) for u in keys])
            p = np.exp(z - z.max()); p /= p.sum()
            ref = sum(pi * v[0, h, u] for pi, u in zip(p, keys))
            assert np.allclose(o[0, h, t], ref, atol=1e-12)
    dq, dk, dv, _, _ = O.attention_backward(q, k, v, g, M, S, scale)
    loss = lambda q_, k_, v_: float((O.attention_forward(q_, k_, v_, M, S, scale)[0] * g).sum())
    eps = 1e-6
    for (arr, grad, which) in ((q, dq, 0), (k, dk, 1), (v, dv, 2)):
        for _ in range(6):
            idx = tuple(int(rng.integers(0, n)) for n in arr.shape)
            ap, am = arr.copy(), arr.copy()
            ap[idx] += eps; am[idx] -= eps
            args_p = [q, k, v]; args_m = [q, k, v]
            args_p[which] = ap; args_m[which] = am
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - grad[idx]) < 1e-6 * max(1.0, abs(fd))


# ---- decode and eviction under an arbitrary mask -------------------------------------------------

def test_decode_row_mask_agrees_with_the_closed_form_decode_on_the_hhst_mask():
    # decode_row evaluates section 4.2's predicate token by token; decode_row_mask takes a row of
    # the forward under the materialised mask: two routes to the same definition
    rng = np.random.default_rng(5)
    H, B, S, D, B_l, s = 3, 9, 4, 6, 2, 3
    M = O.block_mask(H, B, B_l, s)
    k = rng.standard_normal((B * S, D))
    v = rng.standard_normal((B * S, D))
    q = rng.standard_normal(D)
    for h in range(H):
        for L in (1, 4, 5, 17, 35, 36):
            a, la = O.decode_row_mask(q, k, v, L, M[h], S, 0.4)
            b, lb = O.decode_row(q, k, v, L, h, S, B_l, s, 0.4)
            assert np.allclose(a, b, rtol=0, atol=1e-13) and abs(la - lb) < 1e-13


def test_decode_row_mask_zero_query_counts_keys():
    rng = np.random.default_rng(6)
    B, S, D = 6, 4, 3
    Mh = random_mask(rng, 1, B, 0.5)[0]
    v = rng.standard_normal((B * S, D))
    k = rng.standard_normal((B * S, D))
    for L in (1, 3, 4, 9, 24):
        i = (L - 1) // S
        toks = [u for u in range(L) if Mh[i, u // S]]
        o, lse = O.decode_row_mask(np.zeros(D), k, v, L, Mh, S, 1.0)
        assert abs(lse - np.log(len(toks))) < 1e-13
        assert np.allclose(o, v[toks].mean(axis=0), atol=1e-13)


def test_resident_blocks_mask_by_hand():
    # rows: 0:{0} 1:{0,1} 2:{2} 3:{0,3}.  Row 2 does not read block 0, yet row 3 will: it stays
    # (a pattern that is not KV-efficient in section 4.1's sense pays with blocks held but unread)
    Mh = np.zeros((4, 4), dtype=bool)
    for i, cols in enumerate([[0], [0, 1], [2], [0, 3]]):
        Mh[i, cols] = True
    S = 4
    assert O.resident_blocks_mask(Mh, 1, S) == [0]
    assert O.resident_blocks_mask(Mh, 4, S) == [0]
    assert O.resident_blocks_mask(Mh, 5, S) == [0, 1]
    assert O.resident_blocks_mask(Mh, 9, S) == [0, 2]
    assert O.resident_blocks_mask(Mh, 12, S) == [0, 2]
    assert O.resident_blocks_mask(Mh, 13, S) == [0, 3]


def test_resident_blocks_mask_agrees_with_closed_form_far_from_the_end():
    # with enough later rows in the mask, scanning it equals the closed-form scan of the rule
    H, B, S, B_l, s = 4, 40, 8, 3, 5
    M = O.block_mask(H, B, B_l, s)
    for h in range(H):
        for L in (1, 8, 9, 63, 64, 100, 160):
            assert O.resident_blocks_mask(M[h], L, S) == O.resident_blocks(L, h, S, B_l, s)


def test_paged_decode_row_mask_ignores_absent_dropped_blocks_and_flags_absent_kept_ones():
    rng = np.random.default_rng(7)
    B, S, D = 6, 4, 5
    Mh = random_mask(rng, 1, B, 0.4)[0]
    L = 22
    i = (L - 1) // S
    kc = rng.standard_normal((B * S, D))
    vc = rng.standard_normal((B * S, D))
    q = rng.standard_normal(D)
    want, want_lse = O.decode_row_mask(q, kc, vc, L, Mh, S, 0.7)
    kept = [j for j in range(i + 1) if Mh[i, j]]
    table = -np.ones(B, dtype=np.int32)
    perm = rng.permutation(len(kept) + 2)
    for n, j in enumerate(kept):
        table[j] = perm[n]
    kp = rng.standard_normal((len(kept) + 2, S, D))
    vp = rng.standard_normal((len(kept) + 2, S, D))
    for j in kept:
        kp[table[j]] = kc[j * S:(j + 1) * S]
        vp[table[j]] = vc[j * S:(j + 1) * S]
    got, got_lse = O.paged_decode_row_mask(q, kp, vp, table, L, Mh, S, 0.7)
    assert np.allclose(got, want, atol=1e-13) and abs(got_lse - want_lse) < 1e-13
    table[kept[0]] = -1
    got, _ = O.paged_decode_row_mask(q, kp, vp, table, L, Mh, S, 0.7)
    assert np.isnan(got).all()
