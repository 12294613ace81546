"""Pins for the oracle's floating-point path (CPU only).

Checked against: a brute-force dense causal attention written here with plain
Python loops; literal values worked out by hand on a tiny case; closed forms
that hold when Q = 0 or V = 1; central finite differences for the gradients;
and the decode row against the training-path rows.
"""

import math

import numpy as np
import pytest

from oracle import s2_oracle as orc


# ----------------------------------------------------------------- helpers (independent of the oracle)

def brute_dense_causal(q, k, v, scale):
    """Textbook causal softmax attention, one head, Python loops and math.exp."""
    N, D = len(q), len(q[0])
    Dv = len(v[0])
    O = [[0.0] * Dv for _ in range(N)]
    LSE = [0.0] * N
    for t in range(N):
        z = [scale * sum(q[t][d] * k[u][d] for d in range(D)) for u in range(t + 1)]
        mx = max(z)
        w = [math.exp(x - mx) for x in z]
        tot = sum(w)
        LSE[t] = mx + math.log(tot)
        for u in range(t + 1):
            for d in range(Dv):
                O[t][d] += w[u] / tot * v[u][d]
    return np.array(O), np.array(LSE)


def brute_masked(q, k, v, keep_sets, scale):
    """Softmax attention where row t attends exactly the key indices keep_sets[t]."""
    N = len(q)
    O = np.zeros((N, v.shape[1]))
    LSE = np.zeros(N)
    for t in range(N):
        us = sorted(keep_sets[t])
        z = np.array([scale * float(np.dot(q[t], k[u])) for u in us])
        LSE[t] = math.log(sum(math.exp(x) for x in z))
        w = np.array([math.exp(x - LSE[t]) for x in z])
        for wi, u in zip(w, us):
            O[t] += wi * v[u]
    return O, LSE


def rows_from_golden():
    import os
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "hhst_tiny_rows.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            left, right = line.split(":")
            h, i = (int(x) for x in left.split())
            rows[(h, i)] = [int(x) for x in right.split()]
    return rows


# ----------------------------------------------------------------- pins

def test_all_ones_layout_equals_brute_force_dense_causal():
    rng = np.random.default_rng(0)
    N, D, S = 24, 5, 4
    q, k, v = (rng.standard_normal((N, D)) for _ in range(3))
    scale = 0.37
    Mh = orc.block_mask(1, N // S, 1, 0, dense=True)[0]
    O, LSE = orc.attention_forward_head(q, k, v, Mh, S, scale)
    Ob, LSEb = brute_dense_causal(q.tolist(), k.tolist(), v.tolist(), scale)
    np.testing.assert_allclose(O, Ob, rtol=0, atol=1e-13)
    np.testing.assert_allclose(LSE, LSEb, rtol=0, atol=1e-13)
    # B_l >= B is the same thing reached through the sparse rule
    Mh2 = orc.block_mask(1, N // S, N // S, 3)[0]
    O2, LSE2 = orc.attention_forward_head(q, k, v, Mh2, S, scale)
    np.testing.assert_allclose(O2, Ob, rtol=0, atol=1e-13)


def test_hand_computed_softmax_literals():
    """N=8, S=2, B=4, B_l=1, stride 2: scores are logs of integers, so weights are fractions.

    q_t = (1, 0); k_u = (ln c_u, 7) with c = 1..8; scale 1, so exp(z[t][u]) = c_u.
    v_u = (u, 1 if u even else -1).
    Head 0 (o=0): block row 3 keeps blocks {0, 2, 3}; token 7 keeps keys {0,1,4,5,6,7}
       weights c/sum = (1,2,5,6,7,8)/29.
    Head 1 (o=1): block row 3 keeps blocks {1, 3}; token 6 keeps keys {2,3,6}: (3,4,7)/14.
    Token 1 (block 0, diagonal only, both heads): keys {0,1}: (1,2)/3.
    """
    c = np.arange(1, 9, dtype=np.float64)
    q = np.tile(np.array([1.0, 0.0]), (8, 1))
    k = np.stack([np.log(c), np.full(8, 7.0)], axis=1)
    v = np.stack([np.arange(8.0), np.where(np.arange(8) % 2 == 0, 1.0, -1.0)], axis=1)
    M = orc.block_mask(2, 4, 1, 2)
    O0, L0 = orc.attention_forward_head(q, k, v, M[0], 2, 1.0)
    O1, L1 = orc.attention_forward_head(q, k, v, M[1], 2, 1.0)
    # head 0, token 7
    assert abs(L0[7] - math.log(29.0)) < 1e-14
    assert abs(O0[7, 0] - (0 * 1 + 1 * 2 + 4 * 5 + 5 * 6 + 6 * 7 + 7 * 8) / 29.0) < 1e-14
    assert abs(O0[7, 1] - (1 - 2 + 5 - 6 + 7 - 8) / 29.0) < 1e-14
    # head 1, token 6
    assert abs(L1[6] - math.log(14.0)) < 1e-14
    assert abs(O1[6, 0] - (2 * 3 + 3 * 4 + 6 * 7) / 14.0) < 1e-14
    assert abs(O1[6, 1] - (3 - 4 + 7) / 14.0) < 1e-14
    # token 1 on both heads
    for O, L in ((O0, L0), (O1, L1)):
        assert abs(L[1] - math.log(3.0)) < 1e-14
        assert abs(O[1, 0] - 2.0 / 3.0) < 1e-14
        assert abs(O[1, 1] - (1 - 2) / 3.0) < 1e-14
    # token 0: a single key -> weight 1
    assert O0[0].tolist() == [0.0, 1.0] and abs(L0[0]) < 1e-15


def test_softmax_rows_sum_to_one():
    """With V = 1 every output equals the sum of the row's weights."""
    rng = np.random.default_rng(1)
    H, B, S, D = 4, 8, 8, 16
    N = B * S
    q, k = (rng.standard_normal((1, H, N, D)) for _ in range(2))
    v = np.ones((1, H, N, D))
    M = orc.block_mask(H, B, 2, 4)
    O, _ = orc.attention_forward(q, k, v, M, S, 0.25)
    np.testing.assert_allclose(O, 1.0, rtol=0, atol=1e-14)


def test_zero_query_closed_form_counts_keys():
    """Q = 0: LSE[t] = ln(#kept keys of t) and O[t] = mean of the kept value rows.

    The kept sets come from the hand-derived rows, so every row's active set is
    checked through the numerical path.
    """
    rows = rows_from_golden()
    rng = np.random.default_rng(2)
    H, B, S, D = 4, 8, 4, 6
    N = B * S
    k, v = (rng.standard_normal((1, H, N, D)) for _ in range(2))
    q = np.zeros((1, H, N, D))
    M = orc.block_mask(H, B, 2, 4)
    O, LSE = orc.attention_forward(q, k, v, M, S, 1.0)
    for h in range(H):
        for t in range(N):
            i = t // S
            cols = rows[(h, i)]
            cnt = S * (len(cols) - 1) + (t % S) + 1
            assert abs(LSE[0, h, t] - math.log(cnt)) < 1e-13
            keys = [u for j in cols for u in range(j * S, j * S + S) if u <= t]
            assert len(keys) == cnt
            np.testing.assert_allclose(O[0, h, t], v[0, h, keys].mean(axis=0), rtol=0, atol=1e-13)


def test_sparse_forward_against_explicit_key_sets():
    """Random inputs; key sets built from the hand-derived rows, attention by loops."""
    rows = rows_from_golden()
    rng = np.random.default_rng(3)
    H, B, S, D = 4, 8, 3, 5
    N = B * S
    q, k, v = (rng.standard_normal((1, H, N, D)) for _ in range(3))
    M = orc.block_mask(H, B, 2, 4)
    O, LSE = orc.attention_forward(q, k, v, M, S, 0.6)
    for h in range(H):
        keep = [[u for j in rows[(h, t // S)] for u in range(j * S, j * S + S) if u <= t]
                for t in range(N)]
        Ob, Lb = brute_masked(q[0, h], k[0, h], v[0, h], keep, 0.6)
        np.testing.assert_allclose(O[0, h], Ob, rtol=0, atol=1e-13)
        np.testing.assert_allclose(LSE[0, h], Lb, rtol=0, atol=1e-13)


def test_row_chunking_is_invisible():
    """A sequence longer than the oracle's row chunk gives the same rows as one shot."""
    rng = np.random.default_rng(4)
    S, B, D = 16, 80, 8          # N = 1280 > chunk of 1024
    N = S * B
    q, k, v = (rng.standard_normal((N, D)) for _ in range(3))
    Mh = orc.block_mask(3, B, 3, 5)[2]
    O, LSE = orc.attention_forward_head(q, k, v, Mh, S, 0.3)
    idx = np.array([0, 17, 1023, 1024, 1025, N - 1])
    Or, Lr = orc.forward_rows(q[idx], idx, k, v, Mh, S, 0.3)
    np.testing.assert_allclose(O[idx], Or, rtol=0, atol=1e-13)
    np.testing.assert_allclose(LSE[idx], Lr, rtol=0, atol=1e-13)
    keep = orc.token_mask(Mh, S, N)
    sets = [np.flatnonzero(keep[t]).tolist() for t in idx]
    Ob, Lb = brute_masked(q[idx], k, v, sets, 0.3)
    np.testing.assert_allclose(Or, Ob, rtol=0, atol=1e-12)
    np.testing.assert_allclose(Lr, Lb, rtol=0, atol=1e-12)


def _loss(q, k, v, dO, Mh, S, scale):
    O, _ = orc.attention_forward_head(q, k, v, Mh, S, scale)
    return float((O * dO).sum())


@pytest.mark.parametrize("dense", [False, True])
def test_gradients_by_finite_differences(dense):
    rng = np.random.default_rng(5)
    B, S, D = 6, 3, 4
    N = B * S
    q, k, v, dO = (rng.standard_normal((N, D)) for _ in range(4))
    scale = 0.45
    Mh = orc.block_mask(2, B, 2, 2, dense=dense)[1]
    dQ, dK, dV, O, LSE = orc.attention_backward_head(q, k, v, dO, Mh, S, scale)
    O2, LSE2 = orc.attention_forward_head(q, k, v, Mh, S, scale)
    np.testing.assert_allclose(O, O2, rtol=0, atol=1e-14)
    np.testing.assert_allclose(LSE, LSE2, rtol=0, atol=1e-14)
    eps = 1e-6
    for name, arr, grad in (("q", q, dQ), ("k", k, dK), ("v", v, dV)):
        for t in range(N):
            for d in range(D):
                old = arr[t, d]
                arr[t, d] = old + eps
                lp = _loss(q, k, v, dO, Mh, S, scale)
                arr[t, d] = old - eps
                lm = _loss(q, k, v, dO, Mh, S, scale)
                arr[t, d] = old
                fd = (lp - lm) / (2 * eps)
                assert abs(fd - grad[t, d]) < 2e-8, (name, t, d, fd, grad[t, d])


def test_single_key_rows_have_trivial_gradients():
    """Rows that keep one key have weight 1: dS = 0 there, and dV picks up dO unchanged."""
    rng = np.random.default_rng(6)
    B, D = 8, 3
    q, k, v, dO = (rng.standard_normal((B, D)) for _ in range(4))
    Mh = orc.block_mask(1, B, 1, 0)[0]      # one-token blocks, diagonal only
    dQ, dK, dV, O, _ = orc.attention_backward_head(q, k, v, dO, Mh, 1, 1.0)
    assert np.all(dQ == 0.0) and np.all(dK == 0.0)
    np.testing.assert_allclose(dV, dO, atol=1e-15)
    np.testing.assert_allclose(O, v, atol=1e-15)
    # two-token diagonal blocks: the first token of each block still keeps one key
    N = 16
    q, k, v, dO = (rng.standard_normal((N, D)) for _ in range(4))
    dQ, dK, dV, _, _ = orc.attention_backward_head(q, k, v, dO, Mh, 2, 1.0)
    assert np.all(dQ[0::2] == 0.0)
    assert np.any(dQ[1::2] != 0.0)


def test_batched_wrappers_match_per_head():
    rng = np.random.default_rng(8)
    Bt, H, B, S, D = 2, 3, 4, 4, 4
    N = B * S
    q, k, v, dO = (rng.standard_normal((Bt, H, N, D)) for _ in range(4))
    M = orc.block_mask(H, B, 1, 3)
    O, LSE = orc.attention_forward(q, k, v, M, S, 0.5)
    dQ, dK, dV, O2, LSE2 = orc.attention_backward(q, k, v, dO, M, S, 0.5)
    assert np.array_equal(O, O2) and np.array_equal(LSE, LSE2)
    for b in range(Bt):
        for h in range(H):
            sets = [np.flatnonzero(r).tolist() for r in orc.token_mask(M[h], S, N)]
            Ob, Lb = brute_masked(q[b, h], k[b, h], v[b, h], sets, 0.5)
            np.testing.assert_allclose(O[b, h], Ob, atol=1e-13)
            np.testing.assert_allclose(LSE[b, h], Lb, atol=1e-13)


@pytest.mark.parametrize("L", [1, 5, 16, 17, 31, 40])
def test_decode_row_equals_last_training_row(L):
    """Decoding at length L = row L-1 of masked attention over the first L tokens (partial last block)."""
    rng = np.random.default_rng(9)
    S, D, H = 4, 8, 3
    B_l, s = 2, 3
    cap = 48
    kc = rng.standard_normal((H, cap, D))
    vc = rng.standard_normal((H, cap, D))
    qs = rng.standard_normal((H, L, D))       # only the last row is the decode query
    B = (L + S - 1) // S
    M = orc.block_mask(H, B, B_l, s, head_index_base=2)
    for h in range(H):
        O, LSE = orc.attention_forward_head(qs[h], kc[h, :L], vc[h, :L], M[h], S, 0.35)
        o, lse = orc.decode_row(qs[h, L - 1], kc[h], vc[h], L, 2 + h, S, B_l, s, 0.35)
        np.testing.assert_allclose(o, O[L - 1], rtol=0, atol=1e-14)
        assert abs(lse - LSE[L - 1]) < 1e-14
