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
