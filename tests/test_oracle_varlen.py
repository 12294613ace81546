"""Pins for the oracle's packed variable-length forward (serving prefill batches, section 5.3).  CPU only."""
import numpy as np

from oracle import s2_oracle as O


def _case(seed, H, lens, D):
    rng = np.random.default_rng(seed)
    total = int(sum(lens))
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    q, k, v = (rng.standard_normal((H, total, D)) for _ in range(3))
    return q, k, v, cu


def test_equal_lengths_are_the_batched_forward():
    H, S, D, N = 3, 4, 5, 24
    M = O.block_mask(H, N // S, 2, 3)
    q, k, v, cu = _case(1, H, [N, N, N], D)
    got, got_lse = O.attention_forward_varlen(q, k, v, cu, M, S, 0.3)
    as_batch = lambda x: x.reshape(H, 3, N, D).transpose(1, 0, 2, 3)
    want, want_lse = O.attention_forward(as_batch(q), as_batch(k), as_batch(v), M, S, 0.3)
    assert np.array_equal(as_batch(got), want)
    assert np.array_equal(got_lse.reshape(H, 3, N).transpose(1, 0, 2), want_lse)


def test_ragged_sequence_is_the_prefix_of_a_longer_one():
    # causality: the first L rows of a longer sequence's output do not depend on what follows
    H, S, D = 2, 4, 3
    M = O.block_mask(H, 8, 2, 3)
    lens = [7, 1, 13, 0, 32, 5]
    q, k, v, cu = _case(2, H, lens, D)
    got, got_lse = O.attention_forward_varlen(q, k, v, cu, M, S, 0.5)
    rng = np.random.default_rng(3)
    for s, L in enumerate(lens):
        lo = cu[s]
        for h in range(H):
            pad = lambda x: np.concatenate([x[h, lo:lo + L], rng.standard_normal((32 - L, D))])
            full, full_lse = O.attention_forward_head(pad(q), pad(k), pad(v), M[h], S, 0.5)
            assert np.allclose(got[h, lo:lo + L], full[:L], rtol=0, atol=1e-13)
            assert np.allclose(got_lse[h, lo:lo + L], full_lse[:L], rtol=0, atol=1e-13)


def test_zero_queries_count_kept_keys_per_sequence():
    # Q = 0: LSE = ln(#kept keys) and O = mean of the kept V rows, the kept set spelled out with
    # loops over the sequence's own positions
    H, S, D = 3, 4, 2
    B_l, s = 2, 3
    M = O.block_mask(H, 6, B_l, s)
    lens = [9, 24, 2, 17]
    q, k, v, cu = _case(4, H, lens, D)
    got, got_lse = O.attention_forward_varlen(np.zeros_like(q), k, v, cu, M, S, 1.0)
    for sq, L in enumerate(lens):
        lo = cu[sq]
        for h in range(H):
            for t in range(L):
                kept = [u for u in range(t + 1) if M[h, t // S, u // S]]
                assert abs(got_lse[h, lo + t] - np.log(len(kept))) < 1e-13
                assert np.allclose(got[h, lo + t], v[h, lo:lo + L][kept].mean(axis=0), atol=1e-13)


def test_sequences_do_not_see_each_other_and_unowned_rows_are_nan():
    H, S, D = 2, 4, 3
    M = O.block_mask(H, 4, 1, 2)
    lens = [6, 10]
    q, k, v, cu = _case(5, H, lens, D)
    pad = np.zeros((H, 3, D))
    q, k, v = (np.concatenate([x, pad], axis=1) for x in (q, k, v))
    a, a_lse = O.attention_forward_varlen(q, k, v, cu, M, S, 0.4)
    k2, v2 = k.copy(), v.copy()
    k2[:, :6] += 5.0
    v2[:, :6] -= 3.0
    b, b_lse = O.attention_forward_varlen(q, k2, v2, cu, M, S, 0.4)
    assert np.array_equal(a[:, 6:16], b[:, 6:16]) and np.array_equal(a_lse[:, 6:16], b_lse[:, 6:16])
    assert not np.allclose(a[:, :6], b[:, :6])
    assert np.isnan(a[:, 16:]).all() and np.isnan(a_lse[:, 16:]).all()


def test_backward_equal_lengths_is_the_batched_backward():
    H, S, D, N = 2, 4, 3, 16
    M = O.block_mask(H, N // S, 2, 3)
    q, k, v, cu = _case(6, H, [N, N], D)
    dO = np.random.default_rng(7).standard_normal(q.shape)
    got = O.attention_backward_varlen(q, k, v, dO, cu, M, S, 0.3)
    as_batch = lambda x: x.reshape(H, 2, N, -1).transpose(1, 0, 2, 3)
    want = O.attention_backward(as_batch(q), as_batch(k), as_batch(v), as_batch(dO), M, S, 0.3)
    for g, w_ in zip(got[:4], want[:4]):
        assert np.array_equal(as_batch(g), w_)
    assert np.array_equal(got[4].reshape(H, 2, N).transpose(1, 0, 2), want[4])


def test_backward_ragged_by_finite_differences():
    # the loss sum(O * dO) over a ragged packed batch, differentiated numerically in a few coordinates
    H, S, D = 2, 4, 3
    M = O.block_mask(H, 4, 2, 2)
    lens = [5, 11, 0, 3]
    q, k, v, cu = _case(8, H, lens, D)
    rng = np.random.default_rng(9)
    dO = rng.standard_normal(q.shape)
    dQ, dK, dV, _, _ = O.attention_backward_varlen(q, k, v, dO, cu, M, S, 0.6)
    loss = lambda q_, k_, v_: float((O.attention_forward_varlen(q_, k_, v_, cu, M, S, 0.6)[0] * dO).sum())
    eps = 1e-6
    for name, x, grad in (("q", q, dQ), ("k", k, dK), ("v", v, dV)):
        for _ in range(6):
            h, t, d = int(rng.integers(0, H)), int(rng.integers(0, x.shape[1])), int(rng.integers(0, D))
            xp, xm = x.copy(), x.copy()
            xp[h, t, d] += eps
            xm[h, t, d] -= eps
            args_p = dict(q=q, k=k, v=v); args_m = dict(q=q, k=k, v=v)
            args_p[name], args_m[name] = xp, xm
            num = (loss(args_p["q"], args_p["k"], args_p["v"]) - loss(args_m["q"], args_m["k"], args_m["v"])) / (2 * eps)
            assert abs(num - grad[h, t, d]) < 1e-6 * max(1.0, abs(num)), (name, h, t, d)


def test_backward_sequences_are_isolated():
    H, S, D = 2, 4, 3
    M = O.block_mask(H, 4, 1, 2)
    lens = [6, 10]
    q, k, v, cu = _case(10, H, lens, D)
    dO = np.random.default_rng(11).standard_normal(q.shape)
    a = O.attention_backward_varlen(q, k, v, dO, cu, M, S, 0.4)
    q2, dO2 = q.copy(), dO.copy()
    q2[:, :6] += 1.0
    dO2[:, :6] *= -2.0
    b = O.attention_backward_varlen(q2, k, v, dO2, cu, M, S, 0.4)
    for x, y in zip(a[:3], b[:3]):
        assert np.array_equal(x[:, 6:], y[:, 6:]) and not np.allclose(x[:, :6], y[:, :6])
