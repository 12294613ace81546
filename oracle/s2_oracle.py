"""CPU oracle for head-heterogeneous block-sparse causal attention (S2-Attention / HHST).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
HIP library is checked against.  It shares no code with the library, is never
imported by it, and may be imported only by the tests, the smoke check and the
benchmark's CPU-baseline leg.

Everything is computed in float64 with numpy.  Inputs are ordinary arrays
(the callers pass bf16-representable values widened to float); no
intermediate is rounded.

What each function follows:

* ``head_offset`` / ``block_mask`` - the per-head block mask M^h of the paper's
  section 4.2 (the unnumbered equation defining the "Local" and "Stride"
  cases), evaluated independently for every (h, i, j).
* ``with_sink`` / ``homogeneous_mask`` / ``valid_custom_mask`` - the other
  patterns of section 5.1's comparison (attention sink, same shards for all
  heads) and the conditions any custom per-head pattern (section 3's
  customisation claim) must meet.
* ``compressed_layout`` - the compressed-sparse-row storage of that mask that
  section 3.2 ("Warmup") mentions, produced by scanning the dense mask.
* ``token_mask`` - sharding of N tokens into ceil(N/S) blocks (section 3.2)
  plus causality inside the diagonal block.
* ``attention_forward`` / ``attention_backward`` - softmax attention over the
  kept keys only (section 3.2) and its analytic gradient.
* ``attention_forward_varlen`` / ``attention_backward_varlen`` - forward and
  gradients on a packed batch of sequences of different lengths, each an
  independent problem (serving prefill, section 5.3; packed training batches).
* ``decode_row`` - one decoding step against a cache (section 4.1): the last
  row of the same masked attention.
* ``resident_blocks`` / ``paged_decode_row`` - section 4.1's KV-efficient
  cache: which blocks some later query can still attend (the rest may be
  evicted), and decoding against a cache stored as pages behind a block table.
* ``decode_row_mask`` / ``resident_blocks_mask`` / ``paged_decode_row_mask`` -
  the same three for a caller-supplied block mask instead of section 4.2's rule.

Readings taken where the paper is silent (each is also listed in the design
notes): the local case is restricted to j <= i (causal); the head offset is
``global_head_index mod stride``; the local count includes the diagonal block;
the upper bound on i-j in the stride case is a separate ``window_blocks``
parameter (0 = unbounded); scores are multiplied by an explicit ``scale``; LSE
is the natural-log sum-exp of the scaled scores over unmasked keys.
"""

import numpy as np

# --------------------------------------------------------------------------
# Layout (integer work)
# --------------------------------------------------------------------------


def head_offset(global_head, stride):
    """Offset o_h of the vertical stripes of one head (section 4.2).

    The paper leaves o_h unspecified; the workloads define it as the global
    head index modulo the stride, which makes different heads pick different
    shards and, when there are at least ``stride`` heads, cover every shard.
    """
    if stride <= 0:
        return 0
    return int(global_head) % int(stride)


def block_predicate(i, j, o_h, local_blocks, stride, window_blocks):
    """M^h[i][j] for one (i, j): section 4.2's two cases, plus causality.

    Local : 0 <= i-j < B_l.
    Stride: j-o_h is zero or a positive multiple of s, and B_l <= i-j, and
            (if a window is given) i-j < window.
    """
    d = i - j
    if d < 0:
        return False
    if d < local_blocks:
        return True
    if stride <= 0:
        return False
    if window_blocks > 0 and d >= window_blocks:
        return False
    r = j - o_h
    return r >= 0 and r % stride == 0


def block_mask(num_heads, num_blocks, local_blocks, stride, head_index_base=0,
               window_blocks=0, dense=False):
    """Boolean array [H, B, B]: the predicate evaluated at every (h, i, j).

    Vectorised over the (i, j) grid, but each entry depends only on its own
    (h, i, j) - no row is derived from another.
    """
    H, B = int(num_heads), int(num_blocks)
    i = np.arange(B, dtype=np.int64)[:, None]
    j = np.arange(B, dtype=np.int64)[None, :]
    d = i - j
    causal = d >= 0
    M = np.zeros((H, B, B), dtype=bool)
    for h in range(H):
        if dense:
            M[h] = causal
            continue
        local = causal & (d < local_blocks)
        if stride > 0:
            o_h = head_offset(head_index_base + h, stride)
            r = j - o_h
            stripe = (r >= 0) & (r % stride == 0) & (d >= local_blocks)
            if window_blocks > 0:
                stripe &= d < window_blocks
            M[h] = local | stripe
        else:
            M[h] = local
    return M


def with_sink(M, sink_blocks):
    """The mask with the first `sink_blocks` KV blocks added to every row (the "+ Sink" variants
    of section 5.1's table): M'[h][i][j] = M[h][i][j] or (j < sink_blocks and j <= i)."""
    H, B, _ = M.shape
    out = M.copy()
    for i in range(B):
        for j in range(min(int(sink_blocks), i + 1)):
            out[:, i, j] = True
    return out


def homogeneous_mask(num_heads, num_blocks, local_blocks, stride, offset=0, window_blocks=0):
    """Section 5.1's "Homogeneous" group: every head attends the same shards, i.e. the mask of
    section 4.2 with one and the same offset for all heads."""
    one = block_mask(1, num_blocks, local_blocks, stride, head_index_base=offset,
                     window_blocks=window_blocks)
    return np.repeat(one, int(num_heads), axis=0)


def valid_custom_mask(M):
    """What a caller-supplied block mask must satisfy for decoder attention: nothing above the
    diagonal (causal), and the diagonal block kept in every row (a token attends itself, so no
    softmax is empty)."""
    H, B, _ = M.shape
    i = np.arange(B)
    return bool(not np.triu(M, k=1).any() and M[:, i, i].all())


def compressed_layout(M):
    """Canonical CSR and CSC of a [H, B, B] mask, by scanning.

    Rows are ordered head-major then block-row; inside a row the columns are
    strictly ascending.  ``row_ptr[h*B+i]`` is the global offset into
    ``col_idx``.  The CSC side is the exact transpose: columns ordered
    head-major then block-column, row indices ascending inside a column.
    """
    H, B, _ = M.shape
    row_ptr = np.zeros(H * B + 1, dtype=np.int32)
    col_ptr = np.zeros(H * B + 1, dtype=np.int32)
    cols, rows = [], []
    n = 0
    for h in range(H):
        for i in range(B):
            js = np.flatnonzero(M[h, i])
            cols.append(js)
            n += js.size
            row_ptr[h * B + i + 1] = n
    n = 0
    for h in range(H):
        for j in range(B):
            is_ = np.flatnonzero(M[h, :, j])
            rows.append(is_)
            n += is_.size
            col_ptr[h * B + j + 1] = n
    col_idx = np.concatenate(cols).astype(np.int32) if cols else np.zeros(0, np.int32)
    row_idx = np.concatenate(rows).astype(np.int32) if rows else np.zeros(0, np.int32)
    return row_ptr, col_idx, col_ptr, row_idx


def covers_all(M):
    """True iff the union over heads contains every causal block (section 4.2)."""
    B = M.shape[1]
    union = M.any(axis=0)
    return bool(np.array_equal(union, np.tril(np.ones((B, B), dtype=bool))))


def token_mask(Mh, block_size, n_tokens, row_start=0, row_stop=None):
    """Token-level mask rows [row_start, row_stop) x [0, n_tokens) of one head.

    mask[t][u] = M^h[t div S][u div S] and u <= t.  The last block may be
    partial when n_tokens is not a multiple of S (B = ceil(N/S), section 3.2).
    """
    if row_stop is None:
        row_stop = n_tokens
    t = np.arange(row_start, row_stop, dtype=np.int64)
    u = np.arange(n_tokens, dtype=np.int64)
    blk = Mh[(t // block_size)[:, None], (u // block_size)[None, :]]
    return blk & (u[None, :] <= t[:, None])


def unmasked_pairs(M, block_size, n_tokens):
    """Number of (query, key) pairs kept by the mask, summed over heads."""
    total = 0
    for h in range(M.shape[0]):
        for r0 in range(0, n_tokens, 2048):
            r1 = min(n_tokens, r0 + 2048)
            total += int(token_mask(M[h], block_size, n_tokens, r0, r1).sum())
    return total


# --------------------------------------------------------------------------
# Attention (floating point, fp64)
# --------------------------------------------------------------------------

_ROW_CHUNK = 1024  # rows of the score matrix held at once; memory only


def _f64(x):
    return np.asarray(x, dtype=np.float64)


def attention_forward_head(q, k, v, Mh, block_size, scale):
    """One head: q,k [N,D], v [N,Dv] -> O [N,Dv], LSE [N] (section 3.2).

    z = scale * q k^T;  LSE[t] = ln sum_{u kept} exp z[t][u];
    P = exp(z - LSE) on kept keys, 0 elsewhere;  O = P v.
    """
    q, k, v = _f64(q), _f64(k), _f64(v)
    N = q.shape[0]
    O = np.empty((N, v.shape[1]), dtype=np.float64)
    LSE = np.empty(N, dtype=np.float64)
    for r0 in range(0, N, _ROW_CHUNK):
        r1 = min(N, r0 + _ROW_CHUNK)
        keep = token_mask(Mh, block_size, N, r0, r1)
        z = scale * (q[r0:r1] @ k.T)
        z = np.where(keep, z, -np.inf)
        m = z.max(axis=1, keepdims=True)
        e = np.exp(z - m)
        l = e.sum(axis=1, keepdims=True)
        LSE[r0:r1] = (m + np.log(l))[:, 0]
        O[r0:r1] = (e / l) @ v
    return O, LSE


def attention_backward_head(q, k, v, dO, Mh, block_size, scale):
    """One head: gradients of sum(O*dO) w.r.t. q, k, v.

    P as in the forward;  dV = P^T dO;  dP = dO v^T;
    delta[t] = sum_u P[t][u] dP[t][u];  dS = P * (dP - delta);
    dQ = scale * dS k;  dK = scale * dS^T q.
    Returns (dQ, dK, dV, O, LSE).
    """
    q, k, v, dO = _f64(q), _f64(k), _f64(v), _f64(dO)
    N = q.shape[0]
    O = np.empty((N, v.shape[1]), dtype=np.float64)
    LSE = np.empty(N, dtype=np.float64)
    dQ = np.zeros_like(q)
    dK = np.zeros_like(k)
    dV = np.zeros_like(v)
    for r0 in range(0, N, _ROW_CHUNK):
        r1 = min(N, r0 + _ROW_CHUNK)
        keep = token_mask(Mh, block_size, N, r0, r1)
        z = scale * (q[r0:r1] @ k.T)
        z = np.where(keep, z, -np.inf)
        m = z.max(axis=1, keepdims=True)
        e = np.exp(z - m)
        l = e.sum(axis=1, keepdims=True)
        LSE[r0:r1] = (m + np.log(l))[:, 0]
        P = e / l
        O[r0:r1] = P @ v
        dOc = dO[r0:r1]
        dV += P.T @ dOc
        dP = dOc @ v.T
        delta = (P * dP).sum(axis=1, keepdims=True)
        dS = P * (dP - delta)
        dQ[r0:r1] = scale * (dS @ k)
        dK += scale * (dS.T @ q[r0:r1])
    return dQ, dK, dV, O, LSE


def attention_forward(q, k, v, M, block_size, scale):
    """q,k,v [Bt,H,N,D] -> O [Bt,H,N,D], LSE [Bt,H,N]; M is [H,B,B]."""
    q, k, v = np.asarray(q), np.asarray(k), np.asarray(v)
    Bt, H, N, _ = q.shape
    O = np.empty(v.shape, dtype=np.float64)
    LSE = np.empty((Bt, H, N), dtype=np.float64)
    for b in range(Bt):
        for h in range(H):
            O[b, h], LSE[b, h] = attention_forward_head(q[b, h], k[b, h], v[b, h], M[h],
                                                        block_size, scale)
    return O, LSE


def attention_backward(q, k, v, dO, M, block_size, scale):
    """Batched gradients; returns (dQ, dK, dV, O, LSE)."""
    q, k, v, dO = np.asarray(q), np.asarray(k), np.asarray(v), np.asarray(dO)
    Bt, H, N, _ = q.shape
    dQ = np.empty(q.shape, dtype=np.float64)
    dK = np.empty(k.shape, dtype=np.float64)
    dV = np.empty(v.shape, dtype=np.float64)
    O = np.empty(v.shape, dtype=np.float64)
    LSE = np.empty((Bt, H, N), dtype=np.float64)
    for b in range(Bt):
        for h in range(H):
            dQ[b, h], dK[b, h], dV[b, h], O[b, h], LSE[b, h] = attention_backward_head(
                q[b, h], k[b, h], v[b, h], dO[b, h], M[h], block_size, scale)
    return dQ, dK, dV, O, LSE


def attention_forward_varlen(q, k, v, cu_seqlens, M, block_size, scale):
    """Packed batch of sequences of different lengths (serving prefill, section 5.3).

    q,k,v [H,total,D]; sequence s owns rows cu_seqlens[s] .. cu_seqlens[s+1]-1 and
    is an attention problem of its own: its first token is position 0 of the mask,
    its last block may be partial, and it sees no other sequence.  M [H,B,B] needs
    B >= ceil(longest length / S).  Returns O [H,total,D], LSE [H,total]; rows that
    belong to no sequence (after cu_seqlens[-1]) come back as NaN.
    """
    q, k, v = np.asarray(q), np.asarray(k), np.asarray(v)
    H, total, _ = q.shape
    cu = [int(x) for x in cu_seqlens]
    O = np.full(v.shape, np.nan, dtype=np.float64)
    LSE = np.full((H, total), np.nan, dtype=np.float64)
    for lo, hi in zip(cu[:-1], cu[1:]):
        if hi == lo:
            continue
        for h in range(H):
            O[h, lo:hi], LSE[h, lo:hi] = attention_forward_head(q[h, lo:hi], k[h, lo:hi], v[h, lo:hi], M[h],
                                                                block_size, scale)
    return O, LSE


def attention_backward_varlen(q, k, v, dO, cu_seqlens, M, block_size, scale):
    """Gradients of sum(O*dO) for a packed batch (see attention_forward_varlen).

    Every sequence is differentiated on its own.  Returns (dQ, dK, dV, O, LSE) in
    the packed shapes; rows that belong to no sequence come back as NaN.
    """
    q, k, v, dO = np.asarray(q), np.asarray(k), np.asarray(v), np.asarray(dO)
    H, total, _ = q.shape
    cu = [int(x) for x in cu_seqlens]
    dQ = np.full(q.shape, np.nan, dtype=np.float64)
    dK = np.full(k.shape, np.nan, dtype=np.float64)
    dV = np.full(v.shape, np.nan, dtype=np.float64)
    O = np.full(v.shape, np.nan, dtype=np.float64)
    LSE = np.full((H, total), np.nan, dtype=np.float64)
    for lo, hi in zip(cu[:-1], cu[1:]):
        if hi == lo:
            continue
        for h in range(H):
            dQ[h, lo:hi], dK[h, lo:hi], dV[h, lo:hi], O[h, lo:hi], LSE[h, lo:hi] = attention_backward_head(
                q[h, lo:hi], k[h, lo:hi], v[h, lo:hi], dO[h, lo:hi], M[h], block_size, scale)
    return dQ, dK, dV, O, LSE


def forward_rows(q_rows, row_index, k, v, Mh, block_size, scale):
    """Forward for selected query rows of one head (rows are independent).

    q_rows [R,D] are the queries at absolute positions ``row_index`` [R];
    k, v hold the keys from position 0 up to at least the last of those
    positions.  This is also the definition of a prefill chunk (a run of query
    rows against the keys cached so far), and it is used to sample outputs at
    sizes where the full score matrix is too large.
    """
    q_rows, k, v = _f64(q_rows), _f64(k), _f64(v)
    N = k.shape[0]
    t = np.asarray(row_index, dtype=np.int64)
    u = np.arange(N, dtype=np.int64)
    keep = Mh[(t // block_size)[:, None], (u // block_size)[None, :]] & (u[None, :] <= t[:, None])
    z = np.where(keep, scale * (q_rows @ k.T), -np.inf)
    m = z.max(axis=1, keepdims=True)
    e = np.exp(z - m)
    l = e.sum(axis=1, keepdims=True)
    return (e / l) @ v, (m + np.log(l))[:, 0]


def decode_row(q, k_cache, v_cache, length, global_head, block_size, local_blocks, stride,
               scale, window_blocks=0, dense=False):
    """One decoding step of one head (section 4.1).

    The query is the token at position L-1 whose key/value already sit in the
    cache; it attends, among the first L cached tokens, to those whose block
    is active in block-row (L-1) div S of the mask built for B = ceil(L/S)
    blocks.  q [D]; k_cache, v_cache [>=L, D].  Returns (o [D], lse).
    """
    L = int(length)
    q = _f64(q)
    k = _f64(k_cache[:L])
    v = _f64(v_cache[:L])
    i = (L - 1) // block_size
    o_h = head_offset(global_head, stride)
    keep = np.zeros(L, dtype=bool)
    for u in range(L):
        j = u // block_size
        if dense:
            keep[u] = j <= i
        else:
            keep[u] = block_predicate(i, j, o_h, local_blocks, stride, window_blocks)
    z = scale * (k @ q)
    z = np.where(keep, z, -np.inf)
    m = z.max()
    e = np.exp(z - m)
    l = e.sum()
    return (e / l) @ v, m + np.log(l)


# ---------------------------------------------------------------------------------------------
# Paged KV cache with block-aligned eviction (section 4.1)
# ---------------------------------------------------------------------------------------------

def resident_blocks(length, global_head, block_size, local_blocks, stride, window_blocks=0,
                    dense=False):
    """Logical KV blocks of one head that must stay cached once `length` tokens are cached.

    Section 4.1: a KV block may be evicted as soon as no later query can attend to
    it.  Written out as that definition: block j (among the ceil(L/S) blocks that
    exist) stays iff SOME query block row i' >= (L-1) div S keeps it.  The scan
    over future rows stops where the predicate has become constant in i' for
    every j: the local case ends after B_l rows, the stripe case is constant once
    i'-j >= B_l until the window (if any) ends.  Returns an ascending list.
    """
    L = int(length)
    B = -(-L // block_size)
    i = (L - 1) // block_size
    if dense:
        return list(range(B))
    o_h = head_offset(global_head, stride)
    horizon = local_blocks + window_blocks + max(stride, 1) + 2
    keep = []
    for j in range(B):
        if any(block_predicate(ip, j, o_h, local_blocks, stride, window_blocks)
               for ip in range(i, i + horizon)):
            keep.append(j)
    return keep


def gather_pages(pages, table_row, n_blocks, block_size):
    """Logical cache [n_blocks*S, D] of one (sequence, head) from a page pool.

    pages [num_pages, S, D]; table_row[j] = page holding logical block j, or a
    negative number if the block is not resident.  Blocks that are not resident
    come back as NaN, so that any use of an evicted block shows in the result.
    """
    S = block_size
    D = pages.shape[-1]
    out = np.full((n_blocks * S, D), np.nan, dtype=np.float64)
    for j in range(n_blocks):
        pg = int(table_row[j])
        if pg >= 0:
            out[j * S:(j + 1) * S] = _f64(pages[pg])
    return out


def paged_decode_row(q, k_pages, v_pages, table_row, length, global_head, block_size,
                     local_blocks, stride, scale, window_blocks=0, dense=False):
    """decode_row on the logical cache that the page table describes.

    A paged cache is storage only: the result is by definition that of the
    contiguous cache it represents.  Keys of blocks the mask drops are never
    looked at (their score is -inf whatever they hold), so their being absent
    (NaN here) changes nothing; an absent block that the mask keeps makes the
    result NaN.
    """
    L = int(length)
    B = -(-L // block_size)
    k = gather_pages(k_pages, table_row, B, block_size)
    v = gather_pages(v_pages, table_row, B, block_size)
    # decode_row multiplies every cached row by q before masking; rows of absent, dropped blocks
    # must not turn into NaN * 0 there, so they are zeroed exactly where the mask drops them
    i = (L - 1) // block_size
    o_h = head_offset(global_head, stride)
    for j in range(B):
        kept = (j <= i) if dense else block_predicate(i, j, o_h, local_blocks, stride, window_blocks)
        if not kept:
            k[j * block_size:(j + 1) * block_size] = 0.0
            v[j * block_size:(j + 1) * block_size] = 0.0
    return decode_row(q, k, v, L, global_head, block_size, local_blocks, stride, scale,
                      window_blocks, dense)


# ---------------------------------------------------------------------------------------------
# Decode and eviction under a caller-supplied block mask (section 4.1 applied to any pattern)
# ---------------------------------------------------------------------------------------------
def decode_row_mask(q, k_cache, v_cache, length, Mh, block_size, scale):
    """One decoding step of one head whose pattern is the block mask Mh [B,B].

    The newest token, at position L-1, is query row L-1 of the causal attention
    that Mh describes: the result is that row of the forward, by definition.
    q [D]; k_cache, v_cache [>=L, D].  Returns (o [D], lse).
    """
    L = int(length)
    o, lse = forward_rows(_f64(q)[None, :], [L - 1], k_cache[:L], v_cache[:L], Mh, block_size, scale)
    return o[0], lse[0]


def resident_blocks_mask(Mh, length, block_size):
    """Blocks that must stay cached once `length` tokens are cached, for a mask Mh [B,B].

    Section 4.1's rule as a definition: block j among those that exist stays iff
    the row of the newest token or any later row of Mh keeps it.
    """
    L = int(length)
    i = (L - 1) // block_size
    return [j for j in range(i + 1) if bool(Mh[i:, j].any())]


def paged_decode_row_mask(q, k_pages, v_pages, table_row, length, Mh, block_size, scale):
    """decode_row_mask on the logical cache that the page table describes (see paged_decode_row)."""
    L = int(length)
    B = -(-L // block_size)
    k = gather_pages(k_pages, table_row, B, block_size)
    v = gather_pages(v_pages, table_row, B, block_size)
    i = (L - 1) // block_size
    for j in range(B):
        if not Mh[i, j]:  # dropped by the mask: never looked at, so absent (NaN) rows must not reach 0 * NaN
            k[j * block_size:(j + 1) * block_size] = 0.0
            v[j * block_size:(j + 1) * block_size] = 0.0
    return decode_row_mask(q, k, v, L, Mh, block_size, scale)
