"""Seeded synthetic inputs and the workload table.

This module holds no attention arithmetic: it draws random tensors, rounds
them to bf16 and describes the five workloads (shapes and layout parameters).
It is the one module that both the CPU oracle's tests and the HIP library's
callers use, so that both sides see the same bits.

The shapes stand in for the paper's attention benchmark (section 5.3): a
1.3B-parameter shape (16 heads x 128), the Llama-2-7B shape (32 heads x 128),
64-token shards (section 5.1), contexts from 8K to 128K (section 5.2).
"""

from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20240717


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    batch: int
    heads: int
    seqlen: int
    head_dim: int
    block_size: int
    local_blocks: int
    stride: int
    window_blocks: int = 0
    kind: str = "train"          # "train" or "decode"
    min_len: int = 0             # decode only
    max_len: int = 0             # decode only

    @property
    def num_blocks(self):
        return (self.seqlen + self.block_size - 1) // self.block_size

    @property
    def scale(self):
        return 1.0 / float(np.sqrt(self.head_dim))


WORKLOADS = {
    "tiny": Workload("tiny", 1, 1, 4, 512, 64, 64, 2, 4),
    "1p3b_8k": Workload("1p3b_8k", 2, 4, 16, 8192, 128, 64, 4, 8),
    "7b_32k": Workload("7b_32k", 3, 1, 32, 32768, 128, 64, 16, 16),
    "7b_128k": Workload("7b_128k", 4, 1, 32, 131072, 128, 128, 8, 32),
    "7b_decode": Workload("7b_decode", 5, 64, 32, 32768, 128, 64, 16, 16, kind="decode",
                          min_len=8192, max_len=32768),
}


def rng_for(index, stream=0):
    """Generator for workload ``index``; ``stream`` separates independent draws."""
    return np.random.Generator(np.random.PCG64([BASE_SEED + int(index), int(stream)]))


def round_to_bf16_bits(x):
    """float32 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits):
    """uint16 bf16 bit patterns -> float32 values (exact)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(rng, shape):
    """Standard-normal draws rounded to bf16; returns the uint16 bit patterns."""
    return round_to_bf16_bits(rng.standard_normal(size=shape, dtype=np.float32))


def train_inputs(w, heads=None, batch=None, seqlen=None):
    """Q, K, V, dO as bf16 bit patterns [Bt, H, N, D], drawn in that order.

    ``heads`` / ``batch`` / ``seqlen`` shrink the workload for small parity
    cases; the draw order and seed stay those of the workload.
    """
    H = w.heads if heads is None else heads
    Bt = w.batch if batch is None else batch
    N = w.seqlen if seqlen is None else seqlen
    rng = rng_for(w.index)
    shape = (Bt, H, N, w.head_dim)
    return tuple(normal_bf16(rng, shape) for _ in range(4))


def decode_lengths(w, nseq=None, seed_stream=1):
    """Per-sequence cache lengths, integer-uniform in [min_len, max_len]."""
    n = w.batch if nseq is None else nseq
    rng = rng_for(w.index, seed_stream)
    return rng.integers(w.min_len, w.max_len + 1, size=n).astype(np.int32)


def prefill_lengths(w, nseq, min_len, seed_stream=4):
    """Prompt lengths of a serving prefill batch: log-uniform integers in [min_len, w.seqlen], no
    rounding to blocks (the mix of a few long and many short prompts that batches of requests have)."""
    rng = rng_for(w.index, seed_stream)
    x = rng.uniform(np.log(min_len), np.log(w.seqlen), size=nseq)
    return np.minimum(np.exp(x).astype(np.int64), w.seqlen).astype(np.int32)


def decode_inputs_small(w, nseq, heads, max_len, lengths=None):
    """A host-side decode case: q [nseq,H,D], K/V cache [nseq,H,max_len,D] bits, lengths."""
    rng = rng_for(w.index, 2)
    q = normal_bf16(rng, (nseq, heads, w.head_dim))
    kc = normal_bf16(rng, (nseq, heads, max_len, w.head_dim))
    vc = normal_bf16(rng, (nseq, heads, max_len, w.head_dim))
    if lengths is None:
        lengths = rng.integers(max(1, max_len // 4), max_len + 1, size=nseq).astype(np.int32)
    return q, kc, vc, np.asarray(lengths, dtype=np.int32)


def page_table(resident, max_blocks, extra_pages=3, seed_stream=3, index=0):
    """Scatters resident blocks over a page pool.

    resident[b][h] = list of logical block numbers of (sequence b, head h) that are held.  Returns
    (table int32 [nseq, heads, max_blocks] with -1 for blocks not held, num_pages): every held
    block gets its own page, pages handed out in a seeded random order, `extra_pages` pages left
    unused.  Bookkeeping only; which blocks are held is the caller's business.
    """
    nseq, heads = len(resident), len(resident[0])
    total = sum(len(r) for row in resident for r in row)
    num_pages = total + extra_pages
    order = rng_for(index, seed_stream).permutation(num_pages)
    table = np.full((nseq, heads, max_blocks), -1, dtype=np.int32)
    n = 0
    for b in range(nseq):
        for h in range(heads):
            for j in resident[b][h]:
                table[b, h, j] = order[n]
                n += 1
    return table, num_pages


def pages_from_cache(cache_bits, table, num_pages, block_size):
    """Page pool [num_pages, S, D] (bf16 bits) holding the blocks of a contiguous cache
    [nseq, heads, max_len, D] that `table` marks as held; other pages get a recognisable filler."""
    nseq, heads, max_len, D = cache_bits.shape
    pool = np.full((num_pages, block_size, D), 0x7F00, dtype=np.uint16)  # large finite bf16 values
    for b in range(nseq):
        for h in range(heads):
            for j in np.nonzero(table[b, h] >= 0)[0]:
                lo = j * block_size
                rows = cache_bits[b, h, lo:lo + block_size]
                pool[table[b, h, j], :rows.shape[0]] = rows
    return pool
