/*
 * s2attn - head-heterogeneous block-sparse causal attention for AMD MI355X (gfx950).
 *
 * C ABI of libs2attn.so.  Every pointer is marked HOST or DEVICE.  bf16 tensors are
 * raw 16-bit patterns (void*); LSE and workspaces are float / bytes.  The library
 * never takes ownership of a tensor or workspace; it owns only the index arrays
 * inside an s2_layout handle.  All launches are asynchronous on the stream passed
 * in (a hipStream_t cast to void*, NULL = the default stream); no call synchronises
 * the device except s2_layout_build/destroy (one upload / free of small arrays).
 *
 * Threads, streams, graphs: the library keeps no mutable state between calls apart from a
 * per-thread copy of the last HIP error.  A layout handle is read-only after it is built and may
 * drive any number of threads and streams at once; two calls may run concurrently whenever their
 * outputs and workspaces do not overlap.  The compute calls only enqueue kernels (no allocation,
 * no memset, no host synchronisation), so they may be captured into a HIP graph once each kernel
 * has been launched at least once outside a capture.
 *
 * Every function returns an int status: S2_OK (0) or a negative S2_ERR_* code.
 * Arguments are validated before anything is launched; on error no output is
 * written.  No C++ exception crosses this boundary.
 *
 * Vocabulary (the paper's): a sequence of N tokens is cut into B = ceil(N/S) shards
 * ("blocks") of S consecutive tokens (section 3.2).  Head h has a B x B block mask
 * M^h (section 4.2): block row i keeps block column j when
 *     0 <= i-j < B_l                                        (local), or
 *     j-o_h in {0, s, 2s, ...}  and  B_l <= i-j             (stride),
 * where o_h = (head_index_base + h) mod s.  If window_blocks > 0 the stride case
 * also requires i-j < window_blocks (the paper's upper bound on i-j).  Inside the
 * diagonal block the token mask is causal (key position <= query position); all
 * other kept blocks are fully visible.
 */
#ifndef S2ATTN_H
#define S2ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  S2_OK = 0,
  S2_ERR_NULL = -1,       /* a required pointer is NULL                                  */
  S2_ERR_BAD_PARAM = -2,  /* layout parameter out of range (B_l < 1, stride < 0, ...)    */
  S2_ERR_SHAPE = -3,      /* tensor shape does not fit the layout / unsupported head_dim */
  S2_ERR_ALIGN = -4,      /* pointer or stride not 16-byte aligned                       */
  S2_ERR_WORKSPACE = -5,  /* workspace missing or too small                              */
  S2_ERR_HIP = -6,        /* a HIP runtime call failed; see s2_last_hip_error()          */
  S2_ERR_NO_DEVICE = -7,  /* layout has no copy on the current device (built without a GPU,
                             or with another device current)                             */
  S2_ERR_OVERFLOW = -8    /* index arrays would not fit in int32                         */
};

/* Parameters of the per-head block mask of section 4.2.  Plain integers, HOST. */
typedef struct {
  int32_t num_heads;       /* H: heads covered by this layout (>= 1)                          */
  int32_t head_index_base; /* global index of local head 0; o_h uses the global index (>= 0)  */
  int32_t num_blocks;      /* B = N / S (>= 1)                                                */
  int32_t block_size;      /* S in tokens: 16, 32, 64 or 128 (16: num_blocks must be even)   */
  int32_t local_blocks;    /* B_l >= 1; counts the diagonal block                             */
  int32_t stride;          /* s >= 0; 0 = no stripes (pure sliding window)                    */
  int32_t window_blocks;   /* upper bound on i-j for stripes; 0 = unbounded                   */
  int32_t dense;           /* 1 = every causal block kept (the three fields above ignored)    */
} s2_layout_params;

/* Opaque handle: the compressed mask (host and device copies) and the kernels' tile lists. */
typedef struct s2_layout s2_layout;

/* Read-only HOST view of a layout.  Canonical form: rows ordered head-major then block-row,
 * columns strictly ascending inside a row, row_ptr[h*B+i] a global offset into col_idx
 * (compressed sparse row, section 3.2).  col_ptr/row_idx are the exact transpose (per head,
 * per block column, ascending rows).  Pointers stay valid until s2_layout_destroy. */
typedef struct {
  const int32_t* row_ptr;  /* [H*B+1] */
  const int32_t* col_idx;  /* [nnz]   */
  const int32_t* col_ptr;  /* [H*B+1] */
  const int32_t* row_idx;  /* [nnz]   */
  int64_t nnz;             /* kept blocks summed over heads                                   */
  int32_t num_heads, num_blocks, block_size;
  int32_t max_row_blocks;  /* longest row                                                     */
  int32_t covers_all;      /* 1 iff the union over heads keeps every causal block (sec. 4.2)  */
  int32_t on_device;       /* 1 iff the device copies exist                                   */
} s2_layout_view;

/* Training-path tensors.  All bf16 tensors are [batch, heads, seqlen, head_dim] addressed as
 * base + b*stride_b + h*stride_h + t*stride_t + d (strides in ELEMENTS, head_dim contiguous).
 * q, o, d_o, dq share the q_* strides; k, v, dk, dv share the kv_* strides.  Strides must be
 * multiples of 8 elements and base pointers 16-byte aligned.  lse is contiguous fp32
 * [batch, heads, seqlen].  Pointers not used by a call may be NULL. */
typedef struct {
  const void* q;    /* DEVICE bf16, in                    */
  const void* k;    /* DEVICE bf16, in                    */
  const void* v;    /* DEVICE bf16, in                    */
  void* o;          /* DEVICE bf16, fwd out / bwd in      */
  float* lse;       /* DEVICE fp32, fwd out / bwd in      */
  const void* d_o;  /* DEVICE bf16, bwd in                */
  void* dq;         /* DEVICE bf16, bwd out               */
  void* dk;         /* DEVICE bf16, bwd out               */
  void* dv;         /* DEVICE bf16, bwd out               */
  int32_t batch, heads, seqlen, head_dim; /* head_dim 64 or 128; seqlen == B*S            */
  int64_t q_stride_b, q_stride_h, q_stride_t;
  int64_t kv_stride_b, kv_stride_h, kv_stride_t;
} s2_tensors;

/* Decode: nseq sequences, one query token each (the token at position len-1, whose key and
 * value are already in the cache), against a contiguous bf16 KV cache (section 4.1). */
typedef struct {
  const void* q;            /* DEVICE bf16 [nseq, heads, head_dim], contiguous               */
  const void* k_cache;      /* DEVICE bf16, element (b,h,t,d) at b*sb + h*sh + t*st + d      */
  const void* v_cache;      /* DEVICE bf16, same strides                                     */
  const int32_t* seq_lens;  /* DEVICE int32 [nseq], each in [1, max_len]                     */
  void* o;                  /* DEVICE bf16 [nseq, heads, head_dim], out                      */
  float* lse;               /* DEVICE fp32 [nseq, heads], out (may be NULL)                  */
  int32_t nseq, heads, head_dim; /* head_dim 64 or 128                                      */
  int32_t max_len;          /* upper bound on seq_lens, sizes the launch                     */
  int32_t num_splits;       /* KV splits per (sequence, head); 0 = library chooses           */
  int64_t kv_stride_seq, kv_stride_head, kv_stride_tok; /* elements, multiples of 8          */
} s2_decode_args;

/* Decode against a PAGED cache (section 4.1: the cache is kept in fixed-size blocks behind a block
 * table, and a head's blocks that no later query can attend are evicted).  A page holds the
 * block_size tokens of one logical KV block of one (sequence, head); K and V pools use the same
 * page numbers. */
typedef struct {
  const void* q;              /* DEVICE bf16 [nseq, heads, head_dim], contiguous             */
  const void* k_pages;        /* DEVICE bf16, element (page,t,d) at page*sp + t*st + d       */
  const void* v_pages;        /* DEVICE bf16, same strides                                   */
  const int32_t* block_table; /* DEVICE int32 [nseq, heads, max_blocks]: page of logical
                                 block j of (sequence, head), negative = not resident        */
  const int32_t* seq_lens;    /* DEVICE int32 [nseq], each in [1, max_blocks*block_size]     */
  void* o;                    /* DEVICE bf16 [nseq, heads, head_dim], out                    */
  float* lse;                 /* DEVICE fp32 [nseq, heads], out (may be NULL)                */
  int32_t* missing;           /* DEVICE int32[1] or NULL: the call ADDS the number of
                                 (sequence, head, block) triples the mask keeps but the
                                 table does not hold (or holds with a page >= num_pages);
                                 the caller zeroes it                                        */
  int32_t nseq, heads, head_dim; /* head_dim 64 or 128                                       */
  int32_t max_blocks;         /* row length of block_table; bounds seq_lens                  */
  int32_t num_pages;          /* pages in each pool                                          */
  int32_t num_splits;         /* KV splits per (sequence, head); 0 = library chooses         */
  int64_t page_stride, tok_stride; /* elements, multiples of 8; tok_stride >= head_dim       */
} s2_paged_decode_args;

/* ---- layout (section 4.2 mask -> compressed lists, section 3.2) ------------------------- */

/* Builds the per-head lists of kept KV blocks from the closed form of the mask, on the host,
 * and, when a GPU is visible, uploads them to the current device.  *out is owned by the
 * caller until s2_layout_destroy.  Errors: NULL, BAD_PARAM (H<1, B<1, S not 16/32/64/128, S = 16
 * with odd B, B_l<1, stride<0, window<0, head_index_base<0), OVERFLOW (more than 32768 blocks, or
 * 65536 16-token ones; list sizes beyond int32), HIP. */
int s2_layout_build(const s2_layout_params* params, s2_layout** out);
/* A layout from the caller's own per-head pattern instead of the section 4.2 rule (section 3
 * promises patterns customised per head and per context range; section 5.1 compares several:
 * attention sink, the same shards for all heads, plain sliding window).  row_ptr[H*B + 1] and
 * col_idx[row_ptr[H*B]] are HOST int32 arrays in the order s2_layout_get returns them: rows
 * ordered head-major, and inside a row the kept KV block columns strictly ascending, none above
 * the row's own index (causal) and the row's own index last (a token always attends its own
 * block, so no softmax is empty).  The arrays are copied.  The result works with s2_attn_fwd /
 * s2_attn_bwd, and with s2_attn_decode_layout / s2_attn_decode_paged_layout.
 * Errors: NULL, BAD_PARAM (H<1, B<1, S not 16/32/64/128, S = 16 with odd B, or a row breaking the rules above), OVERFLOW,
 * HIP. */
int s2_layout_from_csr(int32_t num_heads, int32_t num_blocks, int32_t block_size,
                       const int32_t* row_ptr, const int32_t* col_idx, s2_layout** out);
int s2_layout_destroy(s2_layout* layout);
int s2_layout_get(const s2_layout* layout, s2_layout_view* out);

/* The work lists the kernels walk, for inspection (section 3.2's Merge-Q: one 128-row query tile
 * serves `group` fine mask rows; its mirror image for key tiles).  HOST pointers into the handle.
 * For head h and tile t the list is ent[ptr[h*T + t] .. ptr[h*T + t + 1]), each entry
 * (unit << 16) | bits: `unit` is a partner block, or with 16-token blocks a pair of adjacent
 * partner blocks (blocks_per_unit = 2), and bit r*blocks_per_unit + c says that member r of the
 * tile keeps block unit*blocks_per_unit + c.  Row tiles (which = S2_TILES_FWD, S2_TILES_DQ): member
 * r is block row t*group + r, partners are KV block columns, ascending.  Column tiles
 * (S2_TILES_DKDV): member r is block column members[(h*T + t)*group + r] (-1 = none), partners are
 * query block rows, descending - except that where a head has eight or more column tiles of one
 * length n, each attending one unbroken run of rows (the local-window tiles), such a tile starts at
 * its row that is a multiple of n and goes down from there, wrapping round to the run's last row, so
 * that tiles running side by side read the same query block at the same time.  order[h*T + k] is the
 * k-th tile of head h by descending length.  Errors: NULL, BAD_PARAM (which). */
enum { S2_TILES_FWD = 0, S2_TILES_DQ = 1, S2_TILES_DKDV = 2 };
typedef struct {
  const int32_t* ptr;      /* [H*T + 1]                              */
  const int32_t* ent;      /* [ptr[H*T]]                             */
  const int32_t* order;    /* [H*T]                                  */
  const int32_t* members;  /* [H*T*group]                            */
  int32_t tiles_per_head;  /* T                                      */
  int32_t group;           /* members per tile                       */
  int32_t blocks_per_unit; /* 1, or 2 with 16-token blocks           */
} s2_tile_view;
int s2_layout_get_tiles(const s2_layout* layout, int which, s2_tile_view* out);

/* Where the backward that keeps dS (see s2_attn_bwd_layout_workspace_bytes) puts it, for inspection.
 * The dK/dV launch walks the S2_TILES_DKDV lists in 64-row chunks (an entry of a 128-token block is
 * two chunks, the later rows first); chunk c of entry e of the `ent` array is step e * cpb + c
 * (cpb = block_size / 64) and leaves two 8 KiB units of 64 queries x 64 keys: 2 * step + r for the
 * keys of member r (64-token blocks) or of the block's 64-key half r (128-token blocks).  dq_units
 * says where the dQ launch finds them again: for chunk c (64 keys, ascending) of entry e of the
 * S2_TILES_DQ `ent` array and 64-row half m of the 128-row query tile, dq_units[(e * cpb + c) * 2 + m]
 * is the unit, or -1 when mask row m does not keep the block or every key of the piece lies after
 * every query.  count = entries of dq_units, ds_units = units per batch element; both 0 when the
 * layout's block size is not 64 or 128 (the path does not apply).  HOST pointers into the handle.
 * Errors: NULL. */
typedef struct {
  const int32_t* dq_units; /* [count]                                */
  int64_t count;
  int64_t ds_units;
} s2_ds_units_view;
int s2_layout_get_ds_units(const s2_layout* layout, s2_ds_units_view* out);

/* ---- forward (section 3.2: softmax over the kept keys only) ------------------------------ */

/* O = softmax(scale * Q K^T restricted to the mask) V, LSE = natural-log sum-exp of the scaled
 * kept scores.  Reads q,k,v; writes o (bf16) and lse (fp32).  scale must be > 0.
 * Requires t->heads == layout heads and t->seqlen == B*S.  Errors: NULL, SHAPE, ALIGN,
 * BAD_PARAM (scale), NO_DEVICE, HIP. */
int s2_attn_fwd(const s2_layout* layout, const s2_tensors* t, float scale, void* stream);

/* The same for a run of query rows only (chunked prefill when serving, section 5.3's prefill
 * measurements): t->q, t->o and t->lse hold q_rows rows, row r being the token at sequence
 * position q_row_start + r; t->k and t->v hold t->seqlen rows from position 0, with
 * q_row_start + q_rows <= t->seqlen <= B*S of the layout (keys after a query are never read).
 * q_row_start and q_rows must be multiples of 128, q_rows >= 128.  lse is [batch, heads, q_rows].
 * Every row comes out bit-identical to the same row of s2_attn_fwd on the whole sequence.
 * Errors as s2_attn_fwd. */
int s2_attn_fwd_rows(const s2_layout* layout, const s2_tensors* t, int32_t q_row_start,
                     int32_t q_rows, float scale, void* stream);

/* The forward for a packed batch of sequences of different lengths (serving prefill batches,
 * section 5.3): t->batch must be 1 and t->seqlen is the number of rows in q, k, v, o; lse is
 * [heads, t->seqlen].  cu_seqlens is DEVICE int32 [num_seqs + 1], ascending from 0: sequence s
 * owns rows cu_seqlens[s] .. cu_seqlens[s+1]-1 and is attended on its own, its first token at
 * position 0 of the mask; any length >= 0 (no multiple of the block size is asked for).  No
 * length may exceed max_seqlen, and max_seqlen <= B*S of the layout.  The array is read by the
 * kernel only: a length above max_seqlen is cut there, rows outside the tensors are never
 * touched, and rows that belong to no sequence are left as they were.  Each row comes out as
 * s2_attn_fwd gives it for the same sequence alone.  Errors: NULL, SHAPE (batch != 1, head
 * count, num_seqs < 1, max_seqlen < 1 or beyond the layout), ALIGN, BAD_PARAM (scale),
 * NO_DEVICE, HIP. */
int s2_attn_fwd_varlen(const s2_layout* layout, const s2_tensors* t, const int32_t* cu_seqlens,
                       int32_t num_seqs, int32_t max_seqlen, float scale, void* stream);

/* ---- backward (gradient of the above) ---------------------------------------------------- */

/* Given q,k,v,o,lse,d_o writes dq,dk,dv (bf16; fp32 accumulation).  workspace is DEVICE memory
 * of at least s2_attn_bwd_workspace_bytes(...) bytes, 256-byte aligned, contents undefined on
 * entry and exit.  Errors as forward plus WORKSPACE. */
int s2_attn_bwd(const s2_layout* layout, const s2_tensors* t, float scale, void* workspace,
                size_t workspace_bytes, void* stream);
size_t s2_attn_bwd_workspace_bytes(int32_t batch, int32_t heads, int32_t seqlen, int32_t head_dim);

/* The larger workspace with which s2_attn_bwd / s2_attn_bwd_stages compute nothing twice.  With the
 * size above, the dQ launch forms the scores and dP = dO V^T a second time to get at
 * dS = P * (dP - delta): seven contractions for the five the gradient consists of.  Given this many
 * bytes instead, the dK/dV launch leaves dS (bf16, 2 bytes per kept block element: 8 KiB per 64 x 64
 * piece the launch visits) in the workspace and the dQ launch is the single contraction
 * dQ = scale * dS K over it.  Same results to rounding (dQ then takes the same bf16 dS that dK takes),
 * bitwise repeatable like the other path.  Covers head_dim 128, mask blocks of 64 or 128 tokens and
 * seqlen a multiple of 128; for any other call the value equals s2_attn_bwd_workspace_bytes and the
 * other path runs.  Which path a call takes is decided by workspace_bytes alone. */
size_t s2_attn_bwd_layout_workspace_bytes(const s2_layout* layout, int32_t batch, int32_t heads,
                                          int32_t seqlen, int32_t head_dim);

/* The backward for a packed batch of sequences of different lengths: the gradient of
 * s2_attn_fwd_varlen, same tensors and cu_seqlens (o and lse as that call left them), d_o / dq /
 * dk / dv packed like q / k / v.  Rows that belong to no sequence are left as they were.
 * workspace: s2_attn_bwd_varlen_workspace_bytes(heads, rows of the tensors, head_dim) bytes,
 * DEVICE, 256-byte aligned.  Errors as s2_attn_fwd_varlen plus WORKSPACE. */
int s2_attn_bwd_varlen(const s2_layout* layout, const s2_tensors* t, const int32_t* cu_seqlens,
                       int32_t num_seqs, int32_t max_seqlen, float scale, void* workspace,
                       size_t workspace_bytes, void* stream);
size_t s2_attn_bwd_varlen_workspace_bytes(int32_t heads, int32_t rows, int32_t head_dim);

/* The backward is two launches: dQ (which also computes delta = rowsum(dO*O) and leaves it in
 * the workspace), then dK/dV (which reads delta).  This variant runs the subset named by `stages`
 * (an OR of the flags below) so that a profiler or a benchmark can time each launch on its own;
 * with S2_BWD_ALL it is s2_attn_bwd.  S2_BWD_DKDV needs delta in the workspace: from S2_BWD_DQ in
 * the same or an earlier call, or from S2_BWD_DELTA, a stand-alone delta kernel that only runs
 * when S2_BWD_DQ is not part of the call.  With the larger workspace of
 * s2_attn_bwd_layout_workspace_bytes the order is delta kernel (S2_BWD_DELTA), dK/dV (S2_BWD_DKDV,
 * needs delta, leaves dS), dQ (S2_BWD_DQ, needs dS from S2_BWD_DKDV in the same or an earlier call
 * on the same workspace).  Errors as s2_attn_bwd, plus BAD_PARAM for stages. */
enum { S2_BWD_DELTA = 1, S2_BWD_DKDV = 2, S2_BWD_DQ = 4, S2_BWD_ALL = 7 };
int s2_attn_bwd_stages(const s2_layout* layout, const s2_tensors* t, float scale, void* workspace,
                       size_t workspace_bytes, int stages, void* stream);

/* ---- dense causal attention: the in-library speed baseline ------------------------------- */

/* Same tensors and outputs as s2_attn_fwd / s2_attn_bwd with every causal key kept; the block
 * loop is arithmetic (no index lists, no layout handle).  seqlen must be a multiple of 128. */
int s2_dense_causal_fwd(const s2_tensors* t, float scale, void* stream);
int s2_dense_causal_bwd(const s2_tensors* t, float scale, void* workspace, size_t workspace_bytes,
                        void* stream);

/* ---- decode (section 4.1: one step against the cache) ------------------------------------ */

/* For sequence b with length L = seq_lens[b]: the query attends, among the first L cached
 * tokens, the blocks kept in block row (L-1) div S of the mask for ceil(L/S) blocks (the last
 * block may be partial).  The KV range is cut into num_splits pieces whose partial
 * (max, sum, accumulator) triples go to workspace and are merged by a second kernel.
 * p->num_heads must equal a->heads; p->num_blocks is ignored.  Errors: NULL, BAD_PARAM, SHAPE,
 * ALIGN, WORKSPACE, HIP. */
int s2_attn_decode(const s2_layout_params* p, const s2_decode_args* a, float scale,
                   void* workspace, size_t workspace_bytes, void* stream);
size_t s2_attn_decode_workspace_bytes(int32_t nseq, int32_t heads, int32_t head_dim,
                                      int32_t max_len, int32_t num_splits);
/* Upper bound on the split count the library picks for num_splits == 0, and the count that
 * s2_attn_decode_workspace_bytes(..., 0) sizes the workspace for.  The call itself may use fewer
 * splits when the pattern keeps so few blocks per row that more splits would leave wavefronts idle. */
int32_t s2_attn_decode_default_splits(int32_t nseq, int32_t heads, int32_t max_len);

/* For callers that cannot allocate or hold device memory for the library: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  s2_attn_decode with the split
 * partials kept in a buffer of S2_DECODE_STATIC_SCRATCH_BYTES that is part of the loaded library
 * (each GPU the library runs on holds its own copy until the process ends) instead of a caller's
 * workspace; the call allocates and frees nothing and gives the same o and lse as s2_attn_decode.
 * Shapes whose partials (s2_attn_decode_workspace_bytes of the same arguments) exceed that size
 * are refused with S2_ERR_WORKSPACE before anything is launched: lower num_splits or use
 * s2_attn_decode.  Every call on a GPU uses that GPU's one buffer, whatever the stream, and the
 * buffer keeps the last call's partials (each call overwrites what it reads, so nothing needs
 * clearing): calls that overlap in time on one GPU race; calls on one stream, or otherwise
 * ordered, do not.  Errors: as s2_attn_decode, plus NO_DEVICE when no GPU is visible. */
#define S2_DECODE_STATIC_SCRATCH_BYTES (8u << 20)
int s2_attn_decode_static(const s2_layout_params* p, const s2_decode_args* a, float scale, void* stream);

/* Same step against a paged cache.  A kept block whose table entry is negative (or not below
 * num_pages) contributes nothing and is counted in *missing when that pointer is given; blocks
 * the mask drops are never looked up, so their entries may hold anything.  A (sequence, head)
 * all of whose kept blocks are missing gets o = 0 and lse = -inf.  Workspace as for
 * s2_attn_decode with max_len = max_blocks * block_size.  Errors: NULL, BAD_PARAM, SHAPE, ALIGN,
 * WORKSPACE, HIP. */
int s2_attn_decode_paged(const s2_layout_params* p, const s2_paged_decode_args* a, float scale,
                         void* workspace, size_t workspace_bytes, void* stream);

/* Host helper for the cache manager (section 4.1, KV-efficient sparsity): the logical KV blocks
 * of local head `head` that some query at position >= length-1 can still attend once `length`
 * tokens are cached; every other block of that head may be evicted for good.  Writes them in
 * ascending order to blocks[0..capacity) (HOST memory, may be NULL when capacity is 0) and the
 * full count to *count.  Errors: NULL, BAD_PARAM (also head outside [0, num_heads), length < 1),
 * OVERFLOW when capacity is too small (count is still set). */
int s2_kv_resident_blocks(const s2_layout_params* p, int32_t head, int32_t length,
                          int32_t* blocks, int32_t capacity, int32_t* count);

/* The three calls above for a layout handle instead of the closed form, so that a pattern given
 * to s2_layout_from_csr (section 3: per head, per context range) also decodes: the token at
 * position L-1 attends the blocks that row (L-1) div S of the layout keeps.  The layout must
 * cover the cache (max_len, or max_blocks * S, at most B*S) and live on the current device.
 * s2_layout_resident_blocks scans the layout's later rows: with a pattern that does not follow
 * section 4.1's rule a block can be resident without being read at this step.  It also accepts
 * layouts from s2_layout_build, where it agrees with s2_kv_resident_blocks as long as the
 * layout has rows beyond the stripe and window reach of the current one.
 * Errors: as the calls above, plus SHAPE (cache longer than the layout), NO_DEVICE; for
 * s2_layout_resident_blocks BAD_PARAM also when length > B*S. */
int s2_attn_decode_layout(const s2_layout* layout, const s2_decode_args* a, float scale,
                          void* workspace, size_t workspace_bytes, void* stream);
int s2_attn_decode_paged_layout(const s2_layout* layout, const s2_paged_decode_args* a, float scale,
                                void* workspace, size_t workspace_bytes, void* stream);
int s2_layout_resident_blocks(const s2_layout* layout, int32_t head, int32_t length,
                              int32_t* blocks, int32_t capacity, int32_t* count);

/* ---- ceiling probes (measurement only) ------------------------------------------------------ */

/* What the chip sustains on the two resources these kernels are bound by, for the benchmark to
 * report beside the published peaks (the roofline section 5.3's comparison implies).  Each call
 * only enqueues one kernel on `stream`; the caller times it.  scratch: DEVICE memory, at least
 * s2_probe_scratch_bytes() for s2_probe_mfma and 4 MiB for s2_probe_read, overwritten.
 * s2_probe_mfma: two wavefronts per SIMD issue 32x32x16 bf16 MFMAs back to back on random operands,
 * `iters` trips of 8 each, optionally with a softmax's vector work per MFMA beside them; *flops
 * receives the flops of the launch.  s2_probe_read: reads `bytes` (16-byte aligned) once.
 * Errors: NULL, BAD_PARAM (iters), ALIGN, HIP. */
/* s2_probe_atomic_add: 8192 workgroups add 64 tiles of 32 x 128 floats each into buf (DEVICE, fp32,
 * `bytes` long, at least 1 MiB, 16-byte aligned; its contents are added to) with coalesced fp32
 * atomic adds; *bytes_added receives the bytes of the launch.  It measures what accumulating
 * partial gradients with atomics costs.  Errors: NULL, ALIGN, BAD_PARAM, HIP. */
int s2_probe_atomic_add(void* buf, size_t bytes, void* stream, double* bytes_added);
size_t s2_probe_scratch_bytes(void);
int s2_probe_mfma(int32_t with_vector_work, int32_t iters, void* scratch, void* stream, double* flops);
int s2_probe_read(const void* src, size_t bytes, void* scratch, void* stream);

/* ---- diagnostics -------------------------------------------------------------------------- */

const char* s2_status_string(int status);
/* hipError_t (as int) of the most recent failing HIP call on this thread, 0 if none. */
int s2_last_hip_error(void);
/* Library version, e.g. 100 = 0.1.0. */
int s2_version(void);

#ifdef __cplusplus
}
#endif
#endif /* S2ATTN_H */
