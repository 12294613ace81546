// Internal: parameter blocks and launch entry points of the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace s2 {

// Merged tile list on the device (see TileList in layout.h).
struct DevTiles {
  const int32_t* ptr = nullptr;
  const int32_t* ent = nullptr;
  const int32_t* order = nullptr;
  const int32_t* members = nullptr;  // block index of each tile member (-1 = none)
  int tiles_per_head = 0;
  int group = 0;
};

struct AttnParams {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  uint16_t* o;
  float* lse;
  const uint16_t* d_o;
  uint16_t* dq;
  uint16_t* dk;
  uint16_t* dv;
  float* delta;  // workspace: rowsum(dO * O), [batch, heads, seqlen]
  float* lse2;   // workspace: lse * log2(e), [batch, heads, seqlen]
  int batch, heads, seqlen, head_dim;
  // forward only: q, o, lse hold q_rows rows, local row r being sequence position q_row0 + r
  // (the whole sequence: q_row0 = 0, q_rows = seqlen)
  int q_row0, q_rows;
  // packed variable-length batch (forward only; nullptr = every sequence has seqlen rows):
  // sequence b owns rows cu_seqlens[b] .. cu_seqlens[b+1]-1 of q, k, v, o and lse; then batch is
  // the number of sequences, seqlen the rows in the tensors and q_rows the longest length allowed
  const int32_t* cu_seqlens;
  // packed batch, set by the launch code: 0 = the launch covers every 128-row tile of every sequence;
  // 1 = only each sequence's last tile, and only where that tile is a partial one (the tiles before it
  // are then computed by the fast-path kernel, which takes whole tiles only)
  int varlen_tail;
  int64_t q_sb, q_sh, q_st;
  int64_t kv_sb, kv_sh, kv_st;
  float scale;        // softmax scale
  float scale_log2e;  // scale * log2(e)
  int block_size;     // S (sparse path); 64 on the dense path
  DevTiles fwd_tiles; // row tiles of the forward kernel -> KV blocks
  DevTiles q_tiles;   // row tiles of the dQ kernel -> KV blocks
  DevTiles kv_tiles;  // column tiles -> Q blocks
  // Backward with dS kept (head_dim 128, mask blocks of 64 or 128 tokens): the dK/dV kernel leaves
  // dS = P * (dP - delta), rounded to bf16, in the workspace, in units of 64 queries x 64 keys (8 KiB),
  // unit (2 * step + wavefront pair) of its walk; the dQ launch is then the one contraction dS K over
  // those units.  ds_store == nullptr: dS is not kept and the dQ kernel recomputes it.
  uint16_t* ds_store;          // [batch][ds_units] units
  int64_t ds_units;            // units per batch element
  const int32_t* dq_units;     // [dQ list chunk][query half of the 128-row tile]: unit, -1 = none
};

struct DecodeParams {
  const uint16_t* q;
  const uint16_t* k_cache;
  const uint16_t* v_cache;
  const int32_t* seq_lens;
  uint16_t* o;
  float* lse;
  float* part_acc;  // [nseq*heads*splits, head_dim]
  float* part_ml;   // [nseq*heads*splits, 2]  (max, sum)
  int nseq, heads, head_dim, max_len, num_splits;
  int64_t kv_ss, kv_sh, kv_st;
  float scale, scale_log2e;
  int block_size, local_blocks, stride, window_blocks, dense, head_index_base;
  // paged cache: k_cache / v_cache are the page pools, kv_ss is the page stride
  const int32_t* block_table;  // [nseq, heads, max_blocks], nullptr = contiguous cache
  int32_t* missing;            // optional counter of kept blocks that are not resident
  int max_blocks, num_pages;
  // caller-supplied pattern: the kept blocks of row i of head h are
  // col_idx[row_ptr[h*num_blocks + i] .. row_ptr[h*num_blocks + i + 1]); nullptr = closed form
  const int32_t* row_ptr;
  const int32_t* col_idx;
  int num_blocks;
};

// Each returns the hipError_t of the launch (hipGetLastError after the launch).
hipError_t launch_fwd(const AttnParams& p, bool dense, hipStream_t stream);
// The forward's fast path (head_dim 128, mask blocks of 64 or 128 tokens, whole 128-row tiles; of a
// packed batch the whole tiles of each sequence): whether it covers a call, and its launch.  launch_fwd
// uses it where it applies.
bool fwd_pipe_applies(const AttnParams& p, bool dense);
hipError_t launch_fwd_pipe(const AttnParams& p, bool dense, hipStream_t stream);
// `stages` selects which of the three backward launches run: 1 = delta, 2 = dK/dV, 4 = dQ.
constexpr int kBwdDelta = 1, kBwdDkDv = 2, kBwdDq = 4, kBwdAll = 7;
hipError_t launch_bwd(const AttnParams& p, bool dense, int stages, hipStream_t stream);
// The dQ launch's fast path (head_dim 128, mask blocks of 64 or 128 tokens, whole 128-row tiles - of a
// packed batch the whole tiles of each sequence; it also leaves delta and base-2 LSE in the workspace):
// whether it covers a call, and its launch.  launch_bwd uses it where it applies.
bool dq_pipe_applies(const AttnParams& p, bool dense);
hipError_t launch_dq_pipe(const AttnParams& p, bool dense, hipStream_t stream);
// The dQ launch of the backward that keeps dS: dQ = scale * dS K over the stored units.
hipError_t launch_dq_gemm(const AttnParams& p, hipStream_t stream);
hipError_t launch_decode(const DecodeParams& p, hipStream_t stream);

}  // namespace s2
