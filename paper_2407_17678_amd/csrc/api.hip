// C ABI of libs2attn.so: argument validation, the layout handle's device copies, and dispatch to
// the kernels.  See include/s2attn.h for the contract of every entry point.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <limits>
#include <new>

#include "../../include/s2attn.h"
#include "config.h"
#include "kernels.h"
#include "layout.h"

namespace {

thread_local int g_last_hip_error = 0;

inline bool hip_ok(hipError_t e) {
  if (e == hipSuccess) return true;
  g_last_hip_error = (int)e;
  return false;
}

bool upload(const std::vector<int32_t>& host, int32_t** dev) {
  *dev = nullptr;
  const size_t bytes = (host.empty() ? 1 : host.size()) * sizeof(int32_t);
  if (!hip_ok(hipMalloc(reinterpret_cast<void**>(dev), bytes))) return false;
  if (host.empty()) return true;
  return hip_ok(hipMemcpy(*dev, host.data(), host.size() * sizeof(int32_t), hipMemcpyHostToDevice));
}

bool upload_tiles(s2::TileList& t) {
  return upload(t.ptr, &t.d_ptr) && upload(t.ent, &t.d_ent) && upload(t.order, &t.d_order) &&
         upload(t.members, &t.d_members);
}

void free_tiles(s2::TileList& t) {
  if (t.d_ptr) (void)hipFree(t.d_ptr);
  if (t.d_ent) (void)hipFree(t.d_ent);
  if (t.d_order) (void)hipFree(t.d_order);
  if (t.d_members) (void)hipFree(t.d_members);
  t.d_ptr = t.d_ent = t.d_order = t.d_members = nullptr;
}

void free_device_copies(s2_layout* L) {
  free_tiles(L->fwd_tiles);
  free_tiles(L->q_tiles);
  free_tiles(L->kv_tiles);
  if (L->d_row_ptr) (void)hipFree(L->d_row_ptr);
  if (L->d_col_idx) (void)hipFree(L->d_col_idx);
  if (L->d_dq_units) (void)hipFree(L->d_dq_units);
  L->d_row_ptr = L->d_col_idx = L->d_dq_units = nullptr;
}

s2::DevTiles dev_tiles(const s2::TileList& t) {
  s2::DevTiles d;
  d.ptr = t.d_ptr;
  d.ent = t.d_ent;
  d.order = t.d_order;
  d.members = t.d_members;
  d.tiles_per_head = t.tiles_per_head;
  d.group = t.group;
  return d;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// The split partials of s2_attn_decode_static live here instead of in a caller's workspace: device
// memory that belongs to the loaded library, one copy per GPU at that GPU's own address, held
// until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the address found there, kept per device, is what the kernels are given.
constexpr size_t kStaticScratchBytes = S2_DECODE_STATIC_SCRATCH_BYTES;
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kScratchMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kScratchMaxDevices];  // zero-initialised: not looked up yet

// Address of `scratch` on the current device, or nullptr (the hipError_t is kept for
// s2_last_hip_error).  The first call on a device asks the runtime; later calls read the slot.
void* scratch_on_current_device() {
  int dev = -1;
  if (!hip_ok(hipGetDevice(&dev))) return nullptr;
  if (dev < 0 || dev >= kScratchMaxDevices) {
    g_last_hip_error = (int)hipErrorInvalidDevice;
    return nullptr;
  }
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr) return ptr;
  if (!hip_ok(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))) || !ptr) return nullptr;
  g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // racing threads store the same address
  return ptr;
}

// Shape / alignment checks shared by forward and backward.  `need_bwd` also checks the
// gradient tensors.
int check_tensors(const s2_tensors* t, bool need_bwd, float scale) {
  if (!t) return S2_ERR_NULL;
  if (!t->q || !t->k || !t->v || !t->o || !t->lse) return S2_ERR_NULL;
  if (need_bwd && (!t->d_o || !t->dq || !t->dk || !t->dv)) return S2_ERR_NULL;
  if (!(scale > 0.f) || !std::isfinite(scale)) return S2_ERR_BAD_PARAM;
  if (t->batch < 1 || t->heads < 1 || t->seqlen < 1) return S2_ERR_SHAPE;
  if (t->head_dim != 64 && t->head_dim != 128) return S2_ERR_SHAPE;
  if ((int64_t)t->batch * t->heads * t->seqlen > (int64_t)1 << 40) return S2_ERR_SHAPE;
  const int64_t strides[6] = {t->q_stride_b, t->q_stride_h, t->q_stride_t,
                              t->kv_stride_b, t->kv_stride_h, t->kv_stride_t};
  for (int64_t s : strides)
    if (s < 0 || (s & 7) != 0) return S2_ERR_ALIGN;
  if (t->q_stride_t < t->head_dim || t->kv_stride_t < t->head_dim) return S2_ERR_ALIGN;
  // the kernels address the 64 rows of a chunk with unsigned 32-bit byte offsets
  if (t->q_stride_t > (1 << 24) || t->kv_stride_t > (1 << 24)) return S2_ERR_SHAPE;
  const void* ptrs[9] = {t->q, t->k, t->v, t->o, t->lse, t->d_o, t->dq, t->dk, t->dv};
  for (int i = 0; i < (need_bwd ? 9 : 5); ++i)
    if (!aligned16(ptrs[i])) return S2_ERR_ALIGN;
  return S2_OK;
}

s2::AttnParams make_params(const s2_tensors* t, float scale) {
  s2::AttnParams p{};
  p.q = static_cast<const uint16_t*>(t->q);
  p.k = static_cast<const uint16_t*>(t->k);
  p.v = static_cast<const uint16_t*>(t->v);
  p.o = static_cast<uint16_t*>(t->o);
  p.lse = t->lse;
  p.d_o = static_cast<const uint16_t*>(t->d_o);
  p.dq = static_cast<uint16_t*>(t->dq);
  p.dk = static_cast<uint16_t*>(t->dk);
  p.dv = static_cast<uint16_t*>(t->dv);
  p.batch = t->batch;
  p.heads = t->heads;
  p.seqlen = t->seqlen;
  p.q_row0 = 0;
  p.q_rows = t->seqlen;
  p.head_dim = t->head_dim;
  p.q_sb = t->q_stride_b;
  p.q_sh = t->q_stride_h;
  p.q_st = t->q_stride_t;
  p.kv_sb = t->kv_stride_b;
  p.kv_sh = t->kv_stride_h;
  p.kv_st = t->kv_stride_t;
  p.scale = scale;
  p.scale_log2e = scale * 1.4426950408889634f;
  return p;
}

// The layout's lists live on the device that was current when it was built.
bool layout_on_current_device(const s2_layout* L) {
  if (!L->on_device) return false;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return dev == L->device;
}

int check_layout_fits(const s2_layout* L, const s2_tensors* t) {
  if (!L) return S2_ERR_NULL;
  if (t->heads != L->p.num_heads) return S2_ERR_SHAPE;
  if ((int64_t)t->seqlen != (int64_t)L->p.num_blocks * L->p.block_size) return S2_ERR_SHAPE;
  return S2_OK;
}

}  // namespace

extern "C" {

namespace {
// Tile lists for the three passes, then the device copy when a GPU is visible.  Takes ownership
// of L: on failure it is deleted.
int finish_layout(s2_layout* L, int st, s2_layout** out) {
  if (st == S2_OK) {
    try {
      const int S = L->p.block_size;
      s2::build_tiles(*L, s2::kFwdBM / S, false, L->fwd_tiles);
      s2::build_tiles(*L, s2::kBwdBM / S, false, L->q_tiles);
      s2::build_tiles(*L, s2::kBwdBN / S, true, L->kv_tiles);
      s2::build_ds_units(*L);
    } catch (const std::bad_alloc&) {
      st = S2_ERR_OVERFLOW;
    }
  }
  if (st != S2_OK) {
    delete L;
    return st;
  }
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) == hipSuccess && ndev > 0) {
    int dev = 0;
    bool ok = hip_ok(hipGetDevice(&dev)) && upload_tiles(L->fwd_tiles) && upload_tiles(L->q_tiles) &&
              upload_tiles(L->kv_tiles) && upload(L->row_ptr, &L->d_row_ptr) &&
              upload(L->col_idx, &L->d_col_idx) && upload(L->dq_units, &L->d_dq_units);
    if (!ok) {
      free_device_copies(L);
      delete L;
      return S2_ERR_HIP;
    }
    L->device = dev;
    L->on_device = true;
  } else {
    (void)hipGetLastError();  // no GPU: a host-only layout is still a valid result
  }
  *out = L;
  return S2_OK;
}
}  // namespace

int s2_layout_build(const s2_layout_params* params, s2_layout** out) {
  if (!params || !out) return S2_ERR_NULL;
  *out = nullptr;
  s2_layout* L = new (std::nothrow) s2_layout();
  if (!L) return S2_ERR_OVERFLOW;
  int st;
  try {
    st = s2::build_host(*params, *L);
  } catch (const std::bad_alloc&) {
    st = S2_ERR_OVERFLOW;
  }
  return finish_layout(L, st, out);
}

int s2_layout_from_csr(int32_t num_heads, int32_t num_blocks, int32_t block_size, const int32_t* row_ptr,
                       const int32_t* col_idx, s2_layout** out) {
  if (!row_ptr || !col_idx || !out) return S2_ERR_NULL;
  *out = nullptr;
  s2_layout* L = new (std::nothrow) s2_layout();
  if (!L) return S2_ERR_OVERFLOW;
  int st;
  try {
    st = s2::build_from_csr(num_heads, num_blocks, block_size, row_ptr, col_idx, *L);
  } catch (const std::bad_alloc&) {
    st = S2_ERR_OVERFLOW;
  }
  return finish_layout(L, st, out);
}

int s2_layout_destroy(s2_layout* layout) {
  if (!layout) return S2_ERR_NULL;
  if (layout->on_device) free_device_copies(layout);
  delete layout;
  return S2_OK;
}

int s2_layout_get(const s2_layout* L, s2_layout_view* out) {
  if (!L || !out) return S2_ERR_NULL;
  out->row_ptr = L->row_ptr.data();
  out->col_idx = L->col_idx.data();
  out->col_ptr = L->col_ptr.data();
  out->row_idx = L->row_idx.data();
  out->nnz = L->nnz;
  out->num_heads = L->p.num_heads;
  out->num_blocks = L->p.num_blocks;
  out->block_size = L->p.block_size;
  out->max_row_blocks = L->max_row_blocks;
  out->covers_all = L->covers_all;
  out->on_device = L->on_device ? 1 : 0;
  return S2_OK;
}

int s2_layout_get_tiles(const s2_layout* L, int which, s2_tile_view* out) {
  if (!L || !out) return S2_ERR_NULL;
  if (which != S2_TILES_FWD && which != S2_TILES_DQ && which != S2_TILES_DKDV) return S2_ERR_BAD_PARAM;
  const s2::TileList& t = which == S2_TILES_FWD ? L->fwd_tiles : which == S2_TILES_DQ ? L->q_tiles : L->kv_tiles;
  out->ptr = t.ptr.data();
  out->ent = t.ent.data();
  out->order = t.order.data();
  out->members = t.members.data();
  out->tiles_per_head = t.tiles_per_head;
  out->group = t.group;
  out->blocks_per_unit = L->p.block_size < 32 ? 32 / L->p.block_size : 1;
  return S2_OK;
}

int s2_layout_get_ds_units(const s2_layout* L, s2_ds_units_view* out) {
  if (!L || !out) return S2_ERR_NULL;
  out->dq_units = L->dq_units.data();
  out->count = (int64_t)L->dq_units.size();
  out->ds_units = L->ds_units;
  return S2_OK;
}

int s2_attn_fwd(const s2_layout* layout, const s2_tensors* t, float scale, void* stream) {
  if (!layout) return S2_ERR_NULL;
  int st = check_tensors(t, false, scale);
  if (st != S2_OK) return st;
  st = check_layout_fits(layout, t);
  if (st != S2_OK) return st;
  if (!layout_on_current_device(layout)) return S2_ERR_NO_DEVICE;
  s2::AttnParams p = make_params(t, scale);
  p.block_size = layout->p.block_size;
  p.fwd_tiles = dev_tiles(layout->fwd_tiles);
  p.q_tiles = dev_tiles(layout->q_tiles);
  p.kv_tiles = dev_tiles(layout->kv_tiles);
  return hip_ok(s2::launch_fwd(p, false, static_cast<hipStream_t>(stream))) ? S2_OK : S2_ERR_HIP;
}

size_t s2_attn_bwd_workspace_bytes(int32_t batch, int32_t heads, int32_t seqlen, int32_t head_dim) {
  (void)head_dim;
  if (batch < 1 || heads < 1 || seqlen < 1) return 0;
  const size_t rows = (size_t)batch * heads * seqlen;
  // delta = rowsum(dO * O) and a copy of LSE in base-2 units, 256-byte aligned each
  return 2 * (((rows * sizeof(float) + 255) / 256) * 256);
}

namespace {
// The backward that keeps dS covers head_dim 128, mask blocks of 64 or 128 tokens (the layout then
// carries the unit table) and whole 128-row tiles.
bool keeps_ds(const s2_layout* L, int32_t seqlen, int32_t head_dim) {
  return L->ds_units > 0 && head_dim == 128 && seqlen % s2::kBwdBM == 0 &&
         (int64_t)seqlen == (int64_t)L->p.num_blocks * L->p.block_size;
}
}  // namespace

size_t s2_attn_bwd_layout_workspace_bytes(const s2_layout* layout, int32_t batch, int32_t heads, int32_t seqlen,
                                          int32_t head_dim) {
  const size_t small = s2_attn_bwd_workspace_bytes(batch, heads, seqlen, head_dim);
  if (!layout || small == 0 || heads != layout->p.num_heads || !keeps_ds(layout, seqlen, head_dim)) return small;
  return small + (size_t)batch * (size_t)layout->ds_units * 8192;
}

int s2_attn_bwd(const s2_layout* layout, const s2_tensors* t, float scale, void* workspace,
                size_t workspace_bytes, void* stream) {
  return s2_attn_bwd_stages(layout, t, scale, workspace, workspace_bytes, S2_BWD_ALL, stream);
}

int s2_attn_fwd_rows(const s2_layout* layout, const s2_tensors* t, int32_t q_row_start, int32_t q_rows,
                     float scale, void* stream) {
  if (!layout) return S2_ERR_NULL;
  int st = check_tensors(t, false, scale);
  if (st != S2_OK) return st;
  if (t->heads != layout->p.num_heads) return S2_ERR_SHAPE;
  if ((int64_t)t->seqlen > (int64_t)layout->p.num_blocks * layout->p.block_size) return S2_ERR_SHAPE;
  if (q_row_start < 0 || q_rows < s2::kFwdBM || q_row_start % s2::kFwdBM != 0 || q_rows % s2::kFwdBM != 0)
    return S2_ERR_SHAPE;
  if ((int64_t)q_row_start + q_rows > t->seqlen) return S2_ERR_SHAPE;
  if (!layout_on_current_device(layout)) return S2_ERR_NO_DEVICE;
  s2::AttnParams p = make_params(t, scale);
  p.q_row0 = q_row_start;
  p.q_rows = q_rows;
  p.block_size = layout->p.block_size;
  p.fwd_tiles = dev_tiles(layout->fwd_tiles);
  p.q_tiles = dev_tiles(layout->q_tiles);
  p.kv_tiles = dev_tiles(layout->kv_tiles);
  return hip_ok(s2::launch_fwd(p, false, static_cast<hipStream_t>(stream))) ? S2_OK : S2_ERR_HIP;
}

int s2_attn_fwd_varlen(const s2_layout* layout, const s2_tensors* t, const int32_t* cu_seqlens,
                       int32_t num_seqs, int32_t max_seqlen, float scale, void* stream) {
  if (!layout || !cu_seqlens) return S2_ERR_NULL;
  int st = check_tensors(t, false, scale);
  if (st != S2_OK) return st;
  if (t->batch != 1 || t->heads != layout->p.num_heads) return S2_ERR_SHAPE;
  if (num_seqs < 1 || max_seqlen < 1) return S2_ERR_SHAPE;
  if ((int64_t)max_seqlen > (int64_t)layout->p.num_blocks * layout->p.block_size) return S2_ERR_SHAPE;
  if ((int64_t)num_seqs * t->heads > std::numeric_limits<int32_t>::max() / 2) return S2_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(cu_seqlens) & 3u) != 0) return S2_ERR_ALIGN;
  if (!layout_on_current_device(layout)) return S2_ERR_NO_DEVICE;
  s2::AttnParams p = make_params(t, scale);
  p.batch = num_seqs;
  p.q_rows = max_seqlen;
  p.cu_seqlens = cu_seqlens;
  p.block_size = layout->p.block_size;
  p.fwd_tiles = dev_tiles(layout->fwd_tiles);
  p.q_tiles = dev_tiles(layout->q_tiles);
  p.kv_tiles = dev_tiles(layout->kv_tiles);
  // one grid slot per (sequence, head, 128-row tile of the longest length allowed)
  const int64_t slots = 8 * (((int64_t)num_seqs * t->heads + 7) / 8) * ((max_seqlen + s2::kFwdBM - 1) / s2::kFwdBM);
  if (slots > std::numeric_limits<int32_t>::max()) return S2_ERR_SHAPE;
  return hip_ok(s2::launch_fwd(p, false, static_cast<hipStream_t>(stream))) ? S2_OK : S2_ERR_HIP;
}

size_t s2_attn_bwd_varlen_workspace_bytes(int32_t heads, int32_t rows, int32_t head_dim) {
  (void)head_dim;
  if (heads < 1 || rows < 1) return 0;
  // delta and base-2 LSE per (head, row), plus one chunk of slack each: the dK/dV kernel fetches the
  // statistics of a whole 64-row chunk even where a sequence ends inside it
  const size_t floats = (size_t)heads * rows + 64;
  return 2 * (((floats * sizeof(float) + 255) / 256) * 256);
}

int s2_attn_bwd_varlen(const s2_layout* layout, const s2_tensors* t, const int32_t* cu_seqlens,
                       int32_t num_seqs, int32_t max_seqlen, float scale, void* workspace,
                       size_t workspace_bytes, void* stream) {
  if (!layout || !cu_seqlens) return S2_ERR_NULL;
  int st = check_tensors(t, true, scale);
  if (st != S2_OK) return st;
  if (t->batch != 1 || t->heads != layout->p.num_heads) return S2_ERR_SHAPE;
  if (num_seqs < 1 || max_seqlen < 1) return S2_ERR_SHAPE;
  if ((int64_t)max_seqlen > (int64_t)layout->p.num_blocks * layout->p.block_size) return S2_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(cu_seqlens) & 3u) != 0) return S2_ERR_ALIGN;
  const size_t need = s2_attn_bwd_varlen_workspace_bytes(t->heads, t->seqlen, t->head_dim);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || workspace_bytes < need)
    return S2_ERR_WORKSPACE;
  if (!layout_on_current_device(layout)) return S2_ERR_NO_DEVICE;
  s2::AttnParams p = make_params(t, scale);
  p.batch = num_seqs;
  p.q_rows = max_seqlen;
  p.cu_seqlens = cu_seqlens;
  p.block_size = layout->p.block_size;
  p.fwd_tiles = dev_tiles(layout->fwd_tiles);
  p.q_tiles = dev_tiles(layout->q_tiles);
  p.kv_tiles = dev_tiles(layout->kv_tiles);
  p.delta = static_cast<float*>(workspace);
  p.lse2 = p.delta + need / 8;
  // one grid slot per (sequence, head, tile): query tiles of the longest length allowed, key tiles of the layout
  const int64_t pairs = 8 * (((int64_t)num_seqs * t->heads + 7) / 8);
  const int64_t slots = pairs * std::max<int64_t>((max_seqlen + s2::kBwdBM - 1) / s2::kBwdBM, layout->kv_tiles.tiles_per_head);
  if (slots > std::numeric_limits<int32_t>::max()) return S2_ERR_SHAPE;
  return hip_ok(s2::launch_bwd(p, false, s2::kBwdAll, static_cast<hipStream_t>(stream))) ? S2_OK : S2_ERR_HIP;
}

int s2_attn_bwd_stages(const s2_layout* layout, const s2_tensors* t, float scale, void* workspace,
                       size_t workspace_bytes, int stages, void* stream) {
  if (!layout) return S2_ERR_NULL;
  if (stages < 1 || stages > S2_BWD_ALL) return S2_ERR_BAD_PARAM;
  int st = check_tensors(t, true, scale);
  if (st != S2_OK) return st;
  st = check_layout_fits(layout, t);
  if (st != S2_OK) return st;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 ||
      workspace_bytes < s2_attn_bwd_workspace_bytes(t->batch, t->heads, t->seqlen, t->head_dim))
    return S2_ERR_WORKSPACE;
  if (!layout_on_current_device(layout)) return S2_ERR_NO_DEVICE;
  s2::AttnParams p = make_params(t, scale);
  p.delta = static_cast<float*>(workspace);
  p.lse2 = p.delta + s2_attn_bwd_workspace_bytes(t->batch, t->heads, t->seqlen, t->head_dim) / 8;
  p.block_size = layout->p.block_size;
  p.fwd_tiles = dev_tiles(layout->fwd_tiles);
  p.q_tiles = dev_tiles(layout->q_tiles);
  p.kv_tiles = dev_tiles(layout->kv_tiles);
  // a workspace large enough to keep dS selects the backward that computes nothing twice
  const size_t small = s2_attn_bwd_workspace_bytes(t->batch, t->heads, t->seqlen, t->head_dim);
  if (keeps_ds(layout, t->seqlen, t->head_dim) &&
      workspace_bytes >= s2_attn_bwd_layout_workspace_bytes(layout, t->batch, t->heads, t->seqlen, t->head_dim)) {
    p.ds_store = reinterpret_cast<uint16_t*>(static_cast<unsigned char*>(workspace) + small);
    p.ds_units = layout->ds_units;
    p.dq_units = layout->d_dq_units;
  }
  return hip_ok(s2::launch_bwd(p, false, stages, static_cast<hipStream_t>(stream))) ? S2_OK : S2_ERR_HIP;
}

static int dense_params(const s2_tensors* t, s2::AttnParams& p) {
  if (t->seqlen % 128 != 0) return S2_ERR_SHAPE;
  p.block_size = s2::kChunk;
  p.fwd_tiles.tiles_per_head = (t->seqlen + s2::kFwdBM - 1) / s2::kFwdBM;
  p.fwd_tiles.group = s2::kFwdBM / s2::kChunk;
  p.q_tiles.tiles_per_head = t->seqlen / s2::kBwdBM;
  p.q_tiles.group = s2::kBwdBM / s2::kChunk;
  p.kv_tiles.tiles_per_head = t->seqlen / s2::kBwdBN;
  p.kv_tiles.group = s2::kBwdBN / s2::kChunk;
  return S2_OK;
}

int s2_dense_causal_fwd(const s2_tensors* t, float scale, void* stream) {
  int st = check_tensors(t, false, scale);
  if (st != S2_OK) return st;
  s2::AttnParams p = make_params(t, scale);
  st = dense_params(t, p);
  if (st != S2_OK) return st;
  return hip_ok(s2::launch_fwd(p, true, static_cast<hipStream_t>(stream))) ? S2_OK : S2_ERR_HIP;
}

int s2_dense_causal_bwd(const s2_tensors* t, float scale, void* workspace, size_t workspace_bytes,
                        void* stream) {
  int st = check_tensors(t, true, scale);
  if (st != S2_OK) return st;
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 ||
      workspace_bytes < s2_attn_bwd_workspace_bytes(t->batch, t->heads, t->seqlen, t->head_dim))
    return S2_ERR_WORKSPACE;
  s2::AttnParams p = make_params(t, scale);
  st = dense_params(t, p);
  if (st != S2_OK) return st;
  p.delta = static_cast<float*>(workspace);
  p.lse2 = p.delta + s2_attn_bwd_workspace_bytes(t->batch, t->heads, t->seqlen, t->head_dim) / 8;
  return hip_ok(s2::launch_bwd(p, true, s2::kBwdAll, static_cast<hipStream_t>(stream))) ? S2_OK : S2_ERR_HIP;
}

int32_t s2_attn_decode_default_splits(int32_t nseq, int32_t heads, int32_t max_len) {
  if (nseq < 1 || heads < 1 || max_len < 1) return 1;
  // aim for a few workgroups per compute unit (256 CUs); never more splits than 1K-token pieces
  const int64_t pairs = (int64_t)nseq * heads;
  int64_t want = (4 * 256 + pairs - 1) / pairs;
  const int64_t cap = (max_len + 1023) / 1024;
  if (want > cap) want = cap;
  if (want < 1) want = 1;
  if (want > 64) want = 64;
  return (int32_t)want;
}

size_t s2_attn_decode_workspace_bytes(int32_t nseq, int32_t heads, int32_t head_dim, int32_t max_len,
                                      int32_t num_splits) {
  if (nseq < 1 || heads < 1 || head_dim < 1) return 0;
  if (num_splits <= 0) num_splits = s2_attn_decode_default_splits(nseq, heads, max_len);
  const size_t items = (size_t)nseq * heads * num_splits;
  return ((items * (head_dim + 2) * sizeof(float) + 255) / 256) * 256;
}

namespace {

bool good_block_size(int S) { return S == 16 || S == 32 || S == 64 || S == 128; }

// The pattern a decode call follows: the closed form of `lp`, or, when `layout` is given, the
// layout's own rows (then lp = &layout->p supplies S and the head count only).
int check_pattern(const s2_layout_params* lp, const s2_layout* layout, int heads, int64_t max_len) {
  if (!good_block_size(lp->block_size)) return S2_ERR_BAD_PARAM;
  if (heads != lp->num_heads) return S2_ERR_SHAPE;
  if (layout) {
    if (max_len > (int64_t)lp->num_blocks * lp->block_size) return S2_ERR_SHAPE;
    return layout_on_current_device(layout) ? S2_OK : S2_ERR_NO_DEVICE;
  }
  if (lp->dense != 0 && lp->dense != 1) return S2_ERR_BAD_PARAM;
  if (!lp->dense && (lp->local_blocks < 1 || lp->stride < 0 || lp->window_blocks < 0)) return S2_ERR_BAD_PARAM;
  if (lp->head_index_base < 0) return S2_ERR_BAD_PARAM;
  return S2_OK;
}

// Split count when the caller leaves it to the library: the public default (enough workgroups to
// fill the chip; it also sizes the workspace, so never more than that), cut down so that a
// workgroup still has about a dozen 64-token units of the longest row to walk: with fewer, its four
// wavefronts mostly idle and the reduce kernel merges partials for nothing.
int choose_splits(const s2_layout_params* lp, const s2_layout* layout, int nseq, int heads, int max_len) {
  int splits = s2_attn_decode_default_splits(nseq, heads, max_len);
  const int S = lp->block_size;
  int64_t blocks = layout ? layout->max_row_blocks : s2::row_blocks(*lp, 0, (max_len - 1) / S, nullptr, 0);
  const int64_t units = blocks * S / 64;  // 64-token units of work in the longest row
  const int64_t cap = units / 12 < 1 ? 1 : units / 12;
  if (splits > cap) splits = (int)cap;
  return splits;
}

void set_pattern(s2::DecodeParams& p, const s2_layout_params* lp, const s2_layout* layout) {
  p.block_size = lp->block_size;
  p.local_blocks = lp->local_blocks;
  p.stride = lp->stride;
  p.window_blocks = lp->window_blocks;
  p.dense = lp->dense;
  p.head_index_base = lp->head_index_base;
  if (layout) {
    p.row_ptr = layout->d_row_ptr;
    p.col_idx = layout->d_col_idx;
    p.num_blocks = lp->num_blocks;
  }
}

int decode_contiguous(const s2_layout_params* lp, const s2_layout* layout, const s2_decode_args* a, float scale,
                      void* workspace, size_t workspace_bytes, void* stream) {
  if (!a->q || !a->k_cache || !a->v_cache || !a->seq_lens || !a->o) return S2_ERR_NULL;
  if (!(scale > 0.f) || !std::isfinite(scale)) return S2_ERR_BAD_PARAM;
  if (a->nseq < 1 || a->heads < 1 || a->max_len < 1) return S2_ERR_SHAPE;
  if (a->head_dim != 64 && a->head_dim != 128) return S2_ERR_SHAPE;
  int st = check_pattern(lp, layout, a->heads, a->max_len);
  if (st != S2_OK) return st;
  if (a->num_splits < 0 || a->num_splits > 64) return S2_ERR_BAD_PARAM;
  const int64_t strides[3] = {a->kv_stride_seq, a->kv_stride_head, a->kv_stride_tok};
  for (int64_t s : strides)
    if (s < 0 || (s & 7) != 0) return S2_ERR_ALIGN;
  if (a->kv_stride_tok < a->head_dim) return S2_ERR_ALIGN;
  if (!aligned16(a->q) || !aligned16(a->k_cache) || !aligned16(a->v_cache) || !aligned16(a->o) ||
      (reinterpret_cast<uintptr_t>(a->seq_lens) & 3u) != 0)
    return S2_ERR_ALIGN;
  const int splits = a->num_splits > 0 ? a->num_splits : choose_splits(lp, layout, a->nseq, a->heads, a->max_len);
  const size_t need = s2_attn_decode_workspace_bytes(a->nseq, a->heads, a->head_dim, a->max_len, splits);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || workspace_bytes < need)
    return S2_ERR_WORKSPACE;

  s2::DecodeParams p{};
  p.q = static_cast<const uint16_t*>(a->q);
  p.k_cache = static_cast<const uint16_t*>(a->k_cache);
  p.v_cache = static_cast<const uint16_t*>(a->v_cache);
  p.seq_lens = a->seq_lens;
  p.o = static_cast<uint16_t*>(a->o);
  p.lse = a->lse;
  const size_t items = (size_t)a->nseq * a->heads * splits;
  p.part_acc = static_cast<float*>(workspace);
  p.part_ml = p.part_acc + items * a->head_dim;
  p.nseq = a->nseq;
  p.heads = a->heads;
  p.head_dim = a->head_dim;
  p.max_len = a->max_len;
  p.num_splits = splits;
  p.kv_ss = a->kv_stride_seq;
  p.kv_sh = a->kv_stride_head;
  p.kv_st = a->kv_stride_tok;
  p.scale = scale;
  p.scale_log2e = scale * 1.4426950408889634f;
  set_pattern(p, lp, layout);
  return hip_ok(s2::launch_decode(p, static_cast<hipStream_t>(stream))) ? S2_OK : S2_ERR_HIP;
}

int decode_paged(const s2_layout_params* lp, const s2_layout* layout, const s2_paged_decode_args* a, float scale,
                 void* workspace, size_t workspace_bytes, void* stream) {
  if (!a->q || !a->k_pages || !a->v_pages || !a->block_table || !a->seq_lens || !a->o) return S2_ERR_NULL;
  if (!(scale > 0.f) || !std::isfinite(scale)) return S2_ERR_BAD_PARAM;
  if (!good_block_size(lp->block_size)) return S2_ERR_BAD_PARAM;
  if (a->nseq < 1 || a->heads < 1 || a->max_blocks < 1 || a->num_pages < 1) return S2_ERR_SHAPE;
  if ((int64_t)a->max_blocks * lp->block_size > std::numeric_limits<int32_t>::max()) return S2_ERR_SHAPE;
  if (a->head_dim != 64 && a->head_dim != 128) return S2_ERR_SHAPE;
  const int max_len = a->max_blocks * lp->block_size;
  int st = check_pattern(lp, layout, a->heads, max_len);
  if (st != S2_OK) return st;
  if (a->num_splits < 0 || a->num_splits > 64) return S2_ERR_BAD_PARAM;
  if (a->page_stride < 0 || (a->page_stride & 7) != 0 || a->tok_stride < 0 || (a->tok_stride & 7) != 0)
    return S2_ERR_ALIGN;
  if (a->tok_stride < a->head_dim) return S2_ERR_ALIGN;
  if (!aligned16(a->q) || !aligned16(a->k_pages) || !aligned16(a->v_pages) || !aligned16(a->o) ||
      (reinterpret_cast<uintptr_t>(a->seq_lens) & 3u) != 0 ||
      (reinterpret_cast<uintptr_t>(a->block_table) & 3u) != 0 ||
      (reinterpret_cast<uintptr_t>(a->missing) & 3u) != 0)
    return S2_ERR_ALIGN;
  const int splits = a->num_splits > 0 ? a->num_splits : choose_splits(lp, layout, a->nseq, a->heads, max_len);
  const size_t need = s2_attn_decode_workspace_bytes(a->nseq, a->heads, a->head_dim, max_len, splits);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0 || workspace_bytes < need)
    return S2_ERR_WORKSPACE;

  s2::DecodeParams p{};
  p.q = static_cast<const uint16_t*>(a->q);
  p.k_cache = static_cast<const uint16_t*>(a->k_pages);
  p.v_cache = static_cast<const uint16_t*>(a->v_pages);
  p.seq_lens = a->seq_lens;
  p.o = static_cast<uint16_t*>(a->o);
  p.lse = a->lse;
  const size_t items = (size_t)a->nseq * a->heads * splits;
  p.part_acc = static_cast<float*>(workspace);
  p.part_ml = p.part_acc + items * a->head_dim;
  p.nseq = a->nseq;
  p.heads = a->heads;
  p.head_dim = a->head_dim;
  p.max_len = max_len;
  p.num_splits = splits;
  p.kv_ss = a->page_stride;
  p.kv_sh = 0;
  p.kv_st = a->tok_stride;
  p.scale = scale;
  p.scale_log2e = scale * 1.4426950408889634f;
  set_pattern(p, lp, layout);
  p.block_table = a->block_table;
  p.missing = a->missing;
  p.max_blocks = a->max_blocks;
  p.num_pages = a->num_pages;
  return hip_ok(s2::launch_decode(p, static_cast<hipStream_t>(stream))) ? S2_OK : S2_ERR_HIP;
}

}  // namespace

int s2_attn_decode(const s2_layout_params* lp, const s2_decode_args* a, float scale, void* workspace,
                   size_t workspace_bytes, void* stream) {
  if (!lp || !a) return S2_ERR_NULL;
  return decode_contiguous(lp, nullptr, a, scale, workspace, workspace_bytes, stream);
}

int s2_attn_decode_static(const s2_layout_params* lp, const s2_decode_args* a, float scale, void* stream) {
  if (!lp || !a) return S2_ERR_NULL;
  // the size check comes first and needs no device: shapes whose partials do not fit are refused
  if (a->nseq < 1 || a->heads < 1 || a->max_len < 1) return S2_ERR_SHAPE;
  if (a->head_dim != 64 && a->head_dim != 128) return S2_ERR_SHAPE;
  if (a->num_splits < 0 || a->num_splits > 64) return S2_ERR_BAD_PARAM;
  // num_splits == 0: the call may pick fewer splits than this bound, never more
  const size_t need = s2_attn_decode_workspace_bytes(a->nseq, a->heads, a->head_dim, a->max_len, a->num_splits);
  if (need > kStaticScratchBytes) return S2_ERR_WORKSPACE;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) {
    (void)hipGetLastError();
    return S2_ERR_NO_DEVICE;
  }
  void* ptr = scratch_on_current_device();
  if (!ptr) return S2_ERR_HIP;
  return decode_contiguous(lp, nullptr, a, scale, ptr, kStaticScratchBytes, stream);
}

int s2_attn_decode_paged(const s2_layout_params* lp, const s2_paged_decode_args* a, float scale,
                         void* workspace, size_t workspace_bytes, void* stream) {
  if (!lp || !a) return S2_ERR_NULL;
  return decode_paged(lp, nullptr, a, scale, workspace, workspace_bytes, stream);
}

int s2_attn_decode_layout(const s2_layout* layout, const s2_decode_args* a, float scale, void* workspace,
                          size_t workspace_bytes, void* stream) {
  if (!layout || !a) return S2_ERR_NULL;
  return decode_contiguous(&layout->p, layout, a, scale, workspace, workspace_bytes, stream);
}

int s2_attn_decode_paged_layout(const s2_layout* layout, const s2_paged_decode_args* a, float scale,
                                void* workspace, size_t workspace_bytes, void* stream) {
  if (!layout || !a) return S2_ERR_NULL;
  return decode_paged(&layout->p, layout, a, scale, workspace, workspace_bytes, stream);
}

int s2_layout_resident_blocks(const s2_layout* L, int32_t head, int32_t length, int32_t* blocks,
                              int32_t capacity, int32_t* count) {
  if (!L || !count) return S2_ERR_NULL;
  if (capacity < 0 || (capacity > 0 && !blocks)) return S2_ERR_NULL;
  const int B = L->p.num_blocks, S = L->p.block_size;
  if (head < 0 || head >= L->p.num_heads || length < 1 || (int64_t)length > (int64_t)B * S)
    return S2_ERR_BAD_PARAM;
  // A block among 0..i (i = row of the newest token) stays while row i or any later row keeps it:
  // walk each such column's list of attending rows (ascending) and look at its last entry.
  const int i = (length - 1) / S;
  int64_t n = 0;
  for (int j = 0; j <= i; ++j) {
    const int32_t lo = L->col_ptr[(size_t)head * B + j], hi = L->col_ptr[(size_t)head * B + j + 1];
    if (hi > lo && L->row_idx[hi - 1] >= i) {
      if (n < capacity) blocks[n] = j;
      ++n;
    }
  }
  *count = (int32_t)n;
  return n > capacity ? S2_ERR_OVERFLOW : S2_OK;
}

int s2_kv_resident_blocks(const s2_layout_params* lp, int32_t head, int32_t length, int32_t* blocks,
                          int32_t capacity, int32_t* count) {
  if (!lp || !count) return S2_ERR_NULL;
  if (capacity < 0 || (capacity > 0 && !blocks)) return S2_ERR_NULL;
  if (!good_block_size(lp->block_size)) return S2_ERR_BAD_PARAM;
  if (lp->dense != 0 && lp->dense != 1) return S2_ERR_BAD_PARAM;
  if (!lp->dense && (lp->local_blocks < 1 || lp->stride < 0 || lp->window_blocks < 0)) return S2_ERR_BAD_PARAM;
  if (lp->head_index_base < 0 || lp->num_heads < 1) return S2_ERR_BAD_PARAM;
  if (head < 0 || head >= lp->num_heads || length < 1) return S2_ERR_BAD_PARAM;
  // Every block a later row keeps among blocks 0..i is also kept by row i = (length-1) div S
  // (the mask only loses columns as the row index grows: a local block drops out of the window,
  // a stripe block stays until the optional window passes it), so the answer is row i itself.
  const int i = (length - 1) / lp->block_size;
  const int64_t n = s2::row_blocks(*lp, head, i, blocks, capacity);
  *count = (int32_t)n;
  return n > capacity ? S2_ERR_OVERFLOW : S2_OK;
}

const char* s2_status_string(int status) {
  switch (status) {
    case S2_OK: return "ok";
    case S2_ERR_NULL: return "a required pointer is NULL";
    case S2_ERR_BAD_PARAM: return "parameter out of range";
    case S2_ERR_SHAPE: return "tensor shape does not fit";
    case S2_ERR_ALIGN: return "pointer or stride not aligned";
    case S2_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case S2_ERR_HIP: return "HIP runtime error";
    case S2_ERR_NO_DEVICE: return "layout has no device copy";
    case S2_ERR_OVERFLOW: return "size overflow or out of memory";
    default: return "unknown status";
  }
}

int s2_last_hip_error(void) { return g_last_hip_error; }
int s2_version(void) { return 100; }

}  // extern "C"
