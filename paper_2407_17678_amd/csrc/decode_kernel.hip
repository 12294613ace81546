// Decode: one query token per sequence against a contiguous KV cache (section 4.1).  The query
// at position L-1 reads only the KV blocks that block row (L-1) div S of the head's mask keeps:
// the head's vertical stripes plus the local window (section 4.2), enumerated in closed form.
// The work is one multiply-add per byte read, so the kernel is a bandwidth kernel: every lane
// issues 16-byte loads, a row of K or V is covered by D/8 adjacent lanes, and both the K and V
// loads of a 64-token unit are in flight before the first score is needed.
//
// A caller-supplied pattern replaces the closed form by row (L-1) div S of the layout's lists.
//
// Paged cache (PAGED = true): a kept block's rows are found through the block table instead of
// by offset into a contiguous cache; nothing else changes, since a page is one contiguous block.
//
// Split-KV: the list of 64-token units of one (sequence, head) is cut into num_splits pieces, one
// workgroup each; the four wavefronts of a workgroup take units round-robin and merge their
// (max, sum, accumulator) through LDS; a second kernel merges the splits.  With one split per
// (sequence, head) the first kernel writes the result itself and the second is not launched.
#include <hip/hip_runtime.h>

#include "config.h"
#include "device_util.h"
#include "kernels.h"

namespace s2 {

namespace {

constexpr float kNegInf = -__builtin_inff();

// Kept blocks of block row i, in ascending order, as (stripe run, local run), or as a list.
struct RowBlocks {
  int first_stripe, n_stripe, stride, local_lo, count;
  const int32_t* cols;  // caller-supplied pattern: the row's list; nullptr = closed form
  __device__ int block(int n) const {
    if (cols) return cols[n];
    return n < n_stripe ? first_stripe + n * stride : local_lo + (n - n_stripe);
  }
};

__device__ inline RowBlocks row_blocks(const DecodeParams& p, int head, int i) {
  RowBlocks r;
  r.stride = p.stride;
  r.first_stripe = 0;
  r.n_stripe = 0;
  r.cols = nullptr;
  r.local_lo = 0;
  if (p.row_ptr) {
    const int32_t lo = p.row_ptr[(int64_t)head * p.num_blocks + i];
    r.cols = p.col_idx + lo;
    r.count = p.row_ptr[(int64_t)head * p.num_blocks + i + 1] - lo;
    return r;
  }
  if (p.dense) {
    r.local_lo = 0;
    r.count = i + 1;
    return r;
  }
  r.local_lo = max(0, i - p.local_blocks + 1);
  if (p.stride > 0) {
    const int o = (p.head_index_base + head) % p.stride;
    const int lo = p.window_blocks > 0 ? max(0, i - p.window_blocks + 1) : 0;
    int first = o;
    if (lo > o) first = o + ((lo - o + p.stride - 1) / p.stride) * p.stride;
    if (first < r.local_lo) {
      r.first_stripe = first;
      r.n_stripe = (r.local_lo - 1 - first) / p.stride + 1;
    }
  }
  r.count = r.n_stripe + (i - r.local_lo + 1);
  return r;
}

// GATHER: the instantiation for 16-token blocks, where a unit of work is four consecutive kept blocks
// of the row's list side by side, so that every load still fetches rows the query attends (a 16-token
// block on its own would fill a quarter of the 64 rows a unit loads).
template <int D, bool PAGED, bool GATHER>
__global__ __launch_bounds__(256, 2) void decode_split_kernel(const DecodeParams p) {
  constexpr int LPR = D / 8;     // lanes covering one row
  constexpr int RPI = 64 / LPR;  // rows covered by one wavefront-wide load
  constexpr int NI = 64 / RPI;   // loads per 64-token unit

  __shared__ float sh_m[4], sh_l[4];
  __shared__ float sh_acc[4][D];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int c = lane % LPR, g = lane / LPR;
  const int item = blockIdx.x;  // (b * heads + h) * splits + split
  const int split = item % p.num_splits;
  const int bh = item / p.num_splits;
  const int b = bh / p.heads, h = bh - b * p.heads;

  int L = p.seq_lens[b];
  L = min(max(L, 1), p.max_len);
  const int32_t* table = PAGED ? p.block_table + ((int64_t)b * p.heads + h) * p.max_blocks : nullptr;
  const int S = p.block_size;
  const int U = min(S, kChunk);  // tokens per unit of work: 64, or a whole block when it is shorter
  const int cpb = S / U;
  constexpr int BPU = 4;         // GATHER: blocks per unit
  const int i = (L - 1) / S;
  const RowBlocks rb = row_blocks(p, h, i);
  const int units = GATHER ? (rb.count + BPU - 1) / BPU : rb.count * cpb;
  const int u_lo = (int)((int64_t)units * split / p.num_splits);
  const int u_hi = (int)((int64_t)units * (split + 1) / p.num_splits);

  // my 8 query features, as floats
  float qv[8];
  {
    const bf16x8 q8 = *reinterpret_cast<const bf16x8*>(p.q + ((int64_t)b * p.heads + h) * D + 8 * c);
#pragma unroll
    for (int e = 0; e < 8; ++e) qv[e] = (float)q8[e];
  }
  const uint16_t* kb = p.k_cache + (PAGED ? 0 : b * p.kv_ss + h * p.kv_sh) + 8 * c;
  const uint16_t* vb = p.v_cache + (PAGED ? 0 : b * p.kv_ss + h * p.kv_sh) + 8 * c;
  int n_missing = 0;
  const float cl = p.scale_log2e;

  float m_run = kNegInf, l_run = 0.f;
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;

  for (int u = u_lo + wave; u < u_hi; u += 4) {
    bf16x8 kr[NI], vr[NI];
    bool live[NI];  // GATHER: whether my row of load n is a token the query attends
    int tok0 = 0, tok_end = 0;
    if constexpr (GATHER) {
      // slot RPI * n + g of the unit is token (slot mod 16) of the unit's block (slot div 16); a slot
      // past the list's end, past L or in a block that is not resident reads the first token of the
      // row's first kept block instead (it exists) and counts for nothing
      int64_t dead = (int64_t)rb.block(0) * S * p.kv_st;
      if (PAGED) {
        const int page = table[rb.block(0)];
        dead = (page >= 0 && page < p.num_pages) ? (int64_t)page * p.kv_ss : 0;  // else page 0 of the pool
      }
      int64_t row_off[NI];
#pragma unroll
      for (int n = 0; n < NI; ++n) {
        const int slot = RPI * n + g;
        const int bi = u * BPU + (slot >> 4);
        const bool inside = bi < rb.count;
        const int blk = rb.block(inside ? bi : 0);
        const int tok = blk * S + (slot & 15);
        bool ok = inside && tok < L;
        int64_t off = (int64_t)tok * p.kv_st;
        if (PAGED) {
          const int page = table[blk];
          const bool resident = page >= 0 && page < p.num_pages;
          // the lane that holds a block's first row counts a kept block that is not there
          if (inside && !resident && (slot & 15) == 0 && lane == 0) ++n_missing;
          ok = ok && resident;
          off = (int64_t)page * p.kv_ss + (int64_t)(slot & 15) * p.kv_st;
        }
        live[n] = ok;
        row_off[n] = ok ? off : dead;
      }
#pragma unroll
      for (int n = 0; n < NI; ++n) kr[n] = *reinterpret_cast<const bf16x8*>(kb + row_off[n]);
#pragma unroll
      for (int n = 0; n < NI; ++n) vr[n] = *reinterpret_cast<const bf16x8*>(vb + row_off[n]);
    } else {
    const int blk = rb.block(u / cpb);
    tok0 = blk * S + (u % cpb) * U;
    tok_end = min(L, tok0 + U);  // a 32-token block fills half of the 64 rows loaded
    if (tok0 >= L) continue;  // second half of a partial last block
    // row `tok` of the cache is at base + (tok - shift) * kv_st
    int64_t base = 0;
    int shift = 0;
    if (PAGED) {
      const int page = table[blk];
      if (page < 0 || page >= p.num_pages) {  // kept by the mask but not resident
        n_missing += (u % cpb) == 0;
        continue;
      }
      base = (int64_t)page * p.kv_ss;
      shift = blk * S;
    }
#pragma unroll
    for (int n = 0; n < NI; ++n) {
      const int tok = min(tok0 + RPI * n + g, tok_end - 1);  // clamp: never read past the unit
      kr[n] = *reinterpret_cast<const bf16x8*>(kb + base + (int64_t)(tok - shift) * p.kv_st);
    }
#pragma unroll
    for (int n = 0; n < NI; ++n) {
      const int tok = min(tok0 + RPI * n + g, tok_end - 1);
      vr[n] = *reinterpret_cast<const bf16x8*>(vb + base + (int64_t)(tok - shift) * p.kv_st);
    }
    }
    float s[NI];
    float mx = kNegInf;
#pragma unroll
    for (int n = 0; n < NI; ++n) {
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) d = __builtin_fmaf(qv[e], (float)kr[n][e], d);
#pragma unroll
      for (int m = 1; m < LPR; m <<= 1) d += __shfl_xor(d, m, 64);
      if (GATHER ? !live[n] : tok0 + RPI * n + g >= tok_end) d = kNegInf;
      s[n] = d;
      mx = fmaxf(mx, d);
    }
#pragma unroll
    for (int m = LPR; m < 64; m <<= 1) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
    const float m_new = fmaxf(m_run, mx);  // finite: token tok0 < L is always valid
    if (GATHER && m_new == kNegInf) continue;  // nothing live yet (a paged cache with the unit's blocks missing)
    const float alpha = fast_exp2((m_run - m_new) * cl);
    const float mc = m_new * cl;
    float psum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] *= alpha;
#pragma unroll
    for (int n = 0; n < NI; ++n) {
      const float pr = fast_exp2(__builtin_fmaf(s[n], cl, -mc));
      psum += pr;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = __builtin_fmaf(pr, (float)vr[n][e], acc[e]);
    }
    l_run = l_run * alpha + psum;  // per row group; groups are summed at the end
    m_run = m_new;
  }

  if (PAGED && p.missing && lane == 0 && n_missing > 0) atomicAdd(p.missing, n_missing);

  // sum the row groups of the wavefront
#pragma unroll
  for (int m = LPR; m < 64; m <<= 1) {
    l_run += __shfl_xor(l_run, m, 64);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], m, 64);
  }
  if (lane == 0) {
    sh_m[wave] = m_run;
    sh_l[wave] = l_run;
  }
  if (g == 0) {
#pragma unroll
    for (int e = 0; e < 8; ++e) sh_acc[wave][8 * c + e] = acc[e];
  }
  __syncthreads();
  if (tid < D) {
    float m = fmaxf(fmaxf(sh_m[0], sh_m[1]), fmaxf(sh_m[2], sh_m[3]));
    float l = 0.f, a = 0.f;
    if (m > kNegInf) {
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float wgt = fast_exp2((sh_m[w] - m) * cl);  // exp2(-inf) = 0 for an idle wavefront
        l += sh_l[w] * wgt;
        a += sh_acc[w][tid] * wgt;
      }
    }
    if (p.num_splits == 1) {
      // the only split of its (sequence, head): the result itself, no partials and no second kernel
      // (l == 0 only when nothing was attended: a paged cache with every kept block missing)
      const __bf16 out = (__bf16)(l > 0.f ? a / l : 0.f);
      p.o[(int64_t)bh * D + tid] = *reinterpret_cast<const uint16_t*>(&out);
      if (tid == 0 && p.lse) p.lse[bh] = l > 0.f ? m * p.scale + __logf(l) : kNegInf;
      return;
    }
    p.part_acc[(int64_t)item * D + tid] = a;
    if (tid == 0) {
      p.part_ml[(int64_t)item * 2 + 0] = m;
      p.part_ml[(int64_t)item * 2 + 1] = l;
    }
  }
}

template <int D>
__global__ __launch_bounds__(D) void decode_reduce_kernel(const DecodeParams p) {
  const int bh = blockIdx.x, d = threadIdx.x;
  const float cl = p.scale_log2e;
  const float* ml = p.part_ml + (int64_t)bh * p.num_splits * 2;
  float m = kNegInf;
  for (int s = 0; s < p.num_splits; ++s) m = fmaxf(m, ml[2 * s]);
  float l = 0.f, a = 0.f;
  for (int s = 0; s < p.num_splits; ++s) {
    const float ms = ml[2 * s];
    if (ms == kNegInf) continue;  // empty split
    const float wgt = fast_exp2((ms - m) * cl);
    l += ml[2 * s + 1] * wgt;
    a += p.part_acc[((int64_t)bh * p.num_splits + s) * D + d] * wgt;
  }
  // l == 0 only when nothing was attended: a paged cache with every kept block missing
  const __bf16 out = (__bf16)(l > 0.f ? a / l : 0.f);
  p.o[(int64_t)bh * D + d] = *reinterpret_cast<const uint16_t*>(&out);
  if (d == 0 && p.lse) p.lse[bh] = l > 0.f ? m * p.scale + __logf(l) : kNegInf;
}

template <int D>
hipError_t launch_one(const DecodeParams& p, hipStream_t stream) {
  const int bh = p.nseq * p.heads;
  const dim3 grid(bh * p.num_splits);
  if (p.block_size == 16) {
    if (p.block_table)
      hipLaunchKernelGGL((decode_split_kernel<D, true, true>), grid, dim3(256), 0, stream, p);
    else
      hipLaunchKernelGGL((decode_split_kernel<D, false, true>), grid, dim3(256), 0, stream, p);
  } else if (p.block_table) {
    hipLaunchKernelGGL((decode_split_kernel<D, true, false>), grid, dim3(256), 0, stream, p);
  } else {
    hipLaunchKernelGGL((decode_split_kernel<D, false, false>), grid, dim3(256), 0, stream, p);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || p.num_splits == 1) return e;  // a single split writes the result itself
  hipLaunchKernelGGL((decode_reduce_kernel<D>), dim3(bh), dim3(D), 0, stream, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode(const DecodeParams& p, hipStream_t stream) {
  return p.head_dim == 128 ? launch_one<128>(p, stream) : launch_one<64>(p, stream);
}

}  // namespace s2
