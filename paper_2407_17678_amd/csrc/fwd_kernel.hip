// Forward kernel: block-sparse causal attention with per-head lists of kept KV blocks
// (section 3.2: iterate K/V tiles through on-chip memory, softmax over the kept keys only;
// section 4.2: which blocks a head keeps).  One workgroup owns a 128-row query tile that spans
// one or two mask rows (the Merge-Q idea of section 3.2: a big tile, a fine mask); it walks the
// merged list of KV blocks any of its rows keeps, and each wavefront skips the blocks its own
// mask row does not keep.
//
// Orientation: the score tile is computed transposed, S^T = K Q^T, so that a lane owns one
// query (one column of the C layout).  Row max / row sum are then in-lane reductions plus one
// exchange with the other half of the wavefront, and the probabilities can be fed to the second
// contraction O^T += V^T P^T straight from the accumulator registers.
#include <hip/hip_runtime.h>

#include "config.h"
#include "device_util.h"
#include "kernels.h"

namespace s2 {

namespace {

constexpr float kNegInf = -__builtin_inff();

template <int D>
struct FwdSmem {
  uint16_t k[2][RowTile<D>::kElems];
  uint16_t vt[2][TransposedTile<D>::kElems];
};

template <int D, bool DENSE>
__global__ __launch_bounds__(kThreads, 2) void fwd_kernel(const AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  FwdSmem<D>& sm = *reinterpret_cast<FwdSmem<D>*>(smem_raw);

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int T = p.q_tiles.tiles_per_head;
  int bh, rank;
  if (!map_workgroup(blockIdx.x, p.batch * p.heads, T, bh, rank)) return;
  const int b = bh / p.heads, h = bh - b * p.heads;
  const int tile = DENSE ? (T - 1 - rank) : p.q_tiles.order[h * T + rank];
  const int S = DENSE ? kChunk : p.block_size;
  const int cpb = S / kChunk;  // 64-key chunks per mask block

  const int N = p.seqlen;
  const int qw0 = tile * kFwdBM + wave * 32;  // first query row of this wavefront
  const bool wave_active = qw0 < N;
  const int my_member = (qw0 / S) - tile * (kFwdBM / S);  // which mask row of the tile I am in

  const uint16_t* qb = p.q + b * p.q_sb + h * p.q_sh;
  const uint16_t* kb = p.k + b * p.kv_sb + h * p.kv_sh;
  const uint16_t* vb = p.v + b * p.kv_sb + h * p.kv_sh;

  // Q^T fragments stay in registers for the whole tile.
  bf16x8 qf[D / 16];
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) {
    if (wave_active)
      qf[kk] = *reinterpret_cast<const bf16x8*>(qb + (int64_t)(qw0 + l32) * p.q_st + 16 * kk + 8 * half);
    else
      qf[kk] = bf16x8{};
  }

  int ent_lo = 0, n_ent;
  if (DENSE) {
    n_ent = min(N, (tile + 1) * kFwdBM) / kChunk;  // every chunk up to the tile's last row
  } else {
    ent_lo = p.q_tiles.ptr[h * T + tile];
    n_ent = p.q_tiles.ptr[h * T + tile + 1] - ent_lo;
  }
  const int total = n_ent * cpb;

  // chunk `it` of the tile's list: first key row, and whether my mask row keeps it
  auto chunk_of = [&](int it, int& kv0, bool& keep) {
    if (DENSE) {
      kv0 = it * kChunk;
      keep = true;
    } else {
      const int e = p.q_tiles.ent[ent_lo + it / cpb];
      kv0 = (e >> 8) * S + (it % cpb) * kChunk;
      keep = (e >> my_member) & 1;
    }
  };

  f32x16 acc_o[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) acc_o[dt] = f32x16{};
  float m_run = kNegInf;  // running max of the raw (unscaled) scores of my query
  float l_run = 0.f;      // running sum over my half's key rows
  const float c = p.scale_log2e;

  u32x4 kreg[RowTile<D>::kPerThread];
  u32x4 vreg[4];
  if (total > 0) {
    int kv0;
    bool keep;
    chunk_of(0, kv0, keep);
    RowTile<D>::load(kreg, kb + (int64_t)kv0 * p.kv_st, p.kv_st, tid);
    TransposedTile<D>::load(vreg, vb + (int64_t)kv0 * p.kv_st, p.kv_st, tid);
    RowTile<D>::store(kreg, sm.k[0], tid);
    TransposedTile<D>::store(vreg, sm.vt[0], tid);
  }
  __syncthreads();

  for (int it = 0; it < total; ++it) {
    const int buf = it & 1;
    int kv0;
    bool keep;
    chunk_of(it, kv0, keep);
    if (it + 1 < total) {
      int kv1;
      bool keep1;
      chunk_of(it + 1, kv1, keep1);
      RowTile<D>::load(kreg, kb + (int64_t)kv1 * p.kv_st, p.kv_st, tid);
      TransposedTile<D>::load(vreg, vb + (int64_t)kv1 * p.kv_st, p.kv_st, tid);
    }

    // keys of this chunk all lie after every one of my 32 queries -> nothing to do
    if (wave_active && keep && kv0 <= qw0 + 31) {
      const uint16_t* ks = sm.k[buf];
      const uint16_t* vs = sm.vt[buf];
      f32x16 s[2] = {f32x16{}, f32x16{}};
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
          s[kt] = mfma32(RowTile<D>::frag(ks, kt, kk, l32, half), qf[kk], s[kt]);
      }
      if (kv0 + kChunk - 1 > qw0) {  // diagonal chunk: key position must not exceed query position
        const int qpos = qw0 + l32;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kv0 + 32 * kt + 8 * (r >> 2) + 4 * half + (r & 3);
            if (key > qpos) s[kt][r] = kNegInf;
          }
      }
      float mx = s[0][0];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kt][r]);
      mx = fmaxf(mx, other_half(mx));
      const float m_new = fmaxf(m_run, mx);
      const float alpha = fast_exp2((m_run - m_new) * c);
      const float mc = m_new * c;
      float psum = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          s[kt][r] = fast_exp2(__builtin_fmaf(s[kt][r], c, -mc));
          psum += s[kt][r];
        }
      l_run = l_run * alpha + psum;
      if (__any(m_new != m_run)) {
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc_o[dt][r] *= alpha;
      }
      m_run = m_new;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const bf16x8 pb = pack8(s[kt][8 * u + 0], s[kt][8 * u + 1], s[kt][8 * u + 2], s[kt][8 * u + 3],
                                  s[kt][8 * u + 4], s[kt][8 * u + 5], s[kt][8 * u + 6], s[kt][8 * u + 7]);
#pragma unroll
          for (int dt = 0; dt < D / 32; ++dt)
            acc_o[dt] = mfma32(TransposedTile<D>::frag(vs, dt, 2 * kt + u, l32, half), pb, acc_o[dt]);
        }
    }

    if (it + 1 < total) {
      RowTile<D>::store(kreg, sm.k[buf ^ 1], tid);
      TransposedTile<D>::store(vreg, sm.vt[buf ^ 1], tid);
    }
    __syncthreads();
  }

  if (!wave_active) return;
  const float l_tot = l_run + other_half(l_run);
  const float inv = 1.0f / l_tot;
  const int qrow = qw0 + l32;
  uint16_t* orow = p.o + b * p.q_sb + h * p.q_sh + (int64_t)qrow * p.q_st;
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 w;
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = (__bf16)(acc_o[dt][4 * g + e] * inv);
      *reinterpret_cast<bf16x4*>(orow + 32 * dt + 8 * g + 4 * half) = w;
    }
  if (half == 0)
    p.lse[((int64_t)b * p.heads + h) * N + qrow] = m_run * p.scale + __logf(l_tot);
}

template <int D, bool DENSE>
hipError_t launch_one(const AttnParams& p, hipStream_t stream) {
  const int T = p.q_tiles.tiles_per_head;
  const int grid = grid_for(p.batch * p.heads, T);
  const size_t smem = sizeof(FwdSmem<D>);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&fwd_kernel<D, DENSE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((fwd_kernel<D, DENSE>), dim3(grid), dim3(kThreads), smem, stream, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd(const AttnParams& p, bool dense, hipStream_t stream) {
  if (p.head_dim == 128) return dense ? launch_one<128, true>(p, stream) : launch_one<128, false>(p, stream);
  return dense ? launch_one<64, true>(p, stream) : launch_one<64, false>(p, stream);
}

}  // namespace s2
