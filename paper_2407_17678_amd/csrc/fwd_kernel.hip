// Forward kernel: block-sparse causal attention with per-head lists of kept KV blocks
// (section 3.2: iterate K/V tiles through on-chip memory, softmax over the kept keys only;
// section 4.2: which blocks a head keeps).  One workgroup owns a query tile of 128 rows that
// spans several mask rows (the Merge-Q idea of section 3.2: a big tile, a fine mask); it walks
// the merged list of KV blocks any of its rows keeps, and each wavefront skips the blocks its own
// mask row does not keep.
//
// Orientation: the score tile is computed transposed, S^T = K Q^T, so that a lane owns one
// query (one column of the C layout).  Row max / row sum are then in-lane reductions plus one
// exchange with the other half of the wavefront, and the probabilities feed the second
// contraction O^T += V^T P^T straight from the accumulator registers.
//
// K and V chunks (64 keys) are brought in by direct global -> LDS loads, double buffered; K is
// read as row fragments, V through the LDS transpose read (DmaTile in device_util.h).
#include <hip/hip_runtime.h>

#include "config.h"
#include "device_util.h"
#include "kernels.h"

namespace s2 {

namespace {

constexpr float kNegInf = -__builtin_inff();


// CH = keys per step (one LDS stage), 64 or 32.  With 32 a workgroup needs half the LDS and fewer
// registers, so three workgroups fit a CU instead of two; measured, that is no faster (twice the
// barriers for the same work), so 64 is what is instantiated.
//
// VARLEN: a packed batch of sequences of different lengths.  A workgroup finds its sequence's rows
// in cu_seqlens and treats them as a sequence of its own; the ragged end costs a clamped load plan
// for the chunks that reach past the last token (their keys are after every query, so the causal
// mask already drops them) and a per-lane guard on the stores.  Where the fast-path kernel applies
// (fwd_pipe_kernel.hip) it computes each sequence's whole 128-row tiles and this kernel is launched for
// the partial last tiles only (AttnParams::varlen_tail).
template <int D, bool DENSE, int CH, bool VARLEN = false>
__global__ __launch_bounds__(kThreads, (CH == 32 ? 3 : 2)) void fwd_kernel(const AttnParams p) {
  typedef DmaTile<D, CH> Tile;
  __shared__ __attribute__((aligned(16))) uint16_t sk[2][Tile::kElems];
  __shared__ __attribute__((aligned(16))) uint16_t sv[2][Tile::kElems];
  constexpr int BM = kFwdBM;
  constexpr int MW = 32;       // rows per wavefront
  constexpr int KT = CH / 32;  // 32-key score tiles per step
  static_assert(BM == 4 * MW, "four wavefronts of 32 query rows");

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int T = p.fwd_tiles.tiles_per_head;      // tiles of the whole sequence (indexes the lists)
  // tiles this launch computes (of a packed batch's sequences possibly the last one only)
  const int T_run = (VARLEN && p.varlen_tail) ? 1 : (p.q_rows + BM - 1) / BM;
  int bh, rank;
  if (!map_workgroup(blockIdx.x, p.batch * p.heads, T_run, bh, rank)) return;
  const int b = bh / p.heads, h = bh - b * p.heads;
  // longest tiles first: by the layout's order for a whole sequence, else simply last row first
  const bool whole = !VARLEN && p.q_row0 == 0 && T_run == T;
  int tile = (DENSE || !whole) ? p.q_row0 / BM + (T_run - 1 - rank) : p.fwd_tiles.order[h * T + rank];
  // rows of the tensors before my sequence, and its length (q, o, lse rows and keys alike)
  int row_base = 0, N = p.seqlen, n_q = p.q_rows;
  if (VARLEN) {
    const int lo = p.cu_seqlens[b], hi = p.cu_seqlens[b + 1];
    row_base = min(max(lo, 0), p.seqlen);  // whatever the array holds, stay inside the tensors
    N = min(min(max(hi - lo, 0), p.q_rows), p.seqlen - row_base);
    n_q = N;
    const int T_seq = (N + BM - 1) / BM;
    if (rank >= T_seq) return;
    tile = T_seq - 1 - rank;
    if (p.varlen_tail && N % BM == 0) return;  // no partial tile: the fast-path launch has computed them all
  }
  const int S = DENSE ? kChunk : p.block_size;
  // 16-token blocks: a list entry is a unit of two blocks (32 keys, one step) and my 32 query rows
  // are two mask rows, so which keys a lane may see is a 2 x 2 pattern of bits per wavefront
  const bool fine = !DENSE && CH == 32 && S == 16;
  const int Sg = fine ? 32 : S;  // tokens per list entry
  const int cpb = Sg / CH;  // steps per entry: a power of two, so / and % below are a shift and a mask
  const int cpb_sh = __builtin_ctz(cpb), cpb_m = cpb - 1;

  const int qw0 = tile * BM + wave * MW;  // first query row of this wavefront (sequence position)
  const int ql0 = qw0 - p.q_row0;         // the same as a row of q / o / lse
  const bool wave_active = ql0 < n_q;
  const int my_member = (qw0 / Sg) - tile * (BM / Sg);  // which mask row of the tile I am in

  const int64_t q_off = (VARLEN ? row_base * p.q_st : b * p.q_sb) + h * p.q_sh;
  const int64_t kv_off = (VARLEN ? row_base * p.kv_st : b * p.kv_sb) + h * p.kv_sh;
  const uint16_t* qb = p.q + q_off;
  const uint16_t* kb = p.k + kv_off;
  const uint16_t* vb = p.v + kv_off;

  // Q^T fragments stay in registers for the whole tile.
  bf16x8 qf[D / 16];
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) {
    if (wave_active)  // a lane past the ragged end reads the last row; its result is never stored
      qf[kk] = *reinterpret_cast<const bf16x8*>(qb + (int64_t)(VARLEN ? min(ql0 + l32, N - 1) : ql0 + l32) * p.q_st +
                                                16 * kk + 8 * half);
    else
      qf[kk] = bf16x8{};
  }

  int ent_lo = 0, n_ent;
  if (DENSE) {
    n_ent = min(N, (tile + 1) * BM) / kChunk;  // every block up to the tile's last row
  } else {
    ent_lo = p.fwd_tiles.ptr[h * T + tile];
    n_ent = p.fwd_tiles.ptr[h * T + tile + 1] - ent_lo;
  }
  const int total = n_ent * cpb;

  EntryList list;
  if (!DENSE) list.init(p.fwd_tiles.ent + ent_lo, n_ent, lane);
  // step `it` of the tile's list: its first key row, and whether my mask row keeps the block
  // `pat` (16-token blocks only): bit 2m + c set when mask row m of my two keeps block c of the unit
  auto chunk_of = [&](int it, int& kv0, bool& keep, int& pat) {
    pat = 0xF;
    if (DENSE) {
      kv0 = it * CH;
      keep = true;
    } else {
      const int e = list.get((it >> cpb_sh), lane);
      kv0 = (e >> 16) * Sg + ((it & cpb_m)) * CH;
      if (fine) {
        pat = (e >> (4 * wave)) & 0xF;
        keep = pat != 0;
      } else {
        keep = (e >> my_member) & 1;
      }
    }
  };
  // first key row of step it+1, right after chunk_of(it)
  auto next_chunk_of = [&](int it, int& kv0_n) {
    if (DENSE) {
      kv0_n = (it + 1) * CH;
    } else {
      const int e = ((it + 1) >> cpb_sh) == (it >> cpb_sh) ? list.get((it >> cpb_sh), lane) : list.peek_next((it >> cpb_sh));
      kv0_n = (e >> 16) * Sg + (((it + 1) & cpb_m)) * CH;
    }
  };

  f32x16 acc_o[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) acc_o[dt] = f32x16{};
  float m_run = kNegInf;  // running max of the raw (unscaled) scores of my query
  float l_run = 0.f;      // running sum over my half's key rows
  const float c = p.scale_log2e;

  const typename Tile::Plan plan = Tile::plan(p.kv_st, wave, lane);
  const int trb = Tile::tr_base(lane);
  constexpr int PW = Tile::kPerWave;
  if (total > 0) {
    int kv0, pat;
    bool keep;
    chunk_of(0, kv0, keep, pat);
    if (VARLEN && kv0 + CH > N) {
      const typename Tile::Plan pr = Tile::plan_rows(p.kv_st, wave, lane, N - kv0);
      Tile::issue(pr, kb + (int64_t)min(kv0, N - 1) * p.kv_st, sk[0], wave);
      Tile::issue(pr, vb + (int64_t)min(kv0, N - 1) * p.kv_st, sv[0], wave);
    } else {
      Tile::issue(plan, kb + (int64_t)kv0 * p.kv_st, sk[0], wave);
      Tile::issue(plan, vb + (int64_t)kv0 * p.kv_st, sv[0], wave);
    }
  }
  wait_all_loads();
  __syncthreads();

  for (int it = 0; it < total; ++it) {
    const uint16_t* ks = sk[it & 1];
    const uint16_t* vs = sv[it & 1];
    const uint16_t* kn = sk[(it & 1) ^ 1];
    const uint16_t* vn = sv[(it & 1) ^ 1];
    int kv0, pat;
    bool keep;
    chunk_of(it, kv0, keep, pat);
    // The next step's direct loads are spread between the MFMAs of the first contraction, or
    // issued at once by a wavefront that has nothing to compute in this step.  The last step
    // loads its own chunk once more into the idle stage: nothing reads it, and the loop body
    // then has no branch between the MFMAs.
    // nothing to do when my mask row drops the block or all keys lie after every one of my queries
    const bool compute = wave_active && keep && kv0 <= qw0 + MW - 1;
    int kv1 = kv0;
    if (it + 1 < total) next_chunk_of(it, kv1);
    // the plan of the loads issued in this step: the usual one, or clamped to the rows that exist
    typename Tile::Plan pl = plan;
    int kv1_row = kv1;
    if (VARLEN && kv1 + CH > N) {
      pl = Tile::plan_rows(p.kv_st, wave, lane, N - kv1);
      kv1_row = min(kv1, N - 1);
    }
    const uint16_t* kg = kb + (int64_t)kv1_row * p.kv_st;
    const uint16_t* vg = vb + (int64_t)kv1_row * p.kv_st;
    if (!compute) {
      Tile::issue(pl, kg, kn, wave);
      Tile::issue(pl, vg, vn, wave);
    }

    if (compute) {
      f32x16 s[KT];
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) s[kt] = f32x16{};
      // all K fragments of the step are requested before the first MFMA needs one
      bf16x8 kfr[KT][D / 16];
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk)
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) kfr[kt][kk] = Tile::row_frag(ks, kt, kk, l32, half);
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk)
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
          s[kt] = mfma32(kfr[kt][kk], qf[kk], s[kt]);
          const int n = KT * kk + kt;
          if (n < PW) Tile::issue_one(pl, n, kg, kn, wave);
          if (n >= PW && n < 2 * PW) Tile::issue_one(pl, n - PW, vg, vn, wave);
        }
      static_assert(2 * PW <= KT * (D / 16), "every load has an MFMA to follow");
      if (CH == 32 && pat != 0xF) {  // 16-token blocks: drop the blocks my mask row does not keep
        const int mine = pat >> (2 * (l32 >> 4));
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (!((mine >> (r >> 3)) & 1)) s[0][r] = kNegInf;  // registers 0..7: block 0, 8..15: block 1
      }
      if (kv0 + CH - 1 > qw0) {  // diagonal: key position must not exceed query position
        const int qpos = qw0 + l32;
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kv0 + 32 * kt + 8 * (r >> 2) + 4 * half + (r & 3);
            if (key > qpos) s[kt][r] = kNegInf;
          }
      }
      float mx = s[0][0];
#pragma unroll
      for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kt][r]);
      mx = max_halves(mx);
      // a tile wholly above the diagonal has mx = -inf; keep the running max unchanged then
      const float m_new = fmaxf(m_run, mx);
      const float m_use = (m_new == kNegInf) ? 0.f : m_new;
      const float alpha = fast_exp2((m_run - m_use) * c);
      const float mc = m_use * c;
      float psum = 0.f;
#pragma unroll
      for (int kt = 0; kt < KT; ++kt)
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
      for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const bf16x8 pb = pack8(s[kt][8 * u + 0], s[kt][8 * u + 1], s[kt][8 * u + 2], s[kt][8 * u + 3],
                                  s[kt][8 * u + 4], s[kt][8 * u + 5], s[kt][8 * u + 6], s[kt][8 * u + 7]);
#pragma unroll
          for (int dt = 0; dt < D / 32; ++dt)
            acc_o[dt] = mfma32(Tile::tr_frag(vs, dt, 2 * kt + u, trb), pb, acc_o[dt]);
        }
    }

    wait_all_loads();
    __syncthreads();
  }

  if (!wave_active) return;
  const float l_tot = sum_halves(l_run);
  const float inv = 1.0f / l_tot;
  const int qrow = ql0 + l32;
  if (VARLEN && qrow >= N) return;  // past the ragged end of my sequence
  uint16_t* orow = p.o + q_off + (int64_t)qrow * p.q_st;
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 w;
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = (__bf16)(acc_o[dt][4 * g + e] * inv);
      *reinterpret_cast<bf16x4*>(orow + 32 * dt + 8 * g + 4 * half) = w;
    }
  const int64_t lse_row = VARLEN ? (int64_t)h * p.seqlen + row_base + qrow  // [heads, rows of the tensors]
                                 : ((int64_t)b * p.heads + h) * p.q_rows + qrow;
  if (half == 0) p.lse[lse_row] = m_run * p.scale + __logf(l_tot);
}

template <int D, bool DENSE>
hipError_t launch_one(const AttnParams& p, hipStream_t stream) {
  const int grid = grid_for(p.batch * p.heads, p.varlen_tail ? 1 : (p.q_rows + kFwdBM - 1) / kFwdBM);
  if (!DENSE && p.cu_seqlens) {  // packed variable-length batch (sparse layouts only)
    if (p.block_size <= 32)
      hipLaunchKernelGGL((fwd_kernel<D, false, 32, true>), dim3(grid), dim3(kThreads), 0, stream, p);
    else
      hipLaunchKernelGGL((fwd_kernel<D, false, kFwdChunk, true>), dim3(grid), dim3(kThreads), 0, stream, p);
    return hipGetLastError();
  }
  if (!DENSE && p.block_size <= 32)  // 16- and 32-token mask blocks: steps of 32 keys
    hipLaunchKernelGGL((fwd_kernel<D, false, 32>), dim3(grid), dim3(kThreads), 0, stream, p);
  else
    hipLaunchKernelGGL((fwd_kernel<D, DENSE, kFwdChunk>), dim3(grid), dim3(kThreads), 0, stream, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fwd(const AttnParams& p, bool dense, hipStream_t stream) {
  if (p.cu_seqlens && fwd_pipe_applies(p, dense)) {
    // packed batch: whole 128-row tiles by the fast path, each sequence's partial last tile here
    hipError_t e = launch_fwd_pipe(p, dense, stream);
    if (e != hipSuccess) return e;
    AttnParams tail = p;
    tail.varlen_tail = 1;
    return launch_one<128, false>(tail, stream);
  }
  if (fwd_pipe_applies(p, dense)) return launch_fwd_pipe(p, dense, stream);
  if (p.head_dim == 128) return dense ? launch_one<128, true>(p, stream) : launch_one<128, false>(p, stream);
  return dense ? launch_one<64, true>(p, stream) : launch_one<64, false>(p, stream);
}

}  // namespace s2
