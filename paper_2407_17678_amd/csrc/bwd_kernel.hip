// Backward kernels: gradients of block-sparse causal attention (the backward pass that goes with
// the forward of section 3.2; the paper names it as the less optimised half of its kernels).
//
// Two launches (three kernels exist), no atomics, bitwise reproducible:
//   delta  : delta[t] = sum_d dO[t][d] * O[t][d].  Folded into the dq launch, which holds the dO
//            fragments anyway; the stand-alone kernel runs only when dK/dV is asked for alone.
//   dq     : row-stationary.  A workgroup owns 128 query rows and walks the merged list of KV
//            blocks its mask rows keep (as the forward does), recomputing P and forming
//            dS = P * (dP - delta), dQ += scale * dS K.
//   dkdv   : column-stationary.  A workgroup owns 128 keys - one or two mask columns, paired by
//            the layout builder so that both are attended by nearly the same query blocks - and
//            walks the query blocks that keep them: dV += P^T dO, dK += scale * dS^T Q.
//
// Both main kernels keep the stationary operand's MFMA fragments in registers with the lane
// owning one stationary row, so the recomputed score tile lands in the C layout with the
// streamed index in registers; it is then fed back as the B operand of the next contraction
// without leaving the lane (see device_util.h).  The streamed 64-row chunk is brought in by
// direct global -> LDS loads (double buffered) and read in both operand forms from the one
// row-major tile: row fragments (k = feature) and LDS transpose reads (k = token).
#include <hip/hip_runtime.h>

#include <atomic>

#include "config.h"
#include "device_util.h"
#include "kernels.h"

namespace s2 {

namespace {

constexpr float kLog2e = 1.4426950408889634f;

// ------------------------------------------------------------------------------------ delta

template <int D>
__global__ __launch_bounds__(256) void delta_kernel(const AttnParams p) {
  constexpr int LPR = D / 8;          // lanes per row
  constexpr int RPB = 256 / LPR;      // rows per block
  const int tid = threadIdx.x;
  const int64_t row = (int64_t)blockIdx.x * RPB + tid / LPR;
  const int c = tid % LPR;
  const int64_t rows_total = (int64_t)p.batch * p.heads * p.seqlen;
  float acc = 0.f;
  if (row < rows_total) {
    const int64_t bh = row / p.seqlen;
    const int t = (int)(row - bh * p.seqlen);
    const int b = (int)(bh / p.heads), h = (int)(bh - (int64_t)b * p.heads);
    const int64_t off = b * p.q_sb + h * p.q_sh + (int64_t)t * p.q_st + 8 * c;
    const bf16x8 o = *reinterpret_cast<const bf16x8*>(p.o + off);
    const bf16x8 g = *reinterpret_cast<const bf16x8*>(p.d_o + off);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc += (float)o[e] * (float)g[e];
  }
#pragma unroll
  for (int m = LPR / 2; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
  if (c == 0 && row < rows_total) {
    p.delta[row] = acc;
    p.lse2[row] = p.lse[row] * kLog2e;  // the main kernels want LSE in base-2 units
  }
}

// ------------------------------------------------------------------------------------ dq

// CH = keys per step: 64, or 32 for 32-token mask blocks.
template <int D, int CH>
struct DqSmem {
  uint16_t k[2][DmaTile<D, CH>::kElems];
  uint16_t v[2][DmaTile<D, CH>::kElems];
};

// VARLEN: a packed batch of sequences of different lengths (see the forward kernel): the workgroup
// finds its sequence in cu_seqlens; loads that would pass the sequence's last token are clamped to
// it (keys there lie after every query, which the causal mask drops) and stores are guarded per lane.
template <int D, bool DENSE, int CH, bool VARLEN = false>
__global__ __launch_bounds__(kThreads, 2) void dq_kernel(const AttnParams p) {
  typedef DmaTile<D, CH> Tile;
  constexpr int KT = CH / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  DqSmem<D, CH>& sm = *reinterpret_cast<DqSmem<D, CH>*>(smem_raw);

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int T = p.q_tiles.tiles_per_head;
  // (of a packed batch's sequences possibly the last tile only)
  const int T_run = VARLEN ? (p.varlen_tail ? 1 : (p.q_rows + kBwdBM - 1) / kBwdBM) : T;
  int bh, rank;
  if (!map_workgroup(blockIdx.x, p.batch * p.heads, T_run, bh, rank)) return;
  const int b = bh / p.heads, h = bh - b * p.heads;
  int tile = DENSE ? (T - 1 - rank) : VARLEN ? 0 : p.q_tiles.order[h * T + rank];
  int row_base = 0, N = p.seqlen;
  if (VARLEN) {
    const int lo = p.cu_seqlens[b], hi = p.cu_seqlens[b + 1];
    row_base = min(max(lo, 0), p.seqlen);  // whatever the array holds, stay inside the tensors
    N = min(min(max(hi - lo, 0), p.q_rows), p.seqlen - row_base);
    const int T_seq = (N + kBwdBM - 1) / kBwdBM;
    if (rank >= T_seq) return;
    tile = T_seq - 1 - rank;
    if (p.varlen_tail && N % kBwdBM == 0) return;  // no partial tile: the fast-path launch has computed them all
  }
  const int S = DENSE ? kChunk : p.block_size;
  // 16-token blocks: a list entry is a unit of two blocks (32 keys, one step) and my 32 query rows
  // are two mask rows, so which keys a lane may see is a 2 x 2 pattern of bits per wavefront
  const bool fine = !DENSE && CH == 32 && S == 16;
  const int Sg = fine ? 32 : S;  // tokens per list entry
  const int cpb = Sg / CH;  // a power of two: / and % below are a shift and a mask
  const int cpb_sh = __builtin_ctz(cpb), cpb_m = cpb - 1;
  const int qw0 = tile * kBwdBM + wave * 32;
  const bool wave_active = qw0 < N;
  const int my_member = (qw0 / Sg) - tile * (kBwdBM / Sg);

  const int64_t q_off = (VARLEN ? row_base * p.q_st : b * p.q_sb) + h * p.q_sh;
  const int64_t kv_off = (VARLEN ? row_base * p.kv_st : b * p.kv_sb) + h * p.kv_sh;
  const uint16_t* kb = p.k + kv_off;
  const uint16_t* vb = p.v + kv_off;

  int ent_lo = 0, n_ent;
  if (DENSE) {
    n_ent = min(N, (tile + 1) * kBwdBM) / kChunk;  // dense blocks are kChunk keys
  } else {
    ent_lo = p.q_tiles.ptr[h * T + tile];
    n_ent = p.q_tiles.ptr[h * T + tile + 1] - ent_lo;
  }
  const int total = n_ent * cpb;
  EntryList list;
  if (!DENSE) list.init(p.q_tiles.ent + ent_lo, n_ent, lane);
  // chunk `it` of the tile's list: its first row, and whether my mask row / column keeps it
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
  // first row of chunk it+1, right after chunk_of(it)
  auto next_chunk_of = [&](int it, int& kv0_n) {
    if (DENSE) {
      kv0_n = (it + 1) * CH;
    } else {
      const int e = ((it + 1) >> cpb_sh) == (it >> cpb_sh) ? list.get((it >> cpb_sh), lane) : list.peek_next((it >> cpb_sh));
      kv0_n = (e >> 16) * Sg + (((it + 1) & cpb_m)) * CH;
    }
  };

  const typename Tile::Plan plan = Tile::plan(p.kv_st, wave, lane);
  const int trb = Tile::tr_base(lane);
  if (total > 0) {
    int kv0, pat;
    bool keep;
    chunk_of(0, kv0, keep, pat);
    if (VARLEN && kv0 + CH > N) {
      const typename Tile::Plan pr = Tile::plan_rows(p.kv_st, wave, lane, N - kv0);
      Tile::issue(pr, kb + (int64_t)min(kv0, N - 1) * p.kv_st, sm.k[0], wave);
      Tile::issue(pr, vb + (int64_t)min(kv0, N - 1) * p.kv_st, sm.v[0], wave);
    } else {
      Tile::issue(plan, kb + (int64_t)kv0 * p.kv_st, sm.k[0], wave);
      Tile::issue(plan, vb + (int64_t)kv0 * p.kv_st, sm.v[0], wave);
    }
  }

  bf16x8 qf[D / 16], gf[D / 16];  // Q^T and dO^T fragments (B operands), lane = query
  float lse_l = 0.f, delta_l = 0.f;
  // delta = rowsum(dO * O) of my query, computed here from the dO fragments the kernel holds
  // anyway (my half of the row's features, then the two halves added), so that a whole backward
  // needs no separate pass over O and dO; it is also written out, with LSE in base-2 units, for
  // the dK/dV kernel, which runs after this one.
  float part = 0.f;
  // my query's row; a lane past the ragged end of a packed sequence reads the last row (never stored)
  const int my_row = VARLEN ? min(qw0 + l32, N - 1) : qw0 + l32;
  const bool my_row_exists = !VARLEN || qw0 + l32 < N;
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) {
    if (wave_active) {
      const int64_t o = q_off + (int64_t)my_row * p.q_st + 16 * kk + 8 * half;
      qf[kk] = *reinterpret_cast<const bf16x8*>(p.q + o);
      gf[kk] = *reinterpret_cast<const bf16x8*>(p.d_o + o);
      const bf16x8 of = *reinterpret_cast<const bf16x8*>(p.o + o);
#pragma unroll
      for (int e = 0; e < 8; ++e) part = __builtin_fmaf((float)gf[kk][e], (float)of[e], part);
    } else {
      qf[kk] = bf16x8{};
      gf[kk] = bf16x8{};
    }
  }
  delta_l = sum_halves(part);
  if (wave_active) {
    const int64_t r = VARLEN ? (int64_t)h * p.seqlen + row_base + my_row  // [heads, rows of the tensors]
                             : ((int64_t)b * p.heads + h) * N + my_row;
    lse_l = p.lse[r] * kLog2e;
    if (half == 0 && my_row_exists) {
      p.delta[r] = delta_l;
      p.lse2[r] = lse_l;
    }
  }

  f32x16 acc[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) acc[dt] = f32x16{};
  const float c = p.scale_log2e;

  wait_all_loads();
  __syncthreads();

  for (int it = 0; it < total; ++it) {
    const int buf = it & 1;
    int kv0, pat;
    bool keep;
    chunk_of(it, kv0, keep, pat);
    if (it + 1 < total) {
      int kv1;
      next_chunk_of(it, kv1);
      if (VARLEN && kv1 + CH > N) {
        const typename Tile::Plan pr = Tile::plan_rows(p.kv_st, wave, lane, N - kv1);
        Tile::issue(pr, kb + (int64_t)min(kv1, N - 1) * p.kv_st, sm.k[buf ^ 1], wave);
        Tile::issue(pr, vb + (int64_t)min(kv1, N - 1) * p.kv_st, sm.v[buf ^ 1], wave);
      } else {
        Tile::issue(plan, kb + (int64_t)kv1 * p.kv_st, sm.k[buf ^ 1], wave);
        Tile::issue(plan, vb + (int64_t)kv1 * p.kv_st, sm.v[buf ^ 1], wave);
      }
    }

    if (wave_active && keep && kv0 <= qw0 + 31) {
      const uint16_t* ks = sm.k[buf];
      const uint16_t* vs = sm.v[buf];
      const int qpos = qw0 + l32;
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) {
        const int kbase = kv0 + 32 * kt;
        if (kbase > qw0 + 31) continue;  // every key of this half-chunk lies after my queries
        f32x16 s = f32x16{}, dp = f32x16{};
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) s = mfma32(Tile::row_frag(ks, kt, kk, l32, half), qf[kk], s);
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) dp = mfma32(Tile::row_frag(vs, kt, kk, l32, half), gf[kk], dp);
        const bool diag = kbase + 31 > qw0;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = fast_exp2(__builtin_fmaf(s[r], c, -lse_l));
        if (diag) {  // only the half-chunks on the diagonal pay for the causal mask
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kbase + 8 * (r >> 2) + 4 * half + (r & 3);
            if (key > qpos) s[r] = 0.f;
          }
        }
        if (CH == 32 && pat != 0xF) {  // 16-token blocks: drop the blocks my mask row does not keep
          const int mine = pat >> (2 * (l32 >> 4));
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (!((mine >> (r >> 3)) & 1)) s[r] = 0.f;  // registers 0..7: block 0, 8..15: block 1
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] *= dp[r] - delta_l;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const bf16x8 dsb = pack8(s[8 * u + 0], s[8 * u + 1], s[8 * u + 2], s[8 * u + 3], s[8 * u + 4],
                                   s[8 * u + 5], s[8 * u + 6], s[8 * u + 7]);
#pragma unroll
          for (int dt = 0; dt < D / 32; ++dt)
            acc[dt] = mfma32(Tile::tr_frag(ks, dt, 2 * kt + u, trb), dsb, acc[dt]);
        }
      }
    }

    wait_all_loads();
    __syncthreads();
  }

  if (!wave_active || !my_row_exists) return;
  uint16_t* row = p.dq + q_off + (int64_t)(qw0 + l32) * p.q_st;
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 w;
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = (__bf16)(acc[dt][4 * g + e] * p.scale);
      *reinterpret_cast<bf16x4*>(row + 32 * dt + 8 * g + 4 * half) = w;
    }
}

// ------------------------------------------------------------------------------------ dk, dv

template <int D, int CH>
struct DkvSmem {
  uint16_t q[2][DmaTile<D, CH>::kElems];
  uint16_t g[2][DmaTile<D, CH>::kElems];
  struct RowStats {
    float delta[CH];
    float lse[CH];         // base-2 units
  } rs[2];                 // one 512-byte direct load fills both arrays of a stage
};

// VARLEN: a packed batch of sequences of different lengths.  A key tile's members are columns of
// the whole layout, so the workgroup first drops out if none of them exists in its sequence, skips
// the list entries (query blocks, last first) that lie after the sequence's end, clamps the loads
// of the ragged last chunk and zeroes P and dS for the query rows of it that do not exist.
// STORE: dS, rounded to bf16 as the dK contraction takes it, is also left in the workspace for the dQ
// launch (launch_dq_gemm), 4 KiB per wavefront and step: [half chunk][16-query slab][key][lane half][8
// queries in the order the lane holds them], i.e. each B operand as it is, 1 KiB per store instruction.
template <int D, bool DENSE, int CH, bool VARLEN = false, bool STORE = false>
__global__ __launch_bounds__(kThreads, 2) void dkdv_kernel(const AttnParams p) {
  typedef DmaTile<D, CH> Tile;
  constexpr int QT = CH / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  DkvSmem<D, CH>& sm = *reinterpret_cast<DkvSmem<D, CH>*>(smem_raw);

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int T = p.kv_tiles.tiles_per_head;
  int bh, rank;
  if (!map_workgroup_interleaved(blockIdx.x, p.batch * p.heads, T, bh, rank)) return;
  const int b = bh / p.heads, h = bh - b * p.heads;
  const int tile = DENSE ? rank : p.kv_tiles.order[h * T + rank];  // dense: first key tiles are longest
  const int S = DENSE ? kChunk : p.block_size;
  // 16-token blocks: a list entry is a unit of two query blocks (32 rows, one step) and my 32 key
  // rows are two adjacent mask columns, so a lane's keep pattern is 2 x 2 bits per wavefront
  const bool fine = !DENSE && CH == 32 && S == 16;
  const int Sg = fine ? 32 : S;  // tokens per list entry
  const int cpb = Sg / CH;  // a power of two: / and % below are a shift and a mask
  const int cpb_sh = __builtin_ctz(cpb), cpb_m = cpb - 1;
  int row_base = 0, N = p.seqlen;
  if (VARLEN) {
    const int lo = p.cu_seqlens[b], hi = p.cu_seqlens[b + 1];
    row_base = min(max(lo, 0), p.seqlen);  // whatever the array holds, stay inside the tensors
    N = min(min(max(hi - lo, 0), p.q_rows), p.seqlen - row_base);
  }

  // my 32 key rows
  int kvw0, my_member = 0;
  bool wave_active;
  if (DENSE) {
    kvw0 = tile * kBwdBN + wave * 32;
    wave_active = kvw0 < N;
  } else {
    my_member = (wave * 32) / S;  // with 16-token blocks the first of my two (adjacent) columns
    const int32_t* mem = p.kv_tiles.members + (h * T + tile) * p.kv_tiles.group;
    if (VARLEN) {  // the whole workgroup leaves together when none of its columns is in the sequence
      bool any = false;
      for (int m = 0; m < p.kv_tiles.group; ++m) any = any || (mem[m] >= 0 && mem[m] * S < N);
      if (!any) return;
    }
    const int blk = mem[my_member];
    kvw0 = blk * S + (wave * 32) % S;
    wave_active = blk >= 0 && kvw0 < N;
  }

  const int64_t q_off = (VARLEN ? row_base * p.q_st : b * p.q_sb) + h * p.q_sh;
  const int64_t kv_off = (VARLEN ? row_base * p.kv_st : b * p.kv_sb) + h * p.kv_sh;
  const uint16_t* qb = p.q + q_off;
  const uint16_t* gb = p.d_o + q_off;
  // packed batch: the row statistics are [heads, rows of the tensors]
  const int64_t stats_off = VARLEN ? (int64_t)h * p.seqlen + row_base : ((int64_t)b * p.heads + h) * N;
  const float* lse_b = p.lse2 + stats_off;
  const float* delta_b = p.delta + stats_off;

  int ent_lo = 0, n_ent;
  if (DENSE) {
    n_ent = (N - tile * kBwdBN) / kChunk;  // query chunks at or after the tile's first key
  } else {
    ent_lo = p.kv_tiles.ptr[h * T + tile];
    n_ent = p.kv_tiles.ptr[h * T + tile + 1] - ent_lo;
  }
  const int total = n_ent * cpb;
  // where this wavefront's dS of step 0 goes: unit 2 * (global step) + wave / 2, its keys' half of it
  uint16_t* ds_wave = nullptr;
  if (STORE)
    ds_wave = p.ds_store + ((int64_t)b * p.ds_units + (((int64_t)ent_lo << cpb_sh) * 2 + (wave >> 1))) * 4096 + (wave & 1) * 2048;
  EntryList list;
  if (!DENSE) list.init(p.kv_tiles.ent + ent_lo, n_ent, lane);
  // chunk `it` of the tile's list: its first row, and whether my mask row / column keeps it
  // `pat` (16-token blocks only): bit 2m + c set when query block c of the unit keeps my column m
  auto chunk_of = [&](int it, int& q0, bool& keep, int& pat) {
    pat = 0xF;
    if (DENSE) {
      q0 = N - CH - it * CH;  // from the last query chunk down, like the sparse lists
      keep = true;
    } else {
      const int e = list.get((it >> cpb_sh), lane);
      q0 = (e >> 16) * Sg + (cpb - 1 - (it & cpb_m)) * CH;
      if (fine) {
        pat = (e >> (4 * wave)) & 0xF;
        keep = pat != 0;
      } else {
        keep = (e >> my_member) & 1;
      }
    }
  };
  // first row of chunk it+1, right after chunk_of(it)
  auto next_chunk_of = [&](int it, int& q0_n) {
    if (DENSE) {
      q0_n = N - CH - (it + 1) * CH;
    } else {
      const int e = ((it + 1) >> cpb_sh) == (it >> cpb_sh) ? list.get((it >> cpb_sh), lane) : list.peek_next((it >> cpb_sh));
      q0_n = (e >> 16) * Sg + (cpb - 1 - ((it + 1) & cpb_m)) * CH;
    }
  };

  const typename Tile::Plan plan = Tile::plan(p.q_st, wave, lane);
  const uint32_t stats_gap = (uint32_t)((const char*)lse_b - (const char*)delta_b);
  // `ln` is the lane number.  The loop passes a copy the optimiser cannot see through, so that
  // what is derived from it is recomputed each step (a few integer operations) rather than kept in
  // registers across the loop: this kernel has no registers to spare, and a spilled constant costs
  // a wait for all outstanding loads when it is fetched back.
  auto issue_chunk = [&](int q0, int buf, int ln) {
    if (VARLEN && q0 + CH > N) {  // ragged end of the sequence: rows past it fetch its last row instead
      // (a list need not be in descending order, so a chunk that lies wholly after the sequence's end
      // can turn up anywhere in it: it fetches the last row 64 times and nothing uses it)
      const int qs = min(q0, N - 1);
      const typename Tile::Plan pr = Tile::plan_rows(p.q_st, wave, ln, N - qs);
      Tile::issue(pr, qb + (int64_t)qs * p.q_st, sm.q[buf], wave);
      Tile::issue(pr, gb + (int64_t)qs * p.q_st, sm.g[buf], wave);
    } else {
      Tile::issue(plan, qb + (int64_t)q0 * p.q_st, sm.q[buf], wave);
      Tile::issue(plan, gb + (int64_t)q0 * p.q_st, sm.g[buf], wave);
    }
    // CH floats of each array: the first CH/4 lanes fetch delta, the next CH/4 lanes lse, 16 bytes
    // each, in one direct load issued by the wavefront that has one load fewer than the others in the two tiles
    constexpr int NL = CH / 4;  // lanes per array, 16 bytes each
    if (wave == 3 && ln < 2 * NL)
      dma16(delta_b + (VARLEN && q0 >= N ? 0 : q0), 16 * ln + (ln < NL ? 0u : stats_gap - 16u * NL), lds_addr(&sm.rs[buf]));
  };
  // first step: a packed sequence skips the leading chunks of query blocks that lie after its end (most
  // lists start at the layout's last row; such chunks further on are walked without being used)
  int it0 = 0;
  if (VARLEN) {
    for (; it0 < total; ++it0) {
      int q0, pat;
      bool keep;
      chunk_of(it0, q0, keep, pat);
      if (q0 < N) break;
    }
  }
  if (it0 < total) {
    int q0, pat;
    bool keep;
    chunk_of(it0, q0, keep, pat);
    issue_chunk(q0, it0 & 1, lane);
  }

  bf16x8 kf[D / 16], vf[D / 16];  // K and V fragments (B operands), lane = key
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) {
    if (wave_active) {
      const int64_t o = kv_off + (int64_t)(VARLEN ? min(kvw0 + l32, N - 1) : kvw0 + l32) * p.kv_st + 16 * kk + 8 * half;
      kf[kk] = *reinterpret_cast<const bf16x8*>(p.k + o);
      vf[kk] = *reinterpret_cast<const bf16x8*>(p.v + o);
    } else {
      kf[kk] = bf16x8{};
      vf[kk] = bf16x8{};
    }
  }

  f32x16 acc_dk[D / 32], acc_dv[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) {
    acc_dk[dt] = f32x16{};
    acc_dv[dt] = f32x16{};
  }
  const float c = p.scale_log2e;

  wait_all_loads();
  __syncthreads();

  for (int it = it0; it < total; ++it) {
    const int buf = it & 1;
    int ln = lane;
    asm volatile("" : "+v"(ln));
    int q0, pat;
    bool keep;
    chunk_of(it, q0, keep, pat);
    if (it + 1 < total) {
      int q1;
      next_chunk_of(it, q1);
      issue_chunk(q1, buf ^ 1, ln);
    }

    int stores = 0;  // dS stores of this step (wave-uniform)
    uint16_t* ds_step = STORE ? ds_wave + (int64_t)it * 8192 : nullptr;
    if (wave_active && keep && q0 + CH - 1 >= kvw0) {
      const uint16_t* qs = sm.q[buf];
      const uint16_t* gs = sm.g[buf];
      const int l32 = ln & 31, half = ln >> 5;
      const int trb = Tile::tr_base(ln);
      const int key = kvw0 + l32;
      const int mine = pat >> (2 * (l32 >> 4));  // 16-token blocks: bit c = query block c keeps my key
#pragma unroll
      for (int qt = 0; qt < QT; ++qt) {
        const int qbase = q0 + 32 * qt;
        if (qbase + 31 < kvw0) continue;  // every query of this half-chunk lies before my keys
        if (VARLEN && qbase >= N) continue;  // ... or after the end of my sequence
        f32x16 s = f32x16{}, dp = f32x16{};
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) s = mfma32(Tile::row_frag(qs, qt, kk, l32, half), kf[kk], s);
#pragma unroll
        for (int kk = 0; kk < D / 16; ++kk) dp = mfma32(Tile::row_frag(gs, qt, kk, l32, half), vf[kk], dp);
        // causal mask: key > qbase + 8g + 4 half + e  <=>  lim > 8g + e, a compare with a constant;
        // away from the diagonal lim = -1 and nothing is dropped
        // (the dense instantiation keeps the plain comparison: with this form the compiler spills there)
        const bool diag = qbase < kvw0 + 31;
        const int lim = diag ? key - qbase - 4 * half : -1;
        // packed batch: query row 8g + 4 half + e of the half-chunk exists iff 8g + e < rows_left
        const int rows_left = VARLEN ? N - qbase - 4 * half : 0;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int r0 = 32 * qt + 8 * g + 4 * half;
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(&sm.rs[buf].lse[r0]);
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(&sm.rs[buf].delta[r0]);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = 4 * g + e;
            float pr = fast_exp2(__builtin_fmaf(s[r], c, -l4[e]));
            if (DENSE ? (diag && key > q0 + r0 + e) : (lim > 8 * g + e)) pr = 0.f;
            if (CH == 32 && !((mine >> (g >> 1)) & 1)) pr = 0.f;  // query rows 0..15: block 0, 16..31: block 1
            float ds = pr * (dp[r] - d4[e]);
            if (VARLEN && 8 * g + e >= rows_left) {  // a row past the sequence's end: its statistics are not its own
              pr = 0.f;
              ds = 0.f;
            }
            s[r] = pr;
            dp[r] = ds;
          }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const bf16x8 pb = pack8(s[8 * u + 0], s[8 * u + 1], s[8 * u + 2], s[8 * u + 3], s[8 * u + 4],
                                  s[8 * u + 5], s[8 * u + 6], s[8 * u + 7]);
          const bf16x8 dsb = pack8(dp[8 * u + 0], dp[8 * u + 1], dp[8 * u + 2], dp[8 * u + 3], dp[8 * u + 4],
                                   dp[8 * u + 5], dp[8 * u + 6], dp[8 * u + 7]);
          if constexpr (STORE) {
            const uint32_t off = 16u * (2 * l32 + half) + 1024u * (2 * qt + u);
            // non-temporal: written once here and read by a later launch, it should not push the Q / dO
            // blocks this kernel re-reads out of L2
            __builtin_nontemporal_store(__builtin_bit_cast(u32x4, dsb),
                                        reinterpret_cast<u32x4*>(reinterpret_cast<unsigned char*>(ds_step) + off));
            ++stores;
          }
#pragma unroll
          for (int dt = 0; dt < D / 32; ++dt) {
            acc_dv[dt] = mfma32(Tile::tr_frag(gs, dt, 2 * qt + u, trb), pb, acc_dv[dt]);
            acc_dk[dt] = mfma32(Tile::tr_frag(qs, dt, 2 * qt + u, trb), dsb, acc_dk[dt]);
          }
        }
      }
    }

    // the next chunk has landed; this step's dS stores, issued after its loads, may stay in flight
    if (STORE && stores == 4)
      wait_loads_but<4>();
    else if (STORE && stores == 2)
      wait_loads_but<2>();
    else
      wait_all_loads();
    __syncthreads();
  }

  if (!wave_active || (VARLEN && kvw0 + l32 >= N)) return;
  if (!VARLEN && CH == 64) {
    // Whole rows exist: dK and dV go out through LDS (free since the loop's last barrier; each
    // wavefront uses regions of its own, so no barrier).  A lane holds its row's features four at a
    // time, and storing them from there touches 32 rows per instruction with 16 bytes each; read back
    // 16 bytes per lane, row after row, an instruction stores four whole rows.
    constexpr int RS = D + 8;  // staging row stride (elements)
    static_assert(4 * 32 * (D + 8) <= 2 * DmaTile<D, CH>::kElems || CH != 64, "the staging rows fit two stages");
    uint16_t* sk_ = &sm.q[0][0] + wave * 32 * RS;
    uint16_t* sv_ = &sm.g[0][0] + wave * 32 * RS;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 wk, wv;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          wk[e] = (__bf16)(acc_dk[dt][4 * g + e] * p.scale);
          wv[e] = (__bf16)(acc_dv[dt][4 * g + e]);
        }
        *reinterpret_cast<bf16x4*>(sk_ + l32 * RS + 32 * dt + 8 * g + 4 * half) = wk;
        *reinterpret_cast<bf16x4*>(sv_ + l32 * RS + 32 * dt + 8 * g + 4 * half) = wv;
      }
    uint16_t* dk_base = p.dk + kv_off + (int64_t)kvw0 * p.kv_st;
    uint16_t* dv_base = p.dv + kv_off + (int64_t)kvw0 * p.kv_st;
    constexpr int PPR = D / 8, RPI = 64 / PPR;  // 16-byte pieces per row, rows per instruction
#pragma unroll
    for (int i = 0; i < 32 / RPI; ++i) {
      const int r = RPI * i + lane / PPR, piece = lane % PPR;
      *reinterpret_cast<u32x4*>(dk_base + (int64_t)r * p.kv_st + 8 * piece) = *reinterpret_cast<const u32x4*>(sk_ + r * RS + 8 * piece);
      *reinterpret_cast<u32x4*>(dv_base + (int64_t)r * p.kv_st + 8 * piece) = *reinterpret_cast<const u32x4*>(sv_ + r * RS + 8 * piece);
    }
    return;
  }
  uint16_t* dk_row = p.dk + kv_off + (int64_t)(kvw0 + l32) * p.kv_st;
  uint16_t* dv_row = p.dv + kv_off + (int64_t)(kvw0 + l32) * p.kv_st;
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 wk, wv;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        wk[e] = (__bf16)(acc_dk[dt][4 * g + e] * p.scale);
        wv[e] = (__bf16)(acc_dv[dt][4 * g + e]);
      }
      *reinterpret_cast<bf16x4*>(dk_row + 32 * dt + 8 * g + 4 * half) = wk;
      *reinterpret_cast<bf16x4*>(dv_row + 32 * dt + 8 * g + 4 * half) = wv;
    }
}

// A kernel's dynamic LDS limit is a per-device attribute: remember, per device, that it is set.
constexpr int kMaxDevices = 64;
struct SmemSet {
  std::atomic<unsigned char> done[kMaxDevices];
};

template <class K>
hipError_t set_smem(K kernel, size_t bytes, SmemSet& flags) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < kMaxDevices;
  if (tracked && flags.done[dev].load(std::memory_order_acquire)) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)bytes);
  if (e == hipSuccess && tracked) flags.done[dev].store(1, std::memory_order_release);
  return e;
}

template <int D, bool DENSE, int CH, bool VARLEN = false>
hipError_t launch_one(const AttnParams& p, int stages, hipStream_t stream) {
  static SmemSet dq_set, dkdv_set;  // zero-initialised
  hipError_t e = set_smem(&dq_kernel<D, DENSE, CH, VARLEN>, sizeof(DqSmem<D, CH>), dq_set);
  if (e != hipSuccess) return e;
  e = set_smem(&dkdv_kernel<D, DENSE, CH, VARLEN>, sizeof(DkvSmem<D, CH>), dkdv_set);
  if (e != hipSuccess) return e;

  const int64_t rows = (int64_t)p.batch * p.heads * p.seqlen;
  constexpr int RPB = 256 / (D / 8);
  const int bh = p.batch * p.heads;
  if constexpr (D == 128 && !DENSE && CH == 64 && !VARLEN) {
    if (p.ds_store) {
      // The backward that keeps dS: delta, then dK/dV (5 contractions' worth of work less the dQ one,
      // leaving dS in the workspace), then dQ = scale * dS K - nothing is computed twice.
      static SmemSet store_set;
      e = set_smem(&dkdv_kernel<D, false, CH, false, true>, sizeof(DkvSmem<D, CH>), store_set);
      if (e != hipSuccess) return e;
      if (stages & kBwdDelta) {
        hipLaunchKernelGGL((delta_kernel<D>), dim3((unsigned)((rows + RPB - 1) / RPB)), dim3(256), 0, stream, p);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
      }
      if (stages & kBwdDkDv) {
        hipLaunchKernelGGL((dkdv_kernel<D, false, CH, false, true>), dim3(grid_for(bh, p.kv_tiles.tiles_per_head)),
                           dim3(kThreads), sizeof(DkvSmem<D, CH>), stream, p);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
      }
      if (stages & kBwdDq) e = launch_dq_gemm(p, stream);
      return e;
    }
  }
  // The dQ kernel computes delta itself and leaves it (and LSE in base-2 units) in the workspace,
  // so it runs first and the stand-alone delta kernel only when dQ is not part of the call
  // (a packed batch is always a whole backward).
  if (!VARLEN && (stages & kBwdDelta) && !(stages & kBwdDq)) {
    hipLaunchKernelGGL((delta_kernel<D>), dim3((unsigned)((rows + RPB - 1) / RPB)), dim3(256), 0, stream, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if ((stages & kBwdDq) && VARLEN && CH == 64 && dq_pipe_applies(p, DENSE)) {
    // packed batch: whole 128-row tiles by the fast path, each sequence's partial last tile by dq_kernel
    e = launch_dq_pipe(p, DENSE, stream);
    if (e != hipSuccess) return e;
    AttnParams tail = p;
    tail.varlen_tail = 1;
    hipLaunchKernelGGL((dq_kernel<D, DENSE, CH, VARLEN>), dim3(grid_for(bh, 1)), dim3(kThreads), sizeof(DqSmem<D, CH>),
                       stream, tail);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  } else if ((stages & kBwdDq) && !VARLEN && CH == 64 && dq_pipe_applies(p, DENSE)) {
    e = launch_dq_pipe(p, DENSE, stream);
    if (e != hipSuccess) return e;
  } else if (stages & kBwdDq) {
    // one slot per 128-row tile: of the sequence, or of the longest length a packed batch allows
    const int q_tiles = VARLEN ? (p.q_rows + kBwdBM - 1) / kBwdBM : p.q_tiles.tiles_per_head;
    hipLaunchKernelGGL((dq_kernel<D, DENSE, CH, VARLEN>), dim3(grid_for(bh, q_tiles)), dim3(kThreads),
                       sizeof(DqSmem<D, CH>), stream, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (stages & kBwdDkDv) {
    hipLaunchKernelGGL((dkdv_kernel<D, DENSE, CH, VARLEN>), dim3(grid_for(bh, p.kv_tiles.tiles_per_head)),
                       dim3(kThreads), sizeof(DkvSmem<D, CH>), stream, p);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace

hipError_t launch_bwd(const AttnParams& p, bool dense, int stages, hipStream_t stream) {
  if (!dense && p.cu_seqlens) {  // packed variable-length batch: a whole backward, sparse layouts only
    if (p.block_size <= 32)
      return p.head_dim == 128 ? launch_one<128, false, 32, true>(p, kBwdAll, stream)
                               : launch_one<64, false, 32, true>(p, kBwdAll, stream);
    return p.head_dim == 128 ? launch_one<128, false, kChunk, true>(p, kBwdAll, stream)
                             : launch_one<64, false, kChunk, true>(p, kBwdAll, stream);
  }
  // 32-token mask blocks are walked in steps of 32 rows, everything else in steps of 64
  if (!dense && p.block_size <= 32)
    return p.head_dim == 128 ? launch_one<128, false, 32>(p, stages, stream) : launch_one<64, false, 32>(p, stages, stream);
  if (p.head_dim == 128)
    return dense ? launch_one<128, true, kChunk>(p, stages, stream) : launch_one<128, false, kChunk>(p, stages, stream);
  return dense ? launch_one<64, true, kChunk>(p, stages, stream) : launch_one<64, false, kChunk>(p, stages, stream);
}

}  // namespace s2
