// Forward kernel for head_dim 128 and mask blocks of 64 or 128 tokens: the fast path of
// block-sparse causal attention (section 3.2: K/V tiles of the kept blocks only go through on-chip
// memory; section 4.2: which blocks a head keeps).  Same tiles, lists, staging and orientation as
// fwd_kernel.hip (a 128-row query tile that spans several mask rows, four wavefronts of 32 query
// rows, scores computed transposed so that a lane owns one query); what differs is the inner loop:
//
//   * it is software pipelined by one step: while the matrix pipe computes the scores of step i+1
//     and then P(i) V(i), the vector pipe turns the scores of step i into probabilities and finds
//     the maximum of step i+1;
//   * the interleave is written out by hand, one MFMA per slot with its share of the vector work,
//     LDS reads and direct loads, and fenced so that the compiler keeps it.  Measured on gfx950, a
//     SIMD only overlaps matrix and vector instructions that alternate finely in the instruction
//     streams; two wavefronts per SIMD then hide each other's scalar work and waits;
//   * the running maximum is only moved when a new score exceeds it by more than 2^kTau: the
//     accumulators are rescaled in a rarely taken branch instead of in every step;
//   * the direct loads of a tile are issued four to a write of M0 (their LDS targets are told apart
//     by the instruction's immediate offset).
#include <hip/hip_runtime.h>

#include "config.h"
#include "device_util.h"
#include "kernels.h"
#include "sched_util.h"

namespace s2 {

namespace {

constexpr float kNegInf = -__builtin_inff();
constexpr float kTau = 8.0f;  // log2 units a score may exceed the reference maximum by

// VARLEN: a packed batch of sequences of different lengths.  A workgroup finds its sequence's rows in
// cu_seqlens and treats them as a sequence of its own; this kernel computes the whole 128-row tiles of
// each sequence (all their keys exist), a partial last tile is left to fwd_kernel.
template <int D, bool DENSE, bool VARLEN = false>
__global__ __launch_bounds__(kThreads, 2) void fwd_pipe_kernel(const AttnParams p) {
  typedef DmaTile<D, 64, 4> Tile;
  __shared__ __attribute__((aligned(16))) uint16_t sk[2][Tile::kElems];
  __shared__ __attribute__((aligned(16))) uint16_t sv[2][Tile::kElems];
  constexpr int BM = kFwdBM, MW = 32, CH = 64;
  constexpr int KK = D / 16, DT = D / 32;
  constexpr int NQK = 2 * KK;  // MFMAs of the score contraction per step
  constexpr int NPV = 4 * DT;  // MFMAs of the second contraction per step
  constexpr int NG = Tile::kGroups;
  constexpr int kLead = 5, kRing = kLead + 1;  // LDS fragments are requested kLead MFMAs ahead (3 to 7 measure the same)
  static_assert(D == 128, "the slot schedule below is laid out for head_dim 128");
  static_assert(NQK == 16 && NPV == 16, "32 slots");

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int T = p.fwd_tiles.tiles_per_head;    // tiles of the whole sequence (indexes the lists)
  const int T_run = p.q_rows / BM;             // tiles this launch computes
  int bh, rank;
  if (!map_workgroup(blockIdx.x, p.batch * p.heads, T_run, bh, rank)) return;
  const int b = bh / p.heads, h = bh - b * p.heads;
  const bool whole = !VARLEN && p.q_row0 == 0 && T_run == T;
  int tile = (DENSE || !whole) ? p.q_row0 / BM + (T_run - 1 - rank) : p.fwd_tiles.order[h * T + rank];
  int N = p.seqlen, row_base = 0;  // my sequence's length, and the rows of the tensors before it
  if (VARLEN) {
    const int lo = p.cu_seqlens[b], hi = p.cu_seqlens[b + 1];
    row_base = min(max(lo, 0), p.seqlen);  // whatever the array holds, stay inside the tensors
    N = min(min(max(hi - lo, 0), p.q_rows), p.seqlen - row_base);
    const int T_full = N / BM;
    if (rank >= T_full) return;
    tile = T_full - 1 - rank;
  }
  const int S = DENSE ? CH : p.block_size;  // 64 or 128
  const int cpb_sh = S == 128 ? 1 : 0, cpb_m = (1 << cpb_sh) - 1;
  const int qw0 = tile * BM + wave * MW;    // first query row of this wavefront (sequence position)
  const int ql0 = qw0 - p.q_row0;           // the same as a row of q / o / lse
  const int my_member = (qw0 / S) - tile * (BM / S);

  const int64_t q_off = (VARLEN ? row_base * p.q_st : b * p.q_sb) + h * p.q_sh;
  const int64_t kv_off = (VARLEN ? row_base * p.kv_st : b * p.kv_sb) + h * p.kv_sh;
  // minus the bias the grouped direct loads put into their lane offsets
  const uint16_t* kb = p.k + kv_off - Tile::kBias / 2;
  const uint16_t* vb = p.v + kv_off - Tile::kBias / 2;

  int ent_lo = 0, n_ent;
  if (DENSE) {
    n_ent = min(N, (tile + 1) * BM) / CH;
  } else {
    ent_lo = p.fwd_tiles.ptr[h * T + tile];
    n_ent = p.fwd_tiles.ptr[h * T + tile + 1] - ent_lo;
  }
  const int total = n_ent << cpb_sh;
  if (total <= 0) return;
  EntryList list;
  if (!DENSE) list.init(p.fwd_tiles.ent + ent_lo, n_ent, lane);

  // Q^T fragments stay in registers for the whole tile (B operands of the score MFMAs)
  bf16x8 qf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk)
    qf[kk] = *reinterpret_cast<const bf16x8*>(p.q + q_off + (int64_t)(ql0 + l32) * p.q_st + 16 * kk + 8 * half);

  // step j of the tile's list (clamped to the last one): its first key row, and whether this
  // wavefront has anything to compute there (its mask row keeps the block, and not every key lies
  // after every one of its queries)
  auto chunk_at = [&](int j, int& kv0, bool& act) S2_INLINE {
    const bool inside = j < total;
    j = min(j, total - 1);
    if (DENSE) {
      kv0 = j * CH;
      act = inside && kv0 <= qw0 + MW - 1;
    } else {
      const int e = list.peek(j >> cpb_sh);
      kv0 = (e >> 16) * S + (j & cpb_m) * CH;
      act = inside && ((e >> my_member) & 1) && kv0 <= qw0 + MW - 1;
    }
  };

  f32x16 acc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) acc[dt] = f32x16{};
  float m_ref = kNegInf;  // reference maximum (raw scores) of my query
  float mc = kNegInf;     // the same times scale * log2(e); 0 while nothing was seen
  float l_run = 0.f;      // sum of the probabilities over my half's key rows
  const float c = p.scale_log2e;
  const typename Tile::BlockPlan plan = Tile::block_plan(p.kv_st, wave, lane);
  const int trb = Tile::tr_base(lane);

  // scores [parity of the step][32-key half].  Zero to begin with: the registers of a step this
  // wavefront skips are still run through the exponential (with a shift of -inf) when the next step
  // is its own, so they must never hold a NaN; after a step they hold its probabilities.
  f32x16 s[2][2];
#pragma unroll
  for (int i = 0; i < 4; ++i) s[i >> 1][i & 1] = f32x16{};

  // ------------------------------------------------------------------ pieces of a step
  // The A operands of a step's 32 MFMAs - 16 row fragments of K, then 16 transposed fragments of
  // V - pass through one ring of kRing registers sets, each requested from LDS kLead slots before
  // the MFMA that uses it.
  // fragment f: K fragment (kk = f / 2, key half f % 2) for f < NQK, else V^T fragment f - NQK
  // (group (f - NQK) / DT = key half, 16-key slab; feature tile (f - NQK) % DT)
  auto frag_load = [&](int f, const uint16_t* ks, const uint16_t* vs, bf16x8 (&fr)[kRing]) S2_INLINE {
    if (f < NQK)
      fr[f % kRing] = Tile::row_frag(ks, f & 1, f >> 1, l32, half);
    else
      fr[f % kRing] = Tile::tr_frag(vs, (f - NQK) % DT, (f - NQK) / DT, trb);
  };
  // MFMA n of the score contraction of a step: kk = n / 2, key half = n % 2; fragment n
  auto qk_mfma = [&](int n, f32x16 (&sn)[2], const bf16x8 (&fr)[kRing]) S2_INLINE {
    const int kk = n >> 1, kt = n & 1;
    sn[kt] = mfma32(fr[n % kRing], qf[kk], kk == 0 ? f32x16{} : sn[kt]);
  };
  // MFMA n of the second contraction: group g = n / DT (key half g / 2, 16-key slab g % 2),
  // feature tile n % DT; fragment NQK + n
  auto pv_mfma = [&](int n, const bf16x8 (&fr)[kRing], const u32x4 (&pb)[4]) S2_INLINE {
    acc[n % DT] = mfma32(fr[(NQK + n) % kRing], __builtin_bit_cast(bf16x8, pb[n / DT]), acc[n % DT]);
  };
  // The probabilities of a step are made in three stages - scale and shift, exponential, sum and
  // pack - that a slot applies to different elements, so that no instruction waits for the one
  // before it.  Elements are numbered in the order the second contraction uses them:
  // e = 8 * g + i is score register 8 * (g % 2) + i of key half g / 2.  Stages 1 and 2 work in
  // place, in the score registers.
  auto p_stage1 = [&](int e0, int e1, f32x16 (&sc)[2]) S2_INLINE {
#pragma unroll
    for (int e = max(e0, 0); e < min(e1, 32); ++e) {
      const int g = e >> 3, r = 8 * (g & 1) + (e & 7);
      sc[g >> 1][r] = __builtin_fmaf(sc[g >> 1][r], c, -mc);
    }
  };
  auto p_stage2 = [&](int e0, int e1, f32x16 (&sc)[2]) S2_INLINE {
#pragma unroll
    for (int e = max(e0, 0); e < min(e1, 32); ++e) {
      const int g = e >> 3, r = 8 * (g & 1) + (e & 7);
      sc[g >> 1][r] = fast_exp2(sc[g >> 1][r]);
    }
  };
  auto p_stage3 = [&](int e0, int e1, f32x16 (&sc)[2], u32x4 (&pb)[4]) S2_INLINE {
#pragma unroll
    for (int e = max(e0, 0); e < min(e1, 32); ++e) {
      const int g = e >> 3, i = e & 7, r = 8 * (g & 1) + i;
      // the sum takes the unrounded probabilities: LSE is held to 1e-3, which a sum of bf16 values
      // cannot promise for rows with one or two keys
      l_run += sc[g >> 1][r];
      if (i & 1) {
        pb[g][i >> 1] = pack2(sc[g >> 1][r - 1], sc[g >> 1][r]);
      }
    }
  };
  // element index reached after slot sl: five elements every four slots
  auto p_upto = [](int sl) S2_INLINE { return (5 * (sl + 1)) / 4; };
  auto mask_diag = [&](f32x16 (&sn)[2], int kv0) S2_INLINE {
    const int qpos = qw0 + l32;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = kv0 + 32 * kt + 8 * (r >> 2) + 4 * half + (r & 3);
        if (key > qpos) sn[kt][r] = kNegInf;
      }
  };
  // running maximum over score registers r0 .. r1-1 (of 32)
  auto max_part = [&](int r0, int r1, const f32x16 (&sn)[2], float& mx) S2_INLINE {
#pragma unroll
    for (int r = r0; r < r1; r += 2) mx = fmaxf(fmaxf(mx, sn[r >> 4][r & 15]), sn[r >> 4][(r + 1) & 15]);
  };
  // moves the reference maximum where the new scores exceed it by more than 2^kTau (always for the
  // first step, when it is -inf) and rescales what has been accumulated so far
  auto update_ref = [&](float mx) S2_INLINE {
    mx = max_halves(mx);
    if (__any(__builtin_fmaf(mx, c, -mc) > kTau)) {
      const float m_new = fmaxf(m_ref, mx);
      const float m_use = (m_new == kNegInf) ? 0.f : m_new;
      const float alpha = fast_exp2((m_ref - m_use) * c);
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[dt][r] *= alpha;
      m_ref = m_new;
      mc = m_use * c;
    }
  };
  // maximum of the scores in sn (masked on the diagonal), then the reference maximum
  auto finish_scores = [&](f32x16 (&sn)[2], int kv0, bool act, bool masked, float mx) S2_INLINE {
    if (masked) {
      mask_diag(sn, kv0);
      mx = kNegInf;
      max_part(0, 32, sn, mx);
    }
    if (!act) mx = kNegInf;
    update_ref(mx);
  };

  // ------------------------------------------------------------------ prologue
  // A step this wavefront has nothing to compute in (its mask row drops the block, or every key
  // lies after its queries) runs through the same instruction stream when the step before or
  // after it is its own, with its scores kept out of the maximum and its probabilities forced to
  // zero; two such steps in a row are skipped.
  int kv0_c, kv0_n, kv0_nn;
  bool act_c, act_n, act_nn;
  chunk_at(0, kv0_c, act_c);
  chunk_at(1, kv0_n, act_n);
  static_for<NG>([&](auto gc) S2_INLINE {
    constexpr int g = decltype(gc)::value;
    Tile::template issue_group<g>(plan, kb + (int64_t)kv0_c * p.kv_st, sk[0], wave);
    Tile::template issue_group<g>(plan, vb + (int64_t)kv0_c * p.kv_st, sv[0], wave);
    Tile::template issue_group<g>(plan, kb + (int64_t)kv0_n * p.kv_st, sk[1], wave);
  });
  wait_all_loads();
  __syncthreads();
  if (act_c) {
    bf16x8 fr[kRing];
#pragma unroll
    for (int f = 0; f < kLead; ++f) frag_load(f, sk[0], sv[0], fr);
    static_for<NQK>([&](auto nc) S2_INLINE {
      constexpr int n = decltype(nc)::value;
      if constexpr (n + kLead < NQK) frag_load(n + kLead, sk[0], sv[0], fr);
      qk_mfma(n, s[0], fr);
      S2_FENCE();
    });
  }
  finish_scores(s[0], kv0_c, act_c, true, kNegInf);  // `true`: the first step may be the diagonal
  __syncthreads();  // all wavefronts are done with K(0) before step 0 loads K(2) over it

  // ------------------------------------------------------------------ one step
  // On entry: K(it+1) and V(it) are in LDS, sc holds the scores of step it and the reference
  // maximum already covers them.
  auto step = [&](int it, f32x16 (&sc)[2], f32x16 (&sn)[2]) S2_INLINE {
    const int par = it & 1;
    chunk_at(it + 2, kv0_nn, act_nn);
    const uint16_t* kg = kb + (int64_t)kv0_nn * p.kv_st;  // K(it+2) -> the stage K(it) was in
    const uint16_t* vg = vb + (int64_t)kv0_n * p.kv_st;   // V(it+1) -> the stage V(it-1) was in
    const uint16_t* ks = sk[par ^ 1];
    const uint16_t* vs = sv[par];
    uint16_t* kn = sk[par];
    uint16_t* vn = sv[par ^ 1];
    // group d of this step's direct loads: 0..NG-1 for K, NG..2*NG-1 for V
    auto dma = [&](auto dc) S2_INLINE {
      constexpr int d = decltype(dc)::value;
      if constexpr (d < NG)
        Tile::template issue_group<d>(plan, kg, kn, wave);
      else if constexpr (d < 2 * NG)
        Tile::template issue_group<d - NG>(plan, vg, vn, wave);
    };
    if (act_c || act_n) {
      const bool mask_next = kv0_n + CH - 1 > qw0;
      // a step that is not mine: every probability exp2(s*c - inf) = 0
      const float mc_keep = mc;
      if (!act_c) mc = __builtin_inff();
      bf16x8 fr[kRing];
      u32x4 pb[4];
      float mx = kNegInf;
#pragma unroll
      for (int f = 0; f < kLead; ++f) frag_load(f, ks, vs, fr);
      S2_FENCE();
      // NQK + NPV slots, one MFMA each
      static_for<NQK + NPV>([&](auto slc) S2_INLINE {
        constexpr int sl = decltype(slc)::value;
        if constexpr (sl + kLead < NQK + NPV) frag_load(sl + kLead, ks, vs, fr);
        if constexpr (sl < NQK)
          qk_mfma(sl, sn, fr);
        else
          pv_mfma(sl - NQK, fr, pb);
        // probabilities of this step, five elements every four slots, each stage one slot behind
        // the one before it (elements 8 g .. 8 g + 7 are packed by slot 7 g + 8 at the latest,
        // their MFMAs start at slot 16 + 4 g)
        p_stage1(p_upto(sl - 1), p_upto(sl), sc);
        p_stage2(p_upto(sl - 2), p_upto(sl - 1), sc);
        p_stage3(p_upto(sl - 3), p_upto(sl - 2), sc, pb);
        // maximum of the next step's scores, once its MFMAs are done
        if constexpr (sl >= 18 && sl < 26) max_part(4 * (sl - 18), 4 * (sl - 18) + 4, sn, mx);
        // Nothing to execute: ties the running sum and maximum to this slot, or the optimiser
        // collects their additions and comparisons after the last MFMA.
        asm volatile("" : "+v"(l_run), "+v"(mx));
        if constexpr (sl < 2 * NG) dma(std::integral_constant<int, sl>{});
        S2_FENCE();
      });
      mc = mc_keep;
      finish_scores(sn, kv0_n, act_n, mask_next, mx);
    } else {
      static_for<2 * NG>([&](auto dc) S2_INLINE { dma(dc); });
    }
    if (!DENSE) (void)list.get(min(it + 1, total - 1) >> cpb_sh, lane);  // keeps the entry window moving
    kv0_c = kv0_n;
    act_c = act_n;
    kv0_n = kv0_nn;
    act_n = act_nn;
    wait_all_loads();
    __syncthreads();
  };

  int it = 0;
  for (; it + 1 < total; it += 2) {
    step(it, s[0], s[1]);
    step(it + 1, s[1], s[0]);
  }
  if (it < total) step(it, s[0], s[1]);

  // ------------------------------------------------------------------ epilogue
  // O = acc / l goes out through LDS (free since the loop's last barrier; each wavefront uses a
  // region of its own, so no barrier): a lane holds its row's features four at a time, and storing
  // them from there would touch 32 rows per instruction with 16 bytes each; read back 16 bytes per
  // lane, row after row, an instruction stores four whole rows.
  const float l_tot = sum_halves(l_run);
  const float inv = 1.0f / l_tot;
  constexpr int RS = D + 8;  // staging row stride (elements): 8-byte writes of a row group spread over the banks
  uint16_t* stage = sk[0] + wave * MW * RS;
  static_assert(4 * MW * RS <= 2 * Tile::kElems, "the staging rows fit the K stages");
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 w;
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = (__bf16)(acc[dt][4 * g + e] * inv);
      *reinterpret_cast<bf16x4*>(stage + l32 * RS + 32 * dt + 8 * g + 4 * half) = w;
    }
  uint16_t* obase = p.o + q_off + (int64_t)ql0 * p.q_st;
#pragma unroll
  for (int i = 0; i < MW / 4; ++i) {
    const int r = 4 * i + (lane >> 4), piece = lane & 15;
    const u32x4 x = *reinterpret_cast<const u32x4*>(stage + r * RS + 8 * piece);
    *reinterpret_cast<u32x4*>(obase + (int64_t)r * p.q_st + 8 * piece) = x;
  }
  const int64_t lse_row = VARLEN ? (int64_t)h * p.seqlen + row_base + ql0 + l32  // [heads, rows of the tensors]
                                 : ((int64_t)b * p.heads + h) * p.q_rows + ql0 + l32;
  if (half == 0) p.lse[lse_row] = m_ref * p.scale + __logf(l_tot);
}

}  // namespace

bool fwd_pipe_applies(const AttnParams& p, bool dense) {
  if (p.cu_seqlens)  // packed batch: the whole tiles of each sequence
    return !dense && p.head_dim == 128 && p.block_size >= 64 && p.q_row0 == 0 && p.q_rows >= kFwdBM;
  return p.head_dim == 128 && (dense || p.block_size >= 64) && p.q_rows % 128 == 0 && p.q_row0 % 128 == 0;
}

hipError_t launch_fwd_pipe(const AttnParams& p, bool dense, hipStream_t stream) {
  const int grid = grid_for(p.batch * p.heads, p.q_rows / kFwdBM);
  if (p.cu_seqlens)
    hipLaunchKernelGGL((fwd_pipe_kernel<128, false, true>), dim3(grid), dim3(kThreads), 0, stream, p);
  else if (dense)
    hipLaunchKernelGGL((fwd_pipe_kernel<128, true>), dim3(grid), dim3(kThreads), 0, stream, p);
  else
    hipLaunchKernelGGL((fwd_pipe_kernel<128, false>), dim3(grid), dim3(kThreads), 0, stream, p);
  return hipGetLastError();
}

}  // namespace s2
