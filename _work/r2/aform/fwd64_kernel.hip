// Forward kernel for head_dim 128 and mask blocks of 64 or 128 tokens: the fast path of
// block-sparse causal attention (section 3.2: K/V tiles of the kept blocks only go through on-chip
// memory; section 4.2: which blocks a head keeps).  Same tiles, lists and orientation as
// fwd_kernel.hip (a 128-row query tile that spans several mask rows, scores computed transposed so
// that a lane owns one query), with a different division of labour:
//
//   * a wavefront owns 64 query rows (two 32-row blocks), so every K / V fragment it fetches from
//     LDS feeds two MFMAs; a workgroup is two wavefronts and a compute unit runs two workgroups,
//     one wavefront per SIMD with all 512 registers: the output accumulators and the Q fragments
//     live in the accumulation registers and are touched by MFMAs only;
//   * the loop is software pipelined by one step: while the matrix pipe computes the scores of
//     step i+1 and then P(i) V(i), the vector pipe turns the scores of step i into probabilities
//     and finds the maximum of step i+1.  Matrix and vector work of ONE instruction stream overlap
//     on this hardware, those of two wavefronts on a SIMD hardly do, so the interleave is written
//     out by hand, one MFMA per slot, and fenced so that the compiler keeps it;
//   * the running maximum is only moved when a new score exceeds it by more than 2^kTau: the
//     accumulators are then rescaled in a rarely taken branch instead of in every step.
//
// The MFMAs are inline assembly so that each one's accumulator can be placed in the register file
// it belongs to.  The compiler does not see through them, so the wait states the hardware needs
// between an MFMA and a vector instruction that reads its result are provided by distance (the
// fences keep at least a dozen instructions in between) or by explicit s_nop.
#include <hip/hip_runtime.h>

#include <atomic>
#include <type_traits>
#include <utility>

#include "config.h"
#include "device_util.h"
#include "kernels.h"

namespace s2 {

namespace {

constexpr float kNegInf = -__builtin_inff();
constexpr float kTau = 8.0f;  // log2 units a score may exceed the reference maximum by

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

#define S2_FENCE() __builtin_amdgcn_sched_barrier(0)
#define S2_INLINE __attribute__((always_inline))

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index is a
// compile-time constant in the body, whatever the optimiser's unrolling limits are
template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

// d (vector registers) = a x b, b in accumulation registers
__device__ __forceinline__ void mfma_vz(f32x16& d, u32x4 a, u32x4 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "a"(b));
}
// d (vector registers) += a x b, b in accumulation registers
__device__ __forceinline__ void mfma_v(f32x16& d, u32x4 a, u32x4 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "a"(b));
}
// d (accumulation registers) += a x b
__device__ __forceinline__ void mfma_a(f32x16& d, u32x4 a, u32x4 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b));
}

template <int D>
struct Fwd64Smem {
  uint16_t k[2][DmaTile<D, 64, 2>::kElems];
  uint16_t v[2][DmaTile<D, 64, 2>::kElems];
};

template <int D, bool DENSE>
__global__ __launch_bounds__(128) void fwd64_kernel(const AttnParams p) {
  typedef DmaTile<D, 64, 2> Tile;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  Fwd64Smem<D>& sm = *reinterpret_cast<Fwd64Smem<D>*>(smem_raw);
  constexpr int BM = 128, MW = 64, CH = 64;
  constexpr int KK = D / 16, DT = D / 32;
  constexpr int NQK = 4 * KK;       // MFMAs of the score contraction per step
  constexpr int NPV = 8 * DT;       // MFMAs of the second contraction per step
  constexpr int NG = Tile::kGroups;  // groups of direct loads per tile and wavefront
  static_assert(D == 128, "the slot schedule below is laid out for head_dim 128");

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int T = p.fwd_tiles.tiles_per_head;    // tiles of the whole sequence (indexes the lists)
  const int T_run = p.q_rows / BM;             // tiles this launch computes
  int bh, rank;
  if (!map_workgroup(blockIdx.x, p.batch * p.heads, T_run, bh, rank)) return;
  const int b = bh / p.heads, h = bh - b * p.heads;
  const bool whole = p.q_row0 == 0 && T_run == T;
  const int tile = (DENSE || !whole) ? p.q_row0 / BM + (T_run - 1 - rank) : p.fwd_tiles.order[h * T + rank];
  const int N = p.seqlen;
  const int S = DENSE ? CH : p.block_size;  // 64 or 128
  const int cpb_sh = S == 128 ? 1 : 0, cpb_m = (1 << cpb_sh) - 1;
  const int qw0 = tile * BM + wave * MW;    // first query row of this wavefront (sequence position)
  const int ql0 = qw0 - p.q_row0;           // the same as a row of q / o / lse
  const int my_member = (qw0 / S) - tile * (BM / S);

  const int64_t q_off = b * p.q_sb + h * p.q_sh;
  const int64_t kv_off = b * p.kv_sb + h * p.kv_sh;
  // minus the bias the grouped direct loads put into their lane offsets
  const uint16_t* kb = p.k + kv_off - Tile::kBias / 2;
  const uint16_t* vb = p.v + kv_off - Tile::kBias / 2;

  // Q^T fragments, loaded straight into accumulation registers (B operands of the score MFMAs)
  u32x4 qf[2][KK];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb)
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const uint16_t* src = p.q + q_off + (int64_t)(ql0 + 32 * qb + l32) * p.q_st + 16 * kk + 8 * half;
      asm volatile("global_load_dwordx4 %0, %1, off" : "=a"(qf[qb][kk]) : "v"(src));
    }

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

  f32x16 acc[2][DT];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) acc[qb][dt] = f32x16{};
  float m_ref[2] = {kNegInf, kNegInf};  // reference maximum (raw scores) per query block
  float mc[2] = {kNegInf, kNegInf};     // the same times scale * log2(e), 0 while nothing was seen
  float l_run[2] = {0.f, 0.f};          // sum of the probabilities over my half's key rows
  const float c = p.scale_log2e;
  const typename Tile::BlockPlan plan = Tile::block_plan(p.kv_st, wave, lane);
  const int trb = Tile::tr_base(lane);

  f32x16 s[2][2][2];  // scores [parity of the step][query block][32-key half]

  // ------------------------------------------------------------------ pieces of a step
  // MFMA n of the score contraction of a step: kk = n / 4, key half = (n / 2) % 2, query block = n % 2
  auto qk_mfma = [&](int n, f32x16 (&sn)[2][2], const u32x4 (&kfr)[4]) S2_INLINE {
    const int kk = n >> 2, kt = (n >> 1) & 1, qb = n & 1;
    if (kk == 0)
      mfma_vz(sn[qb][kt], kfr[(n >> 1) & 3], qf[qb][kk]);
    else
      mfma_v(sn[qb][kt], kfr[(n >> 1) & 3], qf[qb][kk]);
  };
  // fragment f = 0..2*KK-1 of K (kk = f / 2, key half = f % 2), into its slot of a ring of four
  auto k_load = [&](int f, const uint16_t* ks, u32x4 (&kfr)[4]) S2_INLINE {
    kfr[f & 3] = __builtin_bit_cast(u32x4, Tile::row_frag(ks, f & 1, f >> 1, l32, half));
  };
  // MFMA n of the second contraction: group g = n / (2*DT) (key half g / 2, 16-key slab g % 2),
  // feature tile (n / 2) % DT, query block n % 2
  auto pv_mfma = [&](int n, const u32x4 (&vfr)[4], const u32x4 (&pb)[4][2]) S2_INLINE {
    const int g = n / (2 * DT), dt = (n >> 1) % DT, qb = n & 1;
    mfma_a(acc[qb][dt], vfr[(n >> 1) & 3], pb[g][qb]);
  };
  // fragment f = 0..4*DT-1 of V^T (group f / DT, feature tile f % DT)
  auto v_load = [&](int f, const uint16_t* vs, u32x4 (&vfr)[4]) S2_INLINE {
    vfr[f & 3] = __builtin_bit_cast(u32x4, Tile::tr_frag(vs, f % DT, f / DT, trb));
  };
  // The probabilities of a step are made in three stages - scale and shift, exponential, sum and
  // pack - that a slot applies to different elements, so that no instruction waits for the one
  // before it.  Elements are numbered in the order the second contraction uses them:
  // e = 16 * g + 8 * qb + i is score register 8 * (g % 2) + i of key half g / 2 of query block qb.
  // Stages 1 and 2 work in place, in the score registers.
  auto p_stage1 = [&](int e0, int e1, f32x16 (&sc)[2][2]) S2_INLINE {
#pragma unroll
    for (int e = max(e0, 0); e < min(e1, 64); ++e) {
      const int g = e >> 4, qb = (e >> 3) & 1, r = 8 * (g & 1) + (e & 7);
      sc[qb][g >> 1][r] = __builtin_fmaf(sc[qb][g >> 1][r], c, -mc[qb]);
    }
  };
  auto p_stage2 = [&](int e0, int e1, f32x16 (&sc)[2][2]) S2_INLINE {
#pragma unroll
    for (int e = max(e0, 0); e < min(e1, 64); ++e) {
      const int g = e >> 4, qb = (e >> 3) & 1, r = 8 * (g & 1) + (e & 7);
      sc[qb][g >> 1][r] = fast_exp2(sc[qb][g >> 1][r]);
    }
  };
  auto p_stage3 = [&](int e0, int e1, f32x16 (&sc)[2][2], u32x4 (&pb)[4][2]) S2_INLINE {
#pragma unroll
    for (int e = max(e0, 0); e < min(e1, 64); ++e) {
      const int g = e >> 4, qb = (e >> 3) & 1, i = e & 7, r = 8 * (g & 1) + i;
      // the sum takes the unrounded probabilities: LSE is held to 1e-3, which a sum of bf16 values
      // cannot promise for rows with one or two keys
      l_run[qb] += sc[qb][g >> 1][r];
      if (i & 1) {
        bf16x2 w;
        w[0] = (__bf16)sc[qb][g >> 1][r - 1];
        w[1] = (__bf16)sc[qb][g >> 1][r];
        pb[g][qb][i >> 1] = __builtin_bit_cast(uint32_t, w);
      }
    }
  };
  // element index reached after slot sl: five elements every four slots
  auto p_upto = [](int sl) S2_INLINE { return (5 * (sl + 1)) / 4; };
  auto mask_diag = [&](f32x16 (&sn)[2][2], int kv0) S2_INLINE {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const int qpos = qw0 + 32 * qb + l32;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kv0 + 32 * kt + 8 * (r >> 2) + 4 * half + (r & 3);
          if (key > qpos) sn[qb][kt][r] = kNegInf;
        }
    }
  };
  // running maxima of score registers r0 .. r1-1 (of 32 per query block) of both query blocks
  auto max_part = [&](int r0, int r1, const f32x16 (&sn)[2][2], float (&mx)[2]) S2_INLINE {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int r = r0; r < r1; r += 2)
        mx[qb] = fmaxf(fmaxf(mx[qb], sn[qb][r >> 4][r & 15]), sn[qb][r >> 4][(r + 1) & 15]);
  };
  // moves the reference maximum where the new scores exceed it by more than 2^kTau (always for the
  // first step, when it is -inf) and rescales what has been accumulated so far
  auto update_ref = [&](float (&mx)[2]) S2_INLINE {
    bool need = false;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      mx[qb] = max_halves(mx[qb]);
      need = need || (__builtin_fmaf(mx[qb], c, -mc[qb]) > kTau);
    }
    if (__any(need)) {
      // the accumulators were last written by MFMAs: wait states before vector instructions read them
      asm volatile("s_nop 7\n\ts_nop 7"
                   : "+a"(acc[0][0]), "+a"(acc[0][1]), "+a"(acc[0][2]), "+a"(acc[0][3]), "+a"(acc[1][0]),
                     "+a"(acc[1][1]), "+a"(acc[1][2]), "+a"(acc[1][3]));
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        const float m_new = fmaxf(m_ref[qb], mx[qb]);
        const float m_use = (m_new == kNegInf) ? 0.f : m_new;
        const float alpha = fast_exp2((m_ref[qb] - m_use) * c);
        l_run[qb] *= alpha;
        // one accumulator at a time, so that only 16 vector registers are needed to pass them through
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          S2_FENCE();
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[qb][dt][r] *= alpha;
          S2_FENCE();
        }
        m_ref[qb] = m_new;
        mc[qb] = m_use * c;
      }
      // ... and before an MFMA reads what vector instructions wrote
      asm volatile("s_nop 3"
                   : "+a"(acc[0][0]), "+a"(acc[0][1]), "+a"(acc[0][2]), "+a"(acc[0][3]), "+a"(acc[1][0]),
                     "+a"(acc[1][1]), "+a"(acc[1][2]), "+a"(acc[1][3]));
    }
  };

  // ------------------------------------------------------------------ prologue
  // A step this wavefront has nothing to compute in (its mask row drops the block, or every key
  // lies after its queries) still runs through the same instruction stream - there is one code
  // path - with its scores kept out of the maximum and its probabilities forced to zero.
  int kv0_c, kv0_n, kv0_nn;
  bool act_c, act_n, act_nn;
  chunk_at(0, kv0_c, act_c);
  chunk_at(1, kv0_n, act_n);
  static_for<NG>([&](auto gc) S2_INLINE {
    constexpr int g = decltype(gc)::value;
    Tile::template issue_group<g>(plan, kb + (int64_t)kv0_c * p.kv_st, sm.k[0], wave);
    Tile::template issue_group<g>(plan, vb + (int64_t)kv0_c * p.kv_st, sm.v[0], wave);
    Tile::template issue_group<g>(plan, kb + (int64_t)kv0_n * p.kv_st, sm.k[1], wave);
  });
  wait_all_loads();  // also the Q fragments
  __syncthreads();
  // maximum of the scores in sn (masked on the diagonal), then the reference maximum
  auto finish_scores = [&](f32x16 (&sn)[2][2], int kv0, bool act, bool masked, float (&mx)[2]) S2_INLINE {
    if (masked) {
      // the scores were last written by MFMAs: wait states before vector instructions touch them
      asm volatile("s_nop 7\n\ts_nop 3" : "+v"(sn[0][0]), "+v"(sn[0][1]), "+v"(sn[1][0]), "+v"(sn[1][1]));
      mask_diag(sn, kv0);
      mx[0] = kNegInf;
      mx[1] = kNegInf;
      max_part(0, 32, sn, mx);
    }
    if (!act) {
      mx[0] = kNegInf;
      mx[1] = kNegInf;
    }
    update_ref(mx);
  };
  {
    u32x4 kfr[4];
#pragma unroll
    for (int f = 0; f < 3; ++f) k_load(f, sm.k[0], kfr);
    static_for<NQK>([&](auto nc) S2_INLINE {
      constexpr int n = decltype(nc)::value;
      if ((n & 1) == 0 && (n >> 1) + 3 < 2 * KK) k_load((n >> 1) + 3, sm.k[0], kfr);
      qk_mfma(n, s[0], kfr);
      S2_FENCE();
    });
    float mx[2];
    finish_scores(s[0], kv0_c, act_c, true, mx);  // `true`: the first step may be the diagonal, and the fence is needed anyway
  }
  __syncthreads();  // both wavefronts are done with K(0) before step 0 loads K(2) over it

  // ------------------------------------------------------------------ one step
  // On entry: K(it+1) and V(it) are in LDS, sc holds the scores of step it and the reference
  // maximum already covers them.
  auto step = [&](int it, f32x16 (&sc)[2][2], f32x16 (&sn)[2][2]) S2_INLINE {
    const int par = it & 1;
    chunk_at(it + 2, kv0_nn, act_nn);
    const uint16_t* kg = kb + (int64_t)kv0_nn * p.kv_st;  // K(it+2) -> the stage K(it) was in
    const uint16_t* vg = vb + (int64_t)kv0_n * p.kv_st;   // V(it+1) -> the stage V(it-1) was in
    const uint16_t* ks = sm.k[par ^ 1];
    const uint16_t* vs = sm.v[par];
    uint16_t* kn = sm.k[par];
    uint16_t* vn = sm.v[par ^ 1];
    // group d of this step's direct loads: 0..NG-1 for K, NG..2*NG-1 for V
    auto dma = [&](auto dc) S2_INLINE {
      constexpr int d = decltype(dc)::value;
      if constexpr (d < NG)
        Tile::template issue_group<d>(plan, kg, kn, wave);
      else if constexpr (d < 2 * NG)
        Tile::template issue_group<d - NG>(plan, vg, vn, wave);
    };
    const bool mask_next = kv0_n + CH - 1 > qw0;
    // a step that is not mine: every probability exp2(s*c - inf) = 0
    const float mc_keep[2] = {mc[0], mc[1]};
    if (!act_c) {
      mc[0] = __builtin_inff();
      mc[1] = __builtin_inff();
    }
    u32x4 kfr[4], vfr[4], pb[4][2];
    float mx[2] = {kNegInf, kNegInf};
#pragma unroll
    for (int f = 0; f < 3; ++f) k_load(f, ks, kfr);
    S2_FENCE();
    // NQK + NPV slots, one MFMA each
    static_for<NQK + NPV>([&](auto slc) S2_INLINE {
      constexpr int sl = decltype(slc)::value;
      // fragments three MFMA pairs ahead
#if !defined(S2_EXP) || S2_EXP != 4
      if constexpr (sl < NQK && (sl & 1) == 0 && (sl >> 1) + 3 < 2 * KK) k_load((sl >> 1) + 3, ks, kfr);
      if constexpr (sl >= NQK - 6 && (sl & 1) == 0 && ((sl - (NQK - 6)) >> 1) < 4 * DT)
        v_load((sl - (NQK - 6)) >> 1, vs, vfr);
#else
      if constexpr (sl == 0) { v_load(0, vs, vfr); v_load(1, vs, vfr); v_load(2, vs, vfr); v_load(3, vs, vfr); k_load(3, ks, kfr); }
#endif
      if constexpr (sl < NQK)
        qk_mfma(sl, sn, kfr);
      else
        pv_mfma(sl - NQK, vfr, pb);
      // probabilities of this step: three elements every two slots
#if !defined(S2_EXP) || S2_EXP != 5
      // probabilities of this step, five elements every four slots, each stage one slot behind
      // the one before it (elements 16 g .. 16 g + 15 are packed by slot 13 g + 14, their MFMAs
      // start at slot 32 + 8 g)
      p_stage1(p_upto(sl - 1), p_upto(sl), sc);
      p_stage2(p_upto(sl - 2), p_upto(sl - 1), sc);
      p_stage3(p_upto(sl - 3), p_upto(sl - 2), sc, pb);
      // maximum of the next step's scores, once its MFMAs are a dozen instructions back
      if constexpr (sl >= 46 && sl < 62) max_part(2 * (sl - 46), 2 * (sl - 46) + 2, sn, mx);
#endif
      // Nothing to execute: ties the running sums and maxima to this slot, or the optimiser
      // collects their additions and comparisons after the last MFMA, out of its shadow.
      asm volatile("" : "+v"(l_run[0]), "+v"(l_run[1]), "+v"(mx[0]), "+v"(mx[1]));
#if !defined(S2_EXP) || S2_EXP < 2
      if constexpr (sl % 8 == 1 && sl / 8 < 2 * NG) dma(std::integral_constant<int, sl / 8>{});
#endif
      S2_FENCE();
    });
    mc[0] = mc_keep[0];
    mc[1] = mc_keep[1];
    finish_scores(sn, kv0_n, act_n, mask_next, mx);
    if (!DENSE) (void)list.get(min(it + 1, total - 1) >> cpb_sh, lane);  // keeps the entry window moving
    kv0_c = kv0_n;
    act_c = act_n;
    kv0_n = kv0_nn;
    act_n = act_nn;
#if !defined(S2_EXP) || S2_EXP < 3
    wait_all_loads();
    __syncthreads();
#endif
  };

  int it = 0;
  for (; it + 1 < total; it += 2) {
    step(it, s[0], s[1]);
    step(it + 1, s[1], s[0]);
  }
  if (it < total) step(it, s[0], s[1]);

  // ------------------------------------------------------------------ epilogue
  asm volatile("s_nop 7\n\ts_nop 7"
               : "+a"(acc[0][0]), "+a"(acc[0][1]), "+a"(acc[0][2]), "+a"(acc[0][3]), "+a"(acc[1][0]),
                 "+a"(acc[1][1]), "+a"(acc[1][2]), "+a"(acc[1][3]));
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const float l_tot = sum_halves(l_run[qb]);
    const float inv = 1.0f / l_tot;
    const int qrow = ql0 + 32 * qb + l32;
    uint16_t* orow = p.o + q_off + (int64_t)qrow * p.q_st;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (__bf16)(acc[qb][dt][4 * g + e] * inv);
        *reinterpret_cast<bf16x4*>(orow + 32 * dt + 8 * g + 4 * half) = w;
      }
      S2_FENCE();
    }
    if (half == 0) p.lse[((int64_t)b * p.heads + h) * p.q_rows + qrow] = m_ref[qb] * p.scale + __logf(l_tot);
  }
}

// A kernel's dynamic LDS limit is a per-device attribute: remember, per device, that it is set.
constexpr int kMaxDevices = 64;
std::atomic<unsigned char> g_smem_set[2][kMaxDevices];

template <bool DENSE>
hipError_t launch_one(const AttnParams& p, hipStream_t stream) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < kMaxDevices;
  if (!tracked || !g_smem_set[DENSE][dev].load(std::memory_order_acquire)) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&fwd64_kernel<128, DENSE>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(Fwd64Smem<128>));
    if (e != hipSuccess) return e;
    if (tracked) g_smem_set[DENSE][dev].store(1, std::memory_order_release);
  }
  const int grid = grid_for(p.batch * p.heads, p.q_rows / 128);
  hipLaunchKernelGGL((fwd64_kernel<128, DENSE>), dim3(grid), dim3(128), sizeof(Fwd64Smem<128>), stream, p);
  return hipGetLastError();
}

}  // namespace

bool fwd64_applies(const AttnParams& p, bool dense) {
  return p.head_dim == 128 && !p.cu_seqlens && (dense || p.block_size >= 64) && p.q_rows % 128 == 0 &&
         p.q_row0 % 128 == 0;
}

hipError_t launch_fwd64(const AttnParams& p, bool dense, hipStream_t stream) {
  return dense ? launch_one<true>(p, stream) : launch_one<false>(p, stream);
}

}  // namespace s2
