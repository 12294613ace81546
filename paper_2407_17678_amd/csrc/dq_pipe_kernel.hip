// dQ kernel for head_dim 128 and mask blocks of 64 or 128 tokens: the fast path of the
// row-stationary half of the backward pass (the gradient of the forward of section 3.2).  Same
// tiles, lists, staging and orientation as dq_kernel in bwd_kernel.hip - a workgroup owns 128 query
// rows, a wavefront 32 of them, and walks the 64-key chunks of the KV blocks its mask rows keep,
// recomputing P and forming dS = P * (dP - delta), dQ += scale * dS K; it also computes
// delta = rowsum(dO * O) and leaves it, with LSE in base-2 units, in the workspace for the dK/dV
// kernel - with a hand-scheduled inner loop:
//
//   * it runs in half chunks of 32 keys, 24 slots of one MFMA each, skewed by one half: S and dP of
//     the next half are computed around the dQ MFMAs of this one, with this half's dS arithmetic
//     under the former and the next half's exponentials under the latter;
//   * the order is written out, one MFMA per slot with its share of the vector work, LDS reads and
//     direct loads, and fenced so that the compiler keeps it (see sched_util.h for the measurements
//     behind this); the A operands pass through a ring of registers requested five MFMAs ahead;
//   * the direct loads of a tile are issued four to a write of M0.
#include <hip/hip_runtime.h>

#include <atomic>

#include "config.h"
#include "device_util.h"
#include "kernels.h"
#include "sched_util.h"

namespace s2 {

namespace {

constexpr float kNegInf = -__builtin_inff();
constexpr float kLog2e = 1.4426950408889634f;

template <int D>
struct DqPipeSmem {
  uint16_t k[2][DmaTile<D, 64, 4>::kElems];
  uint16_t v[2][DmaTile<D, 64, 4>::kElems];
};

// VARLEN: a packed batch of sequences of different lengths.  A workgroup finds its sequence's rows in
// cu_seqlens and treats them as a sequence of its own; this kernel computes the whole 128-row tiles of
// each sequence (all their keys exist), a partial last tile is left to dq_kernel.
template <int D, bool DENSE, bool VARLEN = false>
__global__ __launch_bounds__(kThreads, 2) void dq_pipe_kernel(const AttnParams p) {
  typedef DmaTile<D, 64, 4> Tile;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  DqPipeSmem<D>& sm = *reinterpret_cast<DqPipeSmem<D>*>(smem_raw);
  constexpr int BM = kBwdBM, MW = 32, CH = 64;
  constexpr int KK = D / 16, DT = D / 32;
  constexpr int NG = Tile::kGroups;
  constexpr int RB = Tile::kStride * 2;  // bytes per tile row
  constexpr int kSlots = 3 * KK;         // MFMAs (and fragments) per half step
  constexpr int kLead = 5, kRing = kLead + 1;  // (3 to 7 measure the same)
  static_assert(D == 128, "the slot schedule below is laid out for head_dim 128");
  static_assert(KK == 8 && DT == 4, "24 slots per half chunk");

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int T = p.q_tiles.tiles_per_head;
  const int T_run = VARLEN ? p.q_rows / BM : T;  // packed batch: whole tiles of the longest length allowed
  int bh, rank;
  if (!map_workgroup(blockIdx.x, p.batch * p.heads, T_run, bh, rank)) return;
  const int b = bh / p.heads, h = bh - b * p.heads;
  int tile = DENSE ? (T - 1 - rank) : VARLEN ? 0 : p.q_tiles.order[h * T + rank];
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
  const int qw0 = tile * BM + wave * MW;  // first query row of this wavefront
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
    ent_lo = p.q_tiles.ptr[h * T + tile];
    n_ent = p.q_tiles.ptr[h * T + tile + 1] - ent_lo;
  }
  const int total = n_ent << cpb_sh;  // chunks
  if (total <= 0) return;
  EntryList list;
  if (!DENSE) list.init(p.q_tiles.ent + ent_lo, n_ent, lane);
  // chunk j of the tile's list (clamped to the last one): its first key row, and whether this
  // wavefront's mask row keeps it
  auto chunk_at = [&](int j, int& kv0, bool& keep) S2_INLINE {
    const bool inside = j < total;
    j = min(j, total - 1);
    if (DENSE) {
      kv0 = j * CH;
      keep = inside;
    } else {
      const int e = list.peek(j >> cpb_sh);
      kv0 = (e >> 16) * S + (j & cpb_m) * CH;
      keep = inside && ((e >> my_member) & 1);
    }
  };

  const typename Tile::BlockPlan plan = Tile::block_plan(p.kv_st, wave, lane);
  auto issue_chunk = [&](int kv0, int stage) S2_INLINE {
    const uint16_t* kg = kb + (int64_t)kv0 * p.kv_st;
    const uint16_t* vg = vb + (int64_t)kv0 * p.kv_st;
    static_for<NG>([&](auto gc) S2_INLINE {
      constexpr int g = decltype(gc)::value;
      Tile::template issue_group<g>(plan, kg, sm.k[stage], wave);
      Tile::template issue_group<g>(plan, vg, sm.v[stage], wave);
    });
  };
  int kv0_c, kv0_n;
  bool keep_c, keep_n;
  chunk_at(0, kv0_c, keep_c);
  chunk_at(1, kv0_n, keep_n);
  issue_chunk(kv0_c, 0);

  // Q^T and dO^T fragments (B operands), lane = query; delta = rowsum(dO * O) of my query from the
  // dO fragments (my half of the row's features, then the two halves added), written out with LSE
  // in base-2 units for the dK/dV kernel, which runs after this one
  bf16x8 qf[KK], gf[KK];
  float part = 0.f;
  const int my_row = qw0 + l32;
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    const int64_t o = q_off + (int64_t)my_row * p.q_st + 16 * kk + 8 * half;
    qf[kk] = *reinterpret_cast<const bf16x8*>(p.q + o);
    gf[kk] = *reinterpret_cast<const bf16x8*>(p.d_o + o);
    const bf16x8 of = *reinterpret_cast<const bf16x8*>(p.o + o);
#pragma unroll
    for (int e = 0; e < 8; ++e) part = __builtin_fmaf((float)gf[kk][e], (float)of[e], part);
  }
  const float delta_l = sum_halves(part);
  const int64_t stat_row = VARLEN ? (int64_t)h * p.seqlen + row_base + my_row  // [heads, rows of the tensors]
                                  : ((int64_t)b * p.heads + h) * N + my_row;
  const float lse_l = p.lse[stat_row] * kLog2e;
  if (half == 0) {
    p.delta[stat_row] = delta_l;
    p.lse2[stat_row] = lse_l;
  }

  f32x16 acc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) acc[dt] = f32x16{};
  const float c = p.scale_log2e;
  const int trb = Tile::tr_base(lane);

  // Scores of a 32-key half: register r is key 8 * (r / 4) + 4 * half + r % 4 of the half, lane % 32
  // the query.  sc holds S, then P in place; dp holds dP, then dS in place.
  f32x16 sc[2], dp;  // sc[parity of the half]
  u32x4 dsb[2];      // dS of this half as B operands [16-key slab]

  // a half whose keys all lie after my queries, or that my mask row drops, gets lse = +inf: P = dS = 0
  auto half_state = [&](int kv0, bool keep, int kt, bool& act, bool& diag) S2_INLINE {
    const int kbase = kv0 + 32 * kt;
    act = keep && kbase <= qw0 + MW - 1;
    diag = kbase + 31 > qw0;  // some key lies after my first query: the causal mask applies
  };
  auto mask_diag = [&](f32x16& s2, int kbase) S2_INLINE {
    const int qpos = qw0 + l32;
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (kbase + 8 * (r >> 2) + 4 * half + (r & 3) > qpos) s2[r] = kNegInf;
  };

  bool act_cur = false;  // whether the half whose P is in sc[parity] is mine

  // ------------------------------------------------------------------ prologue
  wait_all_loads();
  __syncthreads();
  // S, dP and P of the first half, one after the other
  {
    bool act, diag;
    half_state(kv0_c, keep_c, 0, act, diag);
    const uint32_t k_row = lds_addr(sm.k[0]) + l32 * RB + 16 * half;
    const uint32_t v_row = lds_addr(sm.v[0]) + l32 * RB + 16 * half;
    sc[0] = f32x16{};
    dp = f32x16{};
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      sc[0] = mfma32(__builtin_bit_cast(bf16x8, lds_read16(k_row, 32 * kk)), qf[kk], sc[0]);
      dp = mfma32(__builtin_bit_cast(bf16x8, lds_read16(v_row, 32 * kk)), gf[kk], dp);
    }
    act_cur = act;
    if (diag) mask_diag(sc[0], kv0_c);
    const float l0 = act ? lse_l : __builtin_inff();
#pragma unroll
    for (int r = 0; r < 16; ++r) sc[0][r] = fast_exp2(__builtin_fmaf(sc[0][r], c, -l0));
  }

  // ------------------------------------------------------------------ one half step
  // On entry: sc[PAR] holds P of this half (half KT of the chunk in stage stc), dp its dP; K / V of
  // the next half's chunk are in stage stn (the same stage for KT = 0).
  auto half_step = [&](auto par_c, auto kt_c, int stc, int stn, int kvn, bool keep_nx) S2_INLINE {
    constexpr int PAR = decltype(par_c)::value, KT = decltype(kt_c)::value;
    constexpr int KTN = KT ^ 1;  // which half of its chunk the next half is
    bool act_n, diag_n;
    half_state(kvn, keep_nx, KTN, act_n, diag_n);
    // Neither this half nor the next is mine (mask row drops them, or their keys lie after my
    // queries): nothing to compute; the next half's P and dP are zero.  One of the two being mine
    // runs the whole stream (the other's probabilities are zero through lse = +inf).
    const bool act_this = act_cur;
    act_cur = act_n;
    if (!act_this && !act_n) {
      sc[PAR ^ 1] = f32x16{};
      dp = f32x16{};
      return;
    }
    uint32_t k_row = lds_addr(sm.k[stn]) + l32 * RB + 16 * half + 32 * KTN * RB;
    uint32_t v_row = lds_addr(sm.v[stn]) + l32 * RB + 16 * half + 32 * KTN * RB;
    uint32_t k_tr = lds_addr(sm.k[stc]) + 2 * trb + 32 * KT * RB;
    asm volatile("" : "+v"(k_row), "+v"(v_row), "+v"(k_tr));
    bf16x8 fr[kRing];
    // fragment f of the half step, in the order the MFMAs use them: 8 row fragments of the next
    // half's K, 8 transposed fragments of this half's K (16-key slab, feature tile), 8 row fragments
    // of the next half's V
    auto frag_load = [&](auto fc) S2_INLINE {
      constexpr int f = decltype(fc)::value;
      if constexpr (f < 8)
        fr[f % kRing] = __builtin_bit_cast(bf16x8, lds_read16(k_row, 32 * f));
      else if constexpr (f < 16)
        fr[f % kRing] = __builtin_bit_cast(bf16x8, lds_read_tr(k_tr, 16 * ((f - 8) >> 2) * RB + 64 * ((f - 8) & 3), RB));
      else
        fr[f % kRing] = __builtin_bit_cast(bf16x8, lds_read16(v_row, 32 * (f - 16)));
    };
    static_for<kLead>([&](auto fc) S2_INLINE { frag_load(fc); });
    const float ln = act_n ? lse_l : __builtin_inff();
    S2_FENCE();
    static_for<kSlots>([&](auto nc) S2_INLINE {
      constexpr int n = decltype(nc)::value;
      if constexpr (n + kLead < kSlots) frag_load(std::integral_constant<int, n + kLead>{});
      // the MFMA of the slot
      if constexpr (n < 8)  // S of the next half
        sc[PAR ^ 1] = mfma32(fr[n % kRing], qf[n], n == 0 ? f32x16{} : sc[PAR ^ 1]);
      else if constexpr (n < 16)  // dQ of this half: slab (n - 8) / 4, feature tile (n - 8) % 4
        acc[(n - 8) & 3] = mfma32(fr[n % kRing], __builtin_bit_cast(bf16x8, dsb[(n - 8) >> 2]), acc[(n - 8) & 3]);
      else  // dP of the next half
        dp = mfma32(fr[n % kRing], gf[n - 16], n == 16 ? f32x16{} : dp);
      // dS = P * (dP - delta) of this half under the S MFMAs: registers 2n, 2n+1 in slot n < 8;
      // slab 0 packed in slot 4, slab 1 in slot 8
      if constexpr (n < 8) {
#pragma unroll
        for (int r = 2 * n; r < 2 * n + 2; ++r) dp[r] = sc[PAR][r] * (dp[r] - delta_l);
      }
      if constexpr (n == 4 || n == 8) {
        constexpr int u = n == 4 ? 0 : 1;
#pragma unroll
        for (int i = 0; i < 4; ++i) dsb[u][i] = pack2(dp[8 * u + 2 * i], dp[8 * u + 2 * i + 1]);
      }
      // P = exp2(S * c - lse) of the next half under the dQ and dP MFMAs
      if constexpr (n == 9) {
        if (diag_n) mask_diag(sc[PAR ^ 1], kvn + 32 * KTN);
      }
      if constexpr (n >= 10 && n < 18) {
        constexpr int r = 2 * (n - 10);
        sc[PAR ^ 1][r] = __builtin_fmaf(sc[PAR ^ 1][r], c, -ln);
        sc[PAR ^ 1][r + 1] = __builtin_fmaf(sc[PAR ^ 1][r + 1], c, -ln);
      }
      if constexpr (n >= 11 && n < 19) {
        constexpr int r = 2 * (n - 11);
        sc[PAR ^ 1][r] = fast_exp2(sc[PAR ^ 1][r]);
        sc[PAR ^ 1][r + 1] = fast_exp2(sc[PAR ^ 1][r + 1]);
      }
      // Nothing to execute: ties the probabilities to this slot.  Their first use is in the next
      // half step, and the optimiser would otherwise collect the arithmetic there, after the last
      // MFMA of this one and out of its shadow.
      if constexpr (n >= 10 && n < 19) asm volatile("" : "+v"(sc[PAR ^ 1]));
      S2_FENCE();
    });
  };

  // ------------------------------------------------------------------ the loop: one chunk per trip
  // trip ch: half steps (ch, 0) and (ch, 1); chunk ch + 1 is requested at the start of the trip
  // into the other stage (free since the barrier that ended the last trip) and must have landed
  // when the second half step reads its K and V rows
  for (int ch = 0; ch < total; ++ch) {
    const int st = ch & 1;
    issue_chunk(kv0_n, st ^ 1);  // past the end of the list: the last chunk once more
    half_step(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, st, st, kv0_c, keep_c);
    wait_all_loads();
    __syncthreads();
    half_step(std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{}, st, st ^ 1, kv0_n, keep_n);
    if (!DENSE) (void)list.get(min(ch + 1, total - 1) >> cpb_sh, lane);  // keeps the entry window moving
    kv0_c = kv0_n;
    keep_c = keep_n;
    chunk_at(ch + 2, kv0_n, keep_n);
    __syncthreads();  // every wavefront is done with chunk ch before the next trip loads over it
  }

  // ------------------------------------------------------------------ epilogue
  // dQ = scale * acc goes out through LDS (free since the loop's last barrier; each wavefront uses a
  // region of its own, so no barrier): a lane holds its row's features four at a time, and storing
  // them from there would touch 32 rows per instruction with 16 bytes each; read back 16 bytes per
  // lane, row after row, an instruction stores four whole rows.
  constexpr int RS = D + 8;  // staging row stride (elements)
  uint16_t* stage = sm.k[0] + wave * MW * RS;
  static_assert(4 * MW * RS <= 2 * Tile::kElems, "the staging rows fit the K stages");
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 w;
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = (__bf16)(acc[dt][4 * g + e] * p.scale);
      *reinterpret_cast<bf16x4*>(stage + l32 * RS + 32 * dt + 8 * g + 4 * half) = w;
    }
  uint16_t* obase = p.dq + q_off + (int64_t)qw0 * p.q_st;
#pragma unroll
  for (int i = 0; i < MW / 4; ++i) {
    const int r = 4 * i + (lane >> 4), piece = lane & 15;
    const u32x4 x = *reinterpret_cast<const u32x4*>(stage + r * RS + 8 * piece);
    *reinterpret_cast<u32x4*>(obase + (int64_t)r * p.q_st + 8 * piece) = x;
  }
}

// A kernel's dynamic LDS limit is a per-device attribute: remember, per device, that it is set.
constexpr int kMaxDevices = 64;
std::atomic<unsigned char> g_smem_set[3][kMaxDevices];

template <bool DENSE, bool VARLEN>
hipError_t launch_one(const AttnParams& p, hipStream_t stream) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < kMaxDevices;
  constexpr int which = VARLEN ? 2 : DENSE;
  if (!tracked || !g_smem_set[which][dev].load(std::memory_order_acquire)) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dq_pipe_kernel<128, DENSE, VARLEN>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(DqPipeSmem<128>));
    if (e != hipSuccess) return e;
    if (tracked) g_smem_set[which][dev].store(1, std::memory_order_release);
  }
  const int grid = grid_for(p.batch * p.heads, VARLEN ? p.q_rows / kBwdBM : p.q_tiles.tiles_per_head);
  hipLaunchKernelGGL((dq_pipe_kernel<128, DENSE, VARLEN>), dim3(grid), dim3(kThreads), sizeof(DqPipeSmem<128>), stream, p);
  return hipGetLastError();
}

}  // namespace

bool dq_pipe_applies(const AttnParams& p, bool dense) {
  // whole 128-row tiles only: every wavefront of a workgroup owns 32 existing query rows
  if (p.cu_seqlens)  // packed batch: the whole tiles of each sequence
    return !dense && p.head_dim == 128 && p.block_size >= 64 && p.q_rows >= kBwdBM;
  return p.head_dim == 128 && (dense || p.block_size >= 64) && p.seqlen % kBwdBM == 0;
}

hipError_t launch_dq_pipe(const AttnParams& p, bool dense, hipStream_t stream) {
  if (p.cu_seqlens) return launch_one<false, true>(p, stream);
  return dense ? launch_one<true, false>(p, stream) : launch_one<false, false>(p, stream);
}

}  // namespace s2
