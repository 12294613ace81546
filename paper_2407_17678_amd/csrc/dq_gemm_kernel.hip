// dQ launch of the backward that keeps dS (head_dim 128, mask blocks of 64 or 128 tokens): the
// dK/dV kernel, which runs first, has left dS = P * (dP - delta) in the workspace, rounded to bf16
// exactly as its own dK contraction takes it, so what remains of the gradient of section 3.2's
// forward on the query side is the single contraction dQ = scale * dS K over the kept blocks -
// nothing is recomputed (the row-stationary kernels in bwd_kernel.hip / dq_pipe_kernel.hip form S
// and dP a second time to get at dS).
//
// A workgroup owns 128 query rows and walks the 64-key chunks of the KV blocks its mask rows keep,
// as the other row-stationary kernels do.  Its four wavefronts split a chunk two by two: 64 query
// rows (one dS unit) x 32 keys each, so that every transposed K fragment read from LDS feeds two
// MFMAs - the kernel would otherwise be bound by the rate at which LDS takes instructions - and the
// two key halves are added through LDS when the tile is done.  Per chunk the K rows are staged for
// all four wavefronts and, per wavefront, the 4 KiB of dS that are its own: the dK/dV kernel wrote
// dS with the key on the lane, here the query has to be, so the pieces go through LDS and come back
// through the transpose read.  What bounds the kernel then is the one pass over dS in HBM (2 bytes
// per unmasked pair and 128 flop against it).
//
// dS in the workspace: units of 64 queries x 64 keys, 8 KiB each, found through AttnParams::dq_units;
// inside a unit [32-key half][32-query half][16-query slab][key][lane half][8 queries as the writing
// lane held them: 4 * half + 0..3, then 8 + 4 * half + 0..3].
#include <hip/hip_runtime.h>

#include <atomic>

#include "config.h"
#include "device_util.h"
#include "kernels.h"
#include "sched_util.h"

namespace s2 {

namespace {

// One wavefront's dS of a chunk in LDS: four 1 KiB pieces (32-query half t, 16-query slab u of it), piece
// (t, u) at t * 1024 + u * kDsSlabStride.  The 128 odd bytes put the two slabs half a bank row apart, so
// that the four 16-lane groups of a transpose read (slab, lane half) fall on different banks.
constexpr int kDsSlabStride = 2 * 1024 + 128;
constexpr int kDsWaveBytes = 2 * kDsSlabStride;

template <int D>
struct DqGemmSmem {
  union {
    struct {
      uint16_t k[2][DmaTile<D, 64, 4>::kElems];  // K rows of a chunk (the padded tile of device_util.h), two stages
      unsigned char ds[4][kDsWaveBytes];         // per wavefront: its dS of the current chunk
    } loop;
    float reduce[2][64 * D];  // after the loop: the second key half's sums, per 64-row half of the tile
  };
};

// The loads go through registers (plain loads the compiler tracks, two chunks in flight per
// wavefront, each 4 x 16 bytes of K and 4 x 16 bytes of dS per lane) rather than straight into LDS:
// the kernel lives on bytes in flight, registers are what it has plenty of, and with every load
// tracked the compiler's counted waits let the later chunks stay outstanding.
template <int D>
__global__ __launch_bounds__(kThreads, 2) void dq_gemm_kernel(const AttnParams p) {
  typedef DmaTile<D, 64, 4> Tile;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  DqGemmSmem<D>& sm = *reinterpret_cast<DqGemmSmem<D>*>(smem_raw);
  constexpr int BM = kBwdBM, DT = D / 32;
  static_assert(D == 128, "a chunk's K rows are 4 x 16 bytes per lane of the workgroup");

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = tid & 63, l32 = lane & 31, half = lane >> 5;
  const int T = p.q_tiles.tiles_per_head;
  int bh, rank;
  if (!map_workgroup(blockIdx.x, p.batch * p.heads, T, bh, rank)) return;
  const int b = bh / p.heads, h = bh - b * p.heads;
  const int tile = p.q_tiles.order[h * T + rank];
  const int S = p.block_size;  // 64 or 128
  const int cpb_sh = S == 128 ? 1 : 0, cpb_m = (1 << cpb_sh) - 1;
  const int qhalf = wave >> 1;             // which 64-row half of the tile: one dS unit per chunk
  const int khalf = wave & 1;              // which 32 keys of the chunk
  const int q0 = tile * BM + 64 * qhalf;   // first query row of this wavefront

  const int64_t q_off = b * p.q_sb + h * p.q_sh;
  const uint16_t* kb = p.k + b * p.kv_sb + h * p.kv_sh;
  const unsigned char* ds_b = reinterpret_cast<const unsigned char*>(p.ds_store) + (int64_t)b * p.ds_units * 8192;

  const int ent_lo = p.q_tiles.ptr[h * T + tile];
  const int n_ent = p.q_tiles.ptr[h * T + tile + 1] - ent_lo;
  const int total = n_ent << cpb_sh;  // chunks
  EntryList list, units;
  list.init(p.q_tiles.ent + ent_lo, n_ent, lane);
  units.init(p.dq_units + ((int64_t)ent_lo << cpb_sh) * 2, total * 2, lane);
  // chunk j (clamped to the last one): its first key row and the unit that holds dS for my half of
  // the tile (-1: not mine)
  auto chunk_at = [&](int j, int& kv0, int& unit) S2_INLINE {
    const bool inside = j < total;
    j = min(j, total - 1);
    const int e = list.get(j >> cpb_sh, lane);
    kv0 = (e >> 16) * S + (j & cpb_m) * 64;
    unit = units.get(2 * j + qhalf, lane);
    if (!inside) unit = -1;
  };

  // K: the workgroup's 256 lanes fetch 16 rows x 16 pieces per load, this lane row 16 i + tid / 16 of
  // the chunk for load i, piece tid % 16; dS: my key half of the unit, 4 KiB in one run
  const int k_row = tid >> 4, k_piece = tid & 15;
  const int64_t k_goff = (int64_t)k_row * p.kv_st + 8 * k_piece;     // elements
  const int k_loff = k_row * Tile::kStride + 8 * k_piece;            // elements
  const uint32_t ds_goff = 4096 * khalf + lane * 16;                 // bytes
  struct Fetch {
    u32x4 k[4], ds[4];
  };
  auto fetch = [&](Fetch& f, int kv0, int unit) S2_INLINE {
    const uint16_t* kg = kb + (int64_t)kv0 * p.kv_st + k_goff;
#pragma unroll
    for (int i = 0; i < 4; ++i) f.k[i] = *reinterpret_cast<const u32x4*>(kg + (int64_t)(16 * i) * p.kv_st);
    // a chunk that is not mine fetches unit 0 (it exists) so that every step issues the same loads
    const unsigned char* ug = ds_b + (int64_t)max(unit, 0) * 8192 + ds_goff;
#pragma unroll
    for (int i = 0; i < 4; ++i) f.ds[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(ug + 1024 * i));
  };
  // piece i of the run is (32-query half i / 2, slab i % 2)
  auto stash = [&](const Fetch& f, int stage, int unit) S2_INLINE {
    uint16_t* kt = sm.loop.k[stage] + k_loff;
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(kt + 16 * i * Tile::kStride) = f.k[i];
    if (unit < 0) return;
    unsigned char* dw = sm.loop.ds[wave] + lane * 16;
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(dw + 1024 * (i >> 1) + kDsSlabStride * (i & 1)) = f.ds[i];
  };

  f32x16 acc[2][DT];  // [32-query half][feature tile]
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) acc[t][dt] = f32x16{};
  const int trb = Tile::tr_base(lane);
  // lane part of a dS transpose read: group g = lane / 16 reads slab g % 2 for lane half g / 2; lane
  // 4 e + q of a group supplies key 4 (g / 2) + e, queries 4 q .. 4 q + 3 of the slab, which the writer's
  // lane half q % 2 holds as its first (q < 2) or second four
  const int g16 = lane >> 4, e4 = (lane & 15) >> 2, q4 = lane & 3;
  const uint32_t ds_trb = lds_addr(sm.loop.ds[wave]) + (g16 & 1) * kDsSlabStride + (4 * (g16 >> 1) + e4) * 32 + (q4 & 1) * 16 + (q4 >> 1) * 8;

  auto multiply = [&](int kv0, int unit, int stage) S2_INLINE {
    if (unit < 0) return;
    const uint16_t* ks = sm.loop.k[stage];
    const int kb32 = kv0 + 32 * khalf;  // my first key
    // keys all after the first 32 queries: the dK/dV kernel skipped that quarter, nothing was stored
    // (the unit exists, so they are not after the second 32)
    const bool first = kb32 <= q0;
#pragma unroll
    for (int sl = 0; sl < 2; ++sl) {  // 16-key slab of my 32 keys
      const u32x4 r1 = lds_read_tr(ds_trb, 1024 + 512 * sl, 32);
      u32x4 r0 = lds_read_tr(ds_trb, 512 * sl, 32);
      if (!first) r0 = u32x4{0u, 0u, 0u, 0u};  // what LDS holds there is not dS: that quarter counts as zero
      const bf16x8 d0 = __builtin_bit_cast(bf16x8, r0), d1 = __builtin_bit_cast(bf16x8, r1);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const bf16x8 kf = Tile::tr_frag(ks, dt, 2 * khalf + sl, trb);
        acc[0][dt] = mfma32(kf, d0, acc[0][dt]);
        acc[1][dt] = mfma32(kf, d1, acc[1][dt]);
      }
    }
  };

  if (total > 0) {
    // chunks 0 and 1 requested, chunk 0 in LDS
    Fetch fa, fb;
    int kv0[3], unit[3];  // of chunks ch, ch + 1, ch + 2
    chunk_at(0, kv0[0], unit[0]);
    fetch(fa, kv0[0], unit[0]);
    chunk_at(1, kv0[1], unit[1]);
    fetch(fb, kv0[1], unit[1]);
    stash(fa, 0, unit[0]);
    __syncthreads();
    // Step ch: request chunk ch + 2 into the registers chunk ch came through, multiply chunk ch, move
    // chunk ch + 1 from its registers to LDS (the other K stage; my dS region after my own reads of
    // it, LDS serves a wavefront in order), barrier.  Two steps per trip so that the register sets
    // keep their names.
    for (int ch = 0; ch < total; ch += 2) {
      chunk_at(ch + 2, kv0[2], unit[2]);
      fetch(fa, kv0[2], unit[2]);
      multiply(kv0[0], unit[0], 0);
      stash(fb, 1, unit[1]);
      __syncthreads();
      if (ch + 1 >= total) break;
      chunk_at(ch + 3, kv0[0], unit[0]);
      fetch(fb, kv0[0], unit[0]);
      multiply(kv0[1], unit[1], 1);
      stash(fa, 0, unit[2]);
      __syncthreads();
      kv0[1] = kv0[0];
      unit[1] = unit[0];
      kv0[0] = kv0[2];
      unit[0] = unit[2];
    }
  }

  // The second key half hands its sums over through LDS (free since the loop's last barrier), register
  // by register with the lane as the fast index; the first adds them and owns the rows from here on.
  float* red = sm.reduce[qhalf] + lane;
  if (khalf == 1) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) red[((t * DT + dt) * 16 + r) * 64] = acc[t][dt][r];
  }
  __syncthreads();
  if (khalf == 1) return;
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[t][dt][r] += red[((t * DT + dt) * 16 + r) * 64];

  // dQ = scale * acc goes out through LDS (my half of the reduction buffer, which only I read, after my
  // own reads of it), whole rows per store instruction
  constexpr int RS = D + 8;  // staging row stride (elements)
  uint16_t* stage = reinterpret_cast<uint16_t*>(sm.reduce[qhalf]);
  static_assert(64 * RS * 2 <= 64 * D * 4, "the staging rows fit the reduction buffer");
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (__bf16)(acc[t][dt][4 * g + e] * p.scale);
        *reinterpret_cast<bf16x4*>(stage + (32 * t + l32) * RS + 32 * dt + 8 * g + 4 * half) = w;
      }
  uint16_t* obase = p.dq + q_off + (int64_t)q0 * p.q_st;
#pragma unroll
  for (int i = 0; i < 64 / 4; ++i) {
    const int r = 4 * i + (lane >> 4), piece = lane & 15;
    const u32x4 x = *reinterpret_cast<const u32x4*>(stage + r * RS + 8 * piece);
    *reinterpret_cast<u32x4*>(obase + (int64_t)r * p.q_st + 8 * piece) = x;
  }
}

// A kernel's dynamic LDS limit is a per-device attribute: remember, per device, that it is set.
constexpr int kMaxDevices = 64;
std::atomic<unsigned char> g_smem_set[kMaxDevices];

}  // namespace

hipError_t launch_dq_gemm(const AttnParams& p, hipStream_t stream) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < kMaxDevices;
  if (!tracked || !g_smem_set[dev].load(std::memory_order_acquire)) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dq_gemm_kernel<128>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(DqGemmSmem<128>));
    if (e != hipSuccess) return e;
    if (tracked) g_smem_set[dev].store(1, std::memory_order_release);
  }
  const int grid = grid_for(p.batch * p.heads, p.q_tiles.tiles_per_head);
  hipLaunchKernelGGL((dq_gemm_kernel<128>), dim3(grid), dim3(kThreads), sizeof(DqGemmSmem<128>), stream, p);
  return hipGetLastError();
}

}  // namespace s2
