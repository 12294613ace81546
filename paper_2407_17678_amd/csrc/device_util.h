// Internal device-side helpers for the gfx950 kernels: MFMA fragment types, the LDS tile that a
// 64-row bf16 chunk is staged in (direct global -> LDS loads, row and transposed fragment reads),
// and the workgroup -> tile mappings.
//
// Fragment conventions of v_mfma_f32_32x32x16_bf16 (D = A x B + C, 64 lanes, half = lane / 32):
//   A (32 x 16): lane holds row (lane % 32), the 8 k-values of its half.
//   B (16 x 32): lane holds column (lane % 32), the 8 k-values of its half.
//   C/D (32 x 32, 16 floats): lane holds column (lane % 32); register r is row
//        8*(r/4) + 4*half + (r%4).
// The contraction index may be permuted freely as long as A and B agree, which is what lets a
// C-layout tile be fed back as a B operand without moving data between lanes: registers
// 8u..8u+7 of a C tile are, for the lane's half, the rows {16u + 4*half + 0..3,
// 16u + 8 + 4*half + 0..3}; the matching A operand is fetched from LDS in exactly that order
// (see DmaTile::tr_frag).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace s2 {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// x of this lane combined with x of the lane 32 positions away (the other half of the wavefront).
// v_permlane32_swap exchanges the upper half of one register with the lower half of another: fed
// the same value twice it leaves one register holding the lower half's values in both halves and
// the other the upper half's, so no trip through LDS (and no wait on the LDS counter) is needed.
// Written as inline assembly: with this compiler the builtin's two results come back as one and
// the same register.  The s_nop covers the wait states the instruction needs after a VALU write of
// its operands (the compiler cannot see into the assembly to add them).
__device__ __forceinline__ void swap_halves(float x, float& lo, float& hi) {
  lo = x;
  hi = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(lo), "+v"(hi));
}
__device__ __forceinline__ float max_halves(float x) {
  float a, b;
  swap_halves(x, a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float sum_halves(float x) {
  float a, b;
  swap_halves(x, a, b);
  return a + b;
}

// Eight floats -> eight bf16 (round to nearest even, hardware conversion on gfx950).
__device__ __forceinline__ bf16x8 pack8(float a0, float a1, float a2, float a3, float a4, float a5,
                                        float a6, float a7) {
  bf16x8 r;
  r[0] = (__bf16)a0; r[1] = (__bf16)a1; r[2] = (__bf16)a2; r[3] = (__bf16)a3;
  r[4] = (__bf16)a4; r[5] = (__bf16)a5; r[6] = (__bf16)a6; r[7] = (__bf16)a7;
  return r;
}

// ---------------------------------------------------------------------------------------------
// DmaTile: a 64-row x D bf16 chunk kept row-major in LDS and filled by direct global -> LDS loads
// (global_load_lds_dwordx4: no staging registers, no LDS store instructions).  Both operand
// forms are read from this one tile: row fragments with 16-byte reads (k = feature) and
// transposed fragments with the LDS transpose read ds_read_b64_tr_b16 (k = token).
//
// Row stride is 76 dwords for D = 128 and 52 dwords for D = 64: measured on gfx950, these are
// strides at which both the 16-byte row reads (32 consecutive rows, the two wavefront halves 16
// bytes apart) and the transpose reads (groups of 16 lanes covering 4 rows x 32 bytes) run at the
// conflict-free rate.  Both tile sizes are whole multiples of the 1024 bytes one wavefront-wide
// direct load fills.
//
// Direct loads write LDS at (wave-uniform base) + 16 * lane, so LDS position decides which global
// address a lane fetches: position p holds row p / stride, 16-byte piece (p % stride) / 16; lanes
// that fall on the pad pieces at the end of a row fetch something harmless (nothing reads the
// padding).
//
// ds_read_b64_tr_b16, within each group of 16 lanes: lane 4e+q supplies the address of 4
// consecutive bf16 (row e of a 4 x 16 block, piece q); lane i receives element i of rows 0..3.
// So a group pointed at tokens t..t+3, features f..f+15 hands lane i the four tokens of feature
// f+i: exactly the k-order of half a C-layout B operand (see the top of this file).
// ---------------------------------------------------------------------------------------------
typedef short s16x4 __attribute__((ext_vector_type(4)));

// Byte address inside LDS of a pointer to __shared__ memory.
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

// One wavefront-wide direct load: lane i fetches `bytes` (16 or 4) from its own global address
// into LDS at lds_base + bytes * i.  lds_base must be wave-uniform (it goes through M0).
// Written as inline assembly on purpose: the compiler then does not track these loads and so does
// not make unrelated LDS reads wait for a prefetch in flight; the kernels wait for them explicitly
// (wait_all_loads) before the barrier that publishes a stage.  Untracked loads only make the
// compiler's own vmcnt waits more conservative, never less (the counter retires in order).
// The global address is a wave-uniform base (scalar registers) plus a per-lane unsigned 32-bit
// byte offset, so a lane spends one register per load and no 64-bit address arithmetic.
// The s_nop is the wait state a scalar write of M0 needs before an instruction that reads it (the
// compiler would add it for its own code; it does not look inside inline assembly).  M0 is named
// as clobbered so that the compiler does not expect a value of its own to survive there (it warns
// that M0 is a reserved register; the clobber is honoured all the same).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(const void* gbase, uint32_t byte_off, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(byte_off), "s"(gbase), "s"(lds_base)
               : "memory", "m0");
}
__device__ __forceinline__ void dma4(const void* gbase, uint32_t byte_off, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(byte_off), "s"(gbase), "s"(lds_base)
               : "memory", "m0");
}
// Up to four loads that share one M0 value.  The instruction's immediate offset is added to the
// global address AND to the LDS address, so loads whose LDS targets are 1 KiB apart need only
// one scalar write of M0 (and one wait state) between them; the caller takes the immediate back
// out of the lane's global offset.  kCount loads, the i-th with immediate 1024 * i.
template <int kCount>
__device__ __forceinline__ void dma16_group(const void* gbase, uint32_t lds_base, uint32_t o0, uint32_t o1,
                                            uint32_t o2, uint32_t o3) {
  static_assert(kCount >= 1 && kCount <= 4, "immediates 0 .. 3072");
  if constexpr (kCount == 4)
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %2, %0\n\tglobal_load_lds_dwordx4 %3, %0 offset:1024\n\t"
                 "global_load_lds_dwordx4 %4, %0 offset:2048\n\tglobal_load_lds_dwordx4 %5, %0 offset:3072"
                 ::"s"(gbase), "s"(lds_base), "v"(o0), "v"(o1), "v"(o2), "v"(o3)
                 : "m0");
  else if constexpr (kCount == 3)
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %2, %0\n\tglobal_load_lds_dwordx4 %3, %0 offset:1024\n\t"
                 "global_load_lds_dwordx4 %4, %0 offset:2048"
                 ::"s"(gbase), "s"(lds_base), "v"(o0), "v"(o1), "v"(o2)
                 : "m0");
  else if constexpr (kCount == 2)
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %2, %0\n\tglobal_load_lds_dwordx4 %3, %0 offset:1024"
                 ::"s"(gbase), "s"(lds_base), "v"(o0), "v"(o1)
                 : "m0");
  else
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %0" ::"s"(gbase), "s"(lds_base), "v"(o0)
                 : "m0");
}
#pragma clang diagnostic pop

template <int D, int ROWS = 64, int NW = 4>
struct DmaTile {
  static constexpr int kStride = (D == 128) ? 152 : 104;  // elements
  static constexpr int kInstr = (ROWS * kStride * 2 + 1023) / 1024;  // wavefront-wide loads per tile
  static constexpr int kBytes = kInstr * 1024;            // the last load may run past the last row
  static constexpr int kElems = kBytes / 2;
  static constexpr int kPerWave = (kInstr + NW - 1) / NW;  // NW wavefronts share the loads

  struct Plan {
    uint32_t goff[kPerWave];  // byte offset from the chunk's first row, per load of this lane
  };

  // Every lane of every load gets a valid address, so that the loads need no branches around them
  // (a branch would also split the basic block and keep the compiler from scheduling MFMAs and
  // loads together): a lane that falls on row padding fetches a piece of its row again (it lands
  // in the padding, which nothing reads), and a wavefront with one load fewer than the others
  // repeats its last one.
  __device__ static __forceinline__ Plan plan(int64_t row_stride, int wave, int lane) {
    Plan pl;
#pragma unroll
    for (int n = 0; n < kPerWave; ++n) {
      const int instr = min(NW * n + wave, kInstr - 1);
      const int pos = instr * 1024 + lane * 16;
      int row = pos / (kStride * 2);
      int piece = (pos - row * kStride * 2) / 16;
      if (piece >= D / 8) piece -= D / 8;
      if (row >= ROWS) row = ROWS - 1;  // past the tile: lands in the slack after the last row
      pl.goff[n] = (uint32_t)(row * row_stride * 2) + 16 * piece;
    }
    return pl;
  }

  // The same for a chunk of which only the first `rows_valid` rows exist (the ragged end of a
  // sequence): loads of later rows fetch the last existing row instead; nothing may use them.
  __device__ static __forceinline__ Plan plan_rows(int64_t row_stride, int wave, int lane, int rows_valid) {
    Plan pl;
    const int last = max(rows_valid, 1) - 1;
#pragma unroll
    for (int n = 0; n < kPerWave; ++n) {
      const int instr = min(NW * n + wave, kInstr - 1);
      const int pos = instr * 1024 + lane * 16;
      int row = pos / (kStride * 2);
      int piece = (pos - row * kStride * 2) / 16;
      if (piece >= D / 8) piece -= D / 8;
      row = min(min(row, ROWS - 1), last);
      pl.goff[n] = (uint32_t)(row * row_stride * 2) + 16 * piece;
    }
    return pl;
  }

  // One of the kPerWave loads of a chunk, so that a kernel can spread them between MFMAs.
  // Complete after s_waitcnt vmcnt(0).
  __device__ static __forceinline__ void issue_one(const Plan& pl, int n, const uint16_t* gbase,
                                                   const uint16_t* tile, int wave) {
    const int instr = min(NW * n + wave, kInstr - 1);
    dma16(gbase, pl.goff[n], lds_addr(tile) + instr * 1024);
  }
  // ---- loads dealt to the wavefronts in blocks, issued in groups of up to four per M0 write ----
  // Wavefront w fetches kBlock consecutive loads of the tile (consecutive kilobytes of LDS),
  // starting at load min(w * kBlock, kInstr - kBlock): where the blocks do not divide the tile
  // evenly the last wavefront starts early and fetches a load or two twice (same data, same place)
  // rather than having a shorter block, so that every wavefront runs the same instructions.  A group
  // of four shares one M0 value and tells its loads apart by the instruction's immediate offset,
  // which the hardware adds to the global address as well: the lane offsets of the plan have it
  // taken out again, plus kBias so that they stay non-negative (the caller passes the chunk's
  // address minus kBias bytes).
  static constexpr int kBlock = (kInstr + NW - 1) / NW;
  static constexpr int kGroups = (kBlock + 3) / 4;
  static constexpr uint32_t kBias = 3072;
  struct BlockPlan {
    uint32_t goff[kBlock];
  };
  __device__ static __forceinline__ int block_start(int wave) { return min(wave * kBlock, kInstr - kBlock); }
  __device__ static __forceinline__ BlockPlan block_plan(int64_t row_stride, int wave, int lane) {
    BlockPlan pl;
#pragma unroll
    for (int n = 0; n < kBlock; ++n) {
      const int pos = (block_start(wave) + n) * 1024 + lane * 16;
      int row = pos / (kStride * 2);
      int piece = (pos - row * kStride * 2) / 16;
      if (piece >= D / 8) piece -= D / 8;
      if (row >= ROWS) row = ROWS - 1;  // past the tile: lands in the slack after the last row
      pl.goff[n] = (uint32_t)(row * row_stride * 2) + 16 * piece + kBias - 1024 * (n & 3);
    }
    return pl;
  }
  // group G of this wavefront's loads; gbase_biased = address of the chunk's first row minus kBias bytes
  template <int G>
  __device__ static __forceinline__ void issue_group(const BlockPlan& pl, const void* gbase_biased, const uint16_t* tile,
                                                     int wave) {
    static_assert(G >= 0 && G < kGroups, "group index");
    constexpr int first = 4 * G;
    constexpr int count = (kBlock - first) < 4 ? (kBlock - first) : 4;
    const uint32_t lds = lds_addr(tile) + (block_start(wave) + first) * 1024;
    dma16_group<count>(gbase_biased, lds, pl.goff[first], pl.goff[first + (count > 1 ? 1 : 0)],
                       pl.goff[first + (count > 2 ? 2 : 0)], pl.goff[first + (count > 3 ? 3 : 0)]);
  }
  // All loads of one chunk.
  __device__ static __forceinline__ void issue(const Plan& pl, const uint16_t* gbase, const uint16_t* tile,
                                               int wave) {
#pragma unroll
    for (int n = 0; n < kPerWave; ++n) issue_one(pl, n, gbase, tile, wave);
  }

  // row fragment: row = 32*rt + lane%32, features 16*kk + 8*half .. +7
  __device__ static __forceinline__ bf16x8 row_frag(const uint16_t* tile, int rt, int kk, int l32, int half) {
    return *reinterpret_cast<const bf16x8*>(tile + (32 * rt + l32) * kStride + 16 * kk + 8 * half);
  }

  // lane-dependent part of a transposed fragment's address (elements)
  __device__ static __forceinline__ int tr_base(int lane) {
    const int g = lane >> 4, e = (lane & 15) >> 2, q = lane & 3;
    return (4 * (g >> 1) + e) * kStride + 16 * (g & 1) + 4 * q;
  }
  // transposed fragment: features 32*ft + lane%32, the 16 tokens of `slab` in C-layout k order
  __device__ static __forceinline__ bf16x8 tr_frag(const uint16_t* tile, int ft, int slab, int trb) {
    typedef __attribute__((address_space(3))) s16x4* lds_ptr;
    const uint16_t* p = tile + trb + 16 * slab * kStride + 32 * ft;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(p + 8 * kStride));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
  }
};

// Everything outstanding (direct loads included) has landed.  This is the builtin, not inline
// assembly, so that the compiler also learns that its own earlier loads (fragments fetched before
// a loop, say) are complete: otherwise it keeps re-waiting for them inside the loop with small
// vmcnt values, and such a wait drains the untracked direct loads that were issued after them.
__device__ __forceinline__ void wait_all_loads() {
  __builtin_amdgcn_s_waitcnt(0);  // vmcnt(0) expcnt(0) lgkmcnt(0)
  asm volatile("" ::: "memory");
}

// At most N of this wavefront's vector-memory operations are still outstanding.  The counter retires in
// issue order, loads and stores alike, so this says that everything issued before the last N has landed
// (direct loads included) without waiting for the last N themselves - stores whose completion nothing
// in the kernel depends on, or loads that are a further step ahead.
template <int N>
__device__ __forceinline__ void wait_loads_but() {
  static_assert(N >= 0 && N < 64, "the counter has six bits");
  // (the caller counts on its last N operations having been issued by now: no store may sink below)
  asm volatile("" ::: "memory");
  // vmcnt in bits 3:0 and 15:14; expcnt (bits 6:4) and lgkmcnt (bits 11:8) at their maxima: no wait
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
  asm volatile("" ::: "memory");
}

// A tile's entry list, held in registers: lane i of the wavefront keeps entry 64*b + i of the
// current batch of 64 entries, and the next batch is fetched one batch ahead, so the main loops
// read their block index with v_readlane instead of waiting on global memory every iteration.
struct EntryList {
  const int32_t* ent;
  int n;         // entries in the list
  int batch;     // which batch of 64 `cur` holds
  int cur, nxt;  // my entry of the current / next batch
  __device__ __forceinline__ void init(const int32_t* list, int count, int lane) {
    ent = list;
    n = count;
    batch = 0;
    cur = lane < n ? ent[lane] : 0;
    nxt = 64 + lane < n ? ent[64 + lane] : 0;
  }
  // entry e (wave-uniform); e never decreases between calls
  __device__ __forceinline__ int get(int e, int lane) {
    if ((e >> 6) != batch) {  // crossed into the next batch
      batch = e >> 6;
      cur = nxt;
      const int i = 64 * (batch + 1) + lane;
      nxt = i < n ? ent[i] : 0;
    }
    return __builtin_amdgcn_readlane(cur, e & 63);
  }
  // entry j of the current or the next batch (64*batch <= j < 64*batch + 128); does not advance
  __device__ __forceinline__ int peek(int j) const {
    return (j >> 6) != batch ? __builtin_amdgcn_readlane(nxt, j & 63) : __builtin_amdgcn_readlane(cur, j & 63);
  }
  // entry e+1, given that get(e) was the last call; does not advance
  __device__ __forceinline__ int peek_next(int e) const {
    return ((e + 1) >> 6) != batch ? __builtin_amdgcn_readlane(nxt, 0)
                                   : __builtin_amdgcn_readlane(cur, (e + 1) & 63);
  }
};

// Workgroup index -> (batch*head, rank inside the head) such that all tiles of one (batch, head)
// run on one XCD.  Workgroups are handed to the 8 XCDs round-robin by linear index, and each XCD
// has its own L2: keeping a head's key/value stripes and moving window on one XCD lets every
// later query tile of that head hit in that L2.
__device__ __forceinline__ bool map_workgroup(int wg, int bh_total, int tiles, int& bh, int& rank) {
  const int x = wg & 7, slot = wg >> 3;
  const int k = slot / tiles;
  rank = slot - k * tiles;
  bh = x + 8 * k;
  return bh < bh_total;
}
// Same XCD assignment, but the (batch, head) pairs of an XCD are interleaved: all their longest
// tiles are dispatched first, then all their second longest, ...  Used where tile lengths are very
// uneven (key tiles on a stripe are attended by hundreds of query blocks, the others by a few), so
// that the longest tile of the last head does not start late and become the tail of the launch.
__device__ __forceinline__ bool map_workgroup_interleaved(int wg, int bh_total, int tiles, int& bh,
                                                          int& rank) {
  const int x = wg & 7, slot = wg >> 3;
  const int per_xcd = (bh_total + 7) >> 3;  // slots are laid out for the fullest XCD
  rank = slot / per_xcd;
  bh = x + 8 * (slot - rank * per_xcd);
  return bh < bh_total;
}
__host__ __device__ inline int grid_for(int bh_total, int tiles) { return 8 * ((bh_total + 7) / 8) * tiles; }

}  // namespace s2
