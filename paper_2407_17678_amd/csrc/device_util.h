// Internal device-side helpers for the gfx950 kernels: MFMA fragment types, the LDS tile layouts,
// and the global -> register -> LDS staging of a 64-row bf16 chunk, both row-major and
// transposed.
//
// Fragment conventions of v_mfma_f32_32x32x16_bf16 (D = A x B + C, 64 lanes, half = lane / 32):
//   A (32 x 16): lane holds row (lane % 32), the 8 k-values of its half.
//   B (16 x 32): lane holds column (lane % 32), the 8 k-values of its half.
//   C/D (32 x 32, 16 floats): lane holds column (lane % 32); register r is row
//        8*(r/4) + 4*half + (r%4).
// The contraction index may be permuted freely as long as A and B agree, which is what lets a
// C-layout tile be fed back as a B operand without moving data between lanes: registers
// 8u..8u+7 of a C tile are, for the lane's half, the rows {16u + 4*half + 0..3,
// 16u + 8 + 4*half + 0..3}; the matching A operand is stored in LDS in exactly that order
// (see TransposedTile).
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

// Value held by the lane 32 positions away (the other half of the wavefront).
__device__ __forceinline__ float other_half(float x) { return __shfl_xor(x, 32, 64); }

// Eight floats -> eight bf16 (round to nearest even, hardware conversion on gfx950).
__device__ __forceinline__ bf16x8 pack8(float a0, float a1, float a2, float a3, float a4, float a5,
                                        float a6, float a7) {
  bf16x8 r;
  r[0] = (__bf16)a0; r[1] = (__bf16)a1; r[2] = (__bf16)a2; r[3] = (__bf16)a3;
  r[4] = (__bf16)a4; r[5] = (__bf16)a5; r[6] = (__bf16)a6; r[7] = (__bf16)a7;
  return r;
}

// ---------------------------------------------------------------------------------------------
// Row-major LDS tile: 64 rows x D bf16, row stride D+8 elements.  (D+8)*2 bytes = 68 or 36
// dwords per row, so the 16 lanes of a b128 access that differ in row hit disjoint banks.
// Read as an MFMA A/B fragment whose 32-side is the tile row and whose k is the D axis.
// ---------------------------------------------------------------------------------------------
template <int D>
struct RowTile {
  static constexpr int kStride = D + 8;           // elements
  static constexpr int kElems = 64 * kStride;     // per tile
  static constexpr int kPieces = 64 * D / 8;      // 16-byte pieces
  static constexpr int kPerThread = kPieces / 256;

  // global -> registers (coalesced: consecutive threads take consecutive 16 bytes of a row)
  __device__ static __forceinline__ void load(u32x4 (&r)[kPerThread], const uint16_t* base,
                                              int64_t row_stride, int tid) {
#pragma unroll
    for (int n = 0; n < kPerThread; ++n) {
      const int p = tid + 256 * n;
      const int row = p / (D / 8), c = p % (D / 8);
      r[n] = *reinterpret_cast<const u32x4*>(base + (int64_t)row * row_stride + 8 * c);
    }
  }
  // registers -> LDS
  __device__ static __forceinline__ void store(const u32x4 (&r)[kPerThread], uint16_t* tile, int tid) {
#pragma unroll
    for (int n = 0; n < kPerThread; ++n) {
      const int p = tid + 256 * n;
      const int row = p / (D / 8), c = p % (D / 8);
      *reinterpret_cast<u32x4*>(tile + row * kStride + 8 * c) = r[n];
    }
  }
  // registers -> LDS when the chunk was loaded with TransposedTile's thread mapping (thread holds
  // rows 4a..4a+3, features 8c..8c+7), so one global load can feed both tile forms
  __device__ static __forceinline__ void store_quad(const u32x4 (&r)[4], uint16_t* tile, int tid) {
    if (tid >= 16 * (D / 8)) return;
    const int c = (tid & 3) + 4 * (tid >> 6), a = (tid >> 2) & 15;
#pragma unroll
    for (int n = 0; n < 4; ++n)
      *reinterpret_cast<u32x4*>(tile + (4 * a + n) * kStride + 8 * c) = r[n];
  }
  // fragment: row = 32*rt + lane%32, k-slab kk (16 values of D), this lane's half
  __device__ static __forceinline__ bf16x8 frag(const uint16_t* tile, int rt, int kk, int l32, int half) {
    return *reinterpret_cast<const bf16x8*>(tile + (32 * rt + l32) * kStride + 16 * kk + 8 * half);
  }
};

// ---------------------------------------------------------------------------------------------
// Transposed LDS tile: D rows (one per feature) x 64 columns (the chunk's tokens), row stride 72
// elements (36 dwords).  Inside each run of 16 tokens the column order is permuted so that one
// 16-byte read gives a lane the eight tokens its half contracts over when the other operand is
// a C-layout tile: column 16*slab + 8*half + e holds token 16*slab + 8*(e/4) + 4*half + e%4.
// On top of that, rows whose index has bit 4 set swap their two 32-token halves (column ^ 32):
// the 8-byte transposed stores of one wavefront go to rows 8c+e for four values of c, 8 rows are
// 32 banks apart, and without the swap c and c+2 would land on the same banks.
// Read as an MFMA A fragment whose 32-side is the feature and whose k is the token axis.
// ---------------------------------------------------------------------------------------------
template <int D>
struct TransposedTile {
  static constexpr int kStride = 72;
  static constexpr int kElems = D * kStride;
  static constexpr int kChunks = D / 8;  // 8-feature chunks per row of the source

  // thread -> (token group a of 4 rows, feature chunk c); threads beyond 16*kChunks idle
  __device__ static __forceinline__ bool mine(int tid) { return tid < 16 * kChunks; }
  __device__ static __forceinline__ int chunk_of(int tid) { return (tid & 3) + 4 * (tid >> 6); }
  __device__ static __forceinline__ int group_of(int tid) { return (tid >> 2) & 15; }

  __device__ static __forceinline__ void load(u32x4 (&r)[4], const uint16_t* base, int64_t row_stride,
                                              int tid) {
    if (!mine(tid)) return;
    const int c = chunk_of(tid), a = group_of(tid);
#pragma unroll
    for (int n = 0; n < 4; ++n)
      r[n] = *reinterpret_cast<const u32x4*>(base + (int64_t)(4 * a + n) * row_stride + 8 * c);
  }
  __device__ static __forceinline__ void store(const u32x4 (&r)[4], uint16_t* tile, int tid) {
    if (!mine(tid)) return;
    const int c = chunk_of(tid), a = group_of(tid);
    // rows 8c..8c+7 share bit 4 of the row index (c >> 1): the column swizzle below
    const int col = (16 * (a >> 2) + 8 * (a & 1) + 4 * ((a & 3) >> 1)) ^ (32 * ((c >> 1) & 1));
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      // dword m of each source row holds features 2m (low half) and 2m+1 (high half)
      u32x2 even, odd;
      even[0] = __builtin_amdgcn_perm(r[1][m], r[0][m], 0x05040100u);
      even[1] = __builtin_amdgcn_perm(r[3][m], r[2][m], 0x05040100u);
      odd[0] = __builtin_amdgcn_perm(r[1][m], r[0][m], 0x07060302u);
      odd[1] = __builtin_amdgcn_perm(r[3][m], r[2][m], 0x07060302u);
      *reinterpret_cast<u32x2*>(tile + (8 * c + 2 * m) * kStride + col) = even;
      *reinterpret_cast<u32x2*>(tile + (8 * c + 2 * m + 1) * kStride + col) = odd;
    }
  }
  // fragment: feature row = 32*ft + lane%32, token slab (16 tokens), this lane's half
  __device__ static __forceinline__ bf16x8 frag(const uint16_t* tile, int ft, int slab, int l32, int half) {
    const int col = (16 * slab + 8 * half) ^ (32 * ((l32 >> 4) & 1));
    return *reinterpret_cast<const bf16x8*>(tile + (32 * ft + l32) * kStride + col);
  }
};

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
// address a lane fetches: position p holds row p / stride, 16-byte piece (p % stride) / 16; the
// pad pieces at the end of each row fetch piece 0 of the same row (in bounds, never read).
//
// ds_read_b64_tr_b16, within each group of 16 lanes: lane 4e+q supplies the address of 4
// consecutive bf16 (row e of a 4 x 16 block, piece q); lane i receives element i of rows 0..3.
// So a group pointed at tokens t..t+3, features f..f+15 hands lane i the four tokens of feature
// f+i: exactly the k-order of half a C-layout B operand (see the top of this file).
// ---------------------------------------------------------------------------------------------
typedef short s16x4 __attribute__((ext_vector_type(4)));

template <int D>
struct DmaTile {
  static constexpr int kStride = (D == 128) ? 152 : 104;  // elements
  static constexpr int kElems = 64 * kStride;
  static constexpr int kBytes = kElems * 2;
  static constexpr int kInstr = kBytes / 1024;            // wavefront-wide loads per tile
  static constexpr int kPerWave = (kInstr + 3) / 4;
  static_assert(kBytes % 1024 == 0, "tile must be a whole number of wavefront loads");

  struct Plan {
    int32_t goff[kPerWave];  // element offset from the chunk's first row, per load of this lane
  };

  __device__ static __forceinline__ Plan plan(int64_t row_stride, int wave, int lane) {
    Plan pl;
#pragma unroll
    for (int n = 0; n < kPerWave; ++n) {
      const int pos = (4 * n + wave) * 1024 + lane * 16;
      const int row = pos / (kStride * 2);
      int piece = (pos - row * kStride * 2) / 16;
      if (piece >= D / 8) piece = 0;
      pl.goff[n] = (int32_t)(min(row, 63) * row_stride) + 8 * piece;
    }
    return pl;
  }

  // Starts the loads of one chunk; they are complete after s_waitcnt vmcnt(0).
  __device__ static __forceinline__ void issue(const Plan& pl, const uint16_t* gbase, uint16_t* tile,
                                               int wave) {
#pragma unroll
    for (int n = 0; n < kPerWave; ++n) {
      const int instr = 4 * n + wave;
      if (instr < kInstr)
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void*)(gbase + pl.goff[n]),
            (__attribute__((address_space(3))) void*)(tile + instr * 512), 16, 0, 0);
    }
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

// Everything outstanding (direct loads included) has landed.
__device__ __forceinline__ void wait_all_loads() { __builtin_amdgcn_s_waitcnt(0); }

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
__host__ __device__ inline int grid_for(int bh_total, int tiles) { return 8 * ((bh_total + 7) / 8) * tiles; }

}  // namespace s2
