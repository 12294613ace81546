// Internal: helpers for the hand-scheduled kernels (one MFMA per "slot", with its share of the
// vector work, LDS reads and direct loads, fenced so that the compiler keeps the order).
//
// What the schedules are built on, measured on gfx950 with small probes (one or two wavefronts per
// SIMD, random bf16 operands so that the clocks are those of a real load):
//   * a 32x32x16 bf16 MFMA occupies the matrix pipe for 32 cycles and the vector issue port for
//     about 8; four to five ordinary vector instructions (4 cycles each) fit beside it, and the
//     matrix and vector work of ONE instruction stream overlap perfectly when they alternate this
//     finely, while a burst of MFMAs keeps the port from another wavefront's vector instructions;
//   * sustained (tens of milliseconds, power-limited clocks) a SIMD completes one such MFMA every
//     18.6 ns with two wavefronts and nothing else to do: 1.8 PFLOP/s for the chip, 72 % of the
//     2.5 PFLOP/s that 2.4 GHz would give; with the softmax's vector work beside it 21.2 ns;
//   * a lone wavefront on a SIMD issues at most one instruction per 4 cycles of whatever kind, and a
//     scalar ALU instruction between vector ones costs it about 10 cycles; a second wavefront on
//     the SIMD hides all of that, which is why these kernels run two per SIMD (forms with one
//     wavefront per SIMD, 64 rows each and all 512 registers, were built and measured slower);
//   * back-to-back MFMAs into the same accumulator run at full rate.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>
#include <utility>

#include "device_util.h"

namespace s2 {

// Nothing is scheduled across this point.
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

// LDS reads at (32-bit LDS byte address held in a register) + (compile-time byte offset): the hand
// schedules form a lane's address parts once per step and then read at immediates.
#define S2_LDS_PTR(T, addr) ((const __attribute__((address_space(3))) T*)(uintptr_t)(addr))
__device__ __forceinline__ u32x4 lds_read16(uint32_t addr, int byte_off) {
  return *S2_LDS_PTR(u32x4, addr + byte_off);
}
__device__ __forceinline__ f32x4 lds_read_f32x4(uint32_t addr, int byte_off) {
  return *S2_LDS_PTR(f32x4, addr + byte_off);
}
// transposed fragment (see DmaTile::tr_frag): two ds_read_b64_tr_b16, the second 8 rows further on
__device__ __forceinline__ u32x4 lds_read_tr(uint32_t addr, int byte_off, int row_bytes) {
  typedef short s16x4_ __attribute__((ext_vector_type(4)));
  typedef short s16x8_ __attribute__((ext_vector_type(8)));
  typedef __attribute__((address_space(3))) s16x4_* tr_ptr;
  const s16x4_ lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)(uintptr_t)(addr + byte_off));
  const s16x4_ hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)(uintptr_t)(addr + byte_off + 8 * row_bytes));
  const s16x8_ both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(u32x4, both);
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  bf16x2 w;
  w[0] = (__bf16)lo;
  w[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, w);
}

}  // namespace s2
