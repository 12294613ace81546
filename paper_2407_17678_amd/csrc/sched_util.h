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
//     scalar ALU instruction between vector ones costs it about 10 cycles: its schedules keep
//     scalar work out of the loop; a second wavefront on the SIMD hides all of that;
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

// MFMAs as inline assembly, for kernels that run one wavefront per SIMD with all 512 registers:
// the compiler would put EVERY MFMA result of such a kernel into the accumulation registers and
// copy it out for each vector instruction; written this way each accumulator sits in the register
// file it belongs to.  The compiler does not see through them, so the wait states the hardware
// needs between an MFMA and a vector instruction that reads its result (11 for this 8-pass MFMA),
// and between a vector instruction and an MFMA that reads its result (2), are the caller's
// business: mfma_result_fence / mfma_operand_fence below.
// d (vector registers) = a x b
__device__ __forceinline__ void mfma_vz(f32x16& d, u32x4 a, u32x4 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "v"(b));
}
// d (vector registers) += a x b
__device__ __forceinline__ void mfma_v(f32x16& d, u32x4 a, u32x4 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "v"(b));
}
// the same with b in accumulation registers
__device__ __forceinline__ void mfma_vz_ab(f32x16& d, u32x4 a, u32x4 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma_v_ab(f32x16& d, u32x4 a, u32x4 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "a"(b));
}
// d (accumulation registers) += a x b
__device__ __forceinline__ void mfma_a(f32x16& d, u32x4 a, u32x4 b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b));
}
// 12 wait states after the MFMAs that wrote d, before vector instructions read it
__device__ __forceinline__ void mfma_result_fence(f32x16& d) { asm volatile("s_nop 7\n\ts_nop 3" : "+v"(d)); }
__device__ __forceinline__ void mfma_result_fence(f32x16& d0, f32x16& d1) {
  asm volatile("s_nop 7\n\ts_nop 3" : "+v"(d0), "+v"(d1));
}
// 2 wait states after the vector instructions that wrote b, before an MFMA reads it
__device__ __forceinline__ void mfma_operand_fence(u32x4& b) { asm volatile("s_nop 1" : "+v"(b)); }
__device__ __forceinline__ void mfma_operand_fence(u32x4& b0, u32x4& b1) { asm volatile("s_nop 1" : "+v"(b0), "+v"(b1)); }

// 16 bytes from global memory straight into accumulation registers (complete after s_waitcnt vmcnt(0);
// the compiler does not track it)
__device__ __forceinline__ void load_to_agpr(u32x4& dst, const void* src) {
  asm volatile("global_load_dwordx4 %0, %1, off" : "=a"(dst) : "v"(src));
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
