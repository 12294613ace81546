// Ceiling probes: what the chip sustains on the two resources the kernels of this library are
// bound by, measured the same way the kernels are (HIP events around launches of a few
// milliseconds, so that the clocks are the power-limited ones of a real load).  The benchmark
// reports them beside the published peaks.
//   * MFMA: every SIMD runs two wavefronts that issue v_mfma_f32_32x32x16_bf16 back to back on
//     random bf16 operands (operand values matter: constant data draws less power and clocks
//     higher), alone or with the vector work of a softmax per MFMA beside it (one multiply-add,
//     one exponential, one add, half a conversion, half a maximum).
//   * HBM: a grid-stride read of a buffer with 16-byte loads.
//   * fp32 atomic adds to global memory, coalesced (what accumulating dQ partials in a single-pass
//     backward would cost: the reason this library's backward is two launches without atomics).
#include <hip/hip_runtime.h>

#include "../../include/s2attn.h"
#include "device_util.h"

namespace s2 {

namespace {

__device__ inline uint32_t mix32(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7feb352dU;
  x ^= x >> 15;
  x *= 0x846ca68bU;
  x ^= x >> 16;
  return x;
}
// two bf16 with random sign and mantissa and magnitudes in [0.25, 2)
__device__ inline uint32_t random_bf16x2(uint32_t seed) {
  const uint32_t h = mix32(seed);
  const uint32_t lo = (h & 0x80ffu) | 0x3f00u | ((h >> 3) & 0x0080u);
  const uint32_t hi = ((h >> 16) & 0x80ffu) | 0x3e80u;
  return lo | (hi << 16);
}

template <bool MIX>
__global__ __launch_bounds__(256, 2) void probe_mfma_kernel(float* out, int iters) {
  bf16x8 a[4], b[4];
#pragma unroll
  for (int f = 0; f < 4; ++f) {
    u32x4 ua, ub;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      ua[j] = random_bf16x2(threadIdx.x * 131u + f * 17u + j + blockIdx.x * 7919u);
      ub[j] = random_bf16x2(threadIdx.x * 977u + f * 29u + j * 5u + 3u + blockIdx.x * 104729u);
    }
    a[f] = __builtin_bit_cast(bf16x8, ua);
    b[f] = __builtin_bit_cast(bf16x8, ub);
  }
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) acc[j] = f32x16{};
  float v[8], l = 0.f, m = 0.f;
  uint32_t pk = 0;
#pragma unroll
  for (int r = 0; r < 8; ++r) v[r] = 0.5f + 0.001f * threadIdx.x + r;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      // (operands below 2 in magnitude: the sums stay finite for any iters the entry point accepts)
      acc[u & 3] = mfma32(a[u & 3], b[(u + 1) & 3], acc[u & 3]);
      if (MIX) {
        v[u & 7] = __builtin_fmaf(v[u & 7], 0.9991f, 0.0013f);
        v[(u + 3) & 7] = fast_exp2(v[(u + 3) & 7] * 0.01f);
        l += v[(u + 5) & 7];
        if (u & 1) {
          const bf16x4 w = {(__bf16)v[(u + 6) & 7], (__bf16)v[(u + 7) & 7], (__bf16)0.f, (__bf16)0.f};
          pk ^= __builtin_bit_cast(u32x2, w)[0];
        } else {
          m = fmaxf(fmaxf(m, v[(u + 1) & 7]), v[(u + 2) & 7]);
        }
        asm volatile("" : "+v"(l), "+v"(m), "+v"(pk));  // keeps the vector work beside its MFMA
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float s = l + m + (float)pk;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[j][r];
#pragma unroll
  for (int r = 0; r < 8; ++r) s += v[r];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4* src, size_t n16, uint32_t* out) {
  uint32_t s = 0;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
    const u32x4 x = src[i];
    s ^= x[0] ^ x[1] ^ x[2] ^ x[3];
  }
  out[blockIdx.x * 256 + threadIdx.x] = s;
}

// Coalesced fp32 atomic adds, the way a single-pass backward would accumulate dQ partials: each
// workgroup adds 16 KB tiles (32 rows x 128 floats) into a [rows x 128] buffer, the tiles of
// concurrent workgroups apart, later ones revisiting rows as other key tiles would.
__global__ __launch_bounds__(256) void probe_atomic_kernel(float* buf, uint32_t tiles, int tiles_per_wg) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int t = 0; t < tiles_per_wg; ++t) {
    const uint32_t tile = (uint32_t)(((uint64_t)blockIdx.x * 131u + (uint64_t)t * 977u) % tiles);
    float* base = buf + (size_t)tile * 32 * 128;
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
        atomicAdd(base + (size_t)(wave * 8 + 2 * r + (lane >> 5)) * 128 + 32 * dt + (lane & 31), 1.0f);
  }
}

constexpr int kProbeGrid = 512;  // two workgroups of four wavefronts per compute unit

}  // namespace

}  // namespace s2

extern "C" {

size_t s2_probe_scratch_bytes(void) { return (size_t)s2::kProbeGrid * 256 * sizeof(float); }

int s2_probe_mfma(int32_t with_vector_work, int32_t iters, void* scratch, void* stream, double* flops) {
  if (!scratch || !flops) return S2_ERR_NULL;
  if (iters < 1 || iters > (1 << 24)) return S2_ERR_BAD_PARAM;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (with_vector_work)
    hipLaunchKernelGGL((s2::probe_mfma_kernel<true>), dim3(s2::kProbeGrid), dim3(256), 0, st, static_cast<float*>(scratch), iters);
  else
    hipLaunchKernelGGL((s2::probe_mfma_kernel<false>), dim3(s2::kProbeGrid), dim3(256), 0, st, static_cast<float*>(scratch), iters);
  if (hipGetLastError() != hipSuccess) return S2_ERR_HIP;
  // 8 MFMAs per trip and wavefront, 2 * 32 * 32 * 16 flops each
  *flops = (double)s2::kProbeGrid * 4 * (double)iters * 8 * 32768.0;
  return S2_OK;
}

int s2_probe_read(const void* src, size_t bytes, void* scratch, void* stream) {
  if (!src || !scratch) return S2_ERR_NULL;
  if (bytes < 16 || (reinterpret_cast<uintptr_t>(src) & 15u) != 0) return S2_ERR_ALIGN;
  // enough workgroups to cover every compute unit several times over
  hipLaunchKernelGGL(s2::probe_read_kernel, dim3(4096), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const s2::u32x4*>(src), bytes / 16, static_cast<uint32_t*>(scratch));
  return hipGetLastError() == hipSuccess ? S2_OK : S2_ERR_HIP;
}

int s2_probe_atomic_add(void* buf, size_t bytes, void* stream, double* bytes_added) {
  if (!buf || !bytes_added) return S2_ERR_NULL;
  if (bytes < (1u << 20) || (reinterpret_cast<uintptr_t>(buf) & 15u) != 0) return S2_ERR_ALIGN;
  const uint64_t tiles = bytes / 16384;
  if (tiles > 0xffffffffu) return S2_ERR_BAD_PARAM;
  const int wgs = 8192, per_wg = 64;
  hipLaunchKernelGGL(s2::probe_atomic_kernel, dim3(wgs), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<float*>(buf), (uint32_t)tiles, per_wg);
  *bytes_added = (double)wgs * per_wg * 16384.0;
  return hipGetLastError() == hipSuccess ? S2_OK : S2_ERR_HIP;
}

}  // extern "C"
