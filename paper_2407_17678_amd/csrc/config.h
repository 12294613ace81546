// Internal: tile shapes shared by the layout builder (which sizes the merged lists) and the kernels.
#pragma once

namespace s2 {
constexpr int kChunk = 64;      // keys (or queries) staged through LDS per inner step
constexpr int kFwdChunk = 64;   // keys per forward step (one LDS stage): 64 or 32
constexpr int kFwdBM = 128;     // query rows per forward workgroup (4 waves x 32 rows)
constexpr int kBwdBM = 128;     // query rows per dQ workgroup
constexpr int kBwdBN = 128;     // keys per dK/dV workgroup
constexpr int kThreads = 256;   // 4 wavefronts of 64 lanes
}  // namespace s2
