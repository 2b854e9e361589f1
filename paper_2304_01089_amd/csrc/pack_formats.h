// Decoders of the packed 32-code group formats documented in the public header (gfx950 device code).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rptq {

// Byte offset of the dword holding padded columns 8u..8u+7 of output row o.
__device__ __host__ __forceinline__ size_t weight_dword_offset(int o, int u, int k_padded) {
  const int rb = o >> 5, r = o & 31;
  const int kb = u >> 4, s = (u >> 2) & 3, k8 = u & 3, h = k8 >> 1, v = k8 & 1;
  // block [rb][kb] of 2 KiB = two halves of 1 KiB (slices 0,1 | 2,3), each: 64 lanes x 16 bytes
  return ((static_cast<size_t>(rb) * (k_padded / 128) + kb) * 2 + (s >> 1)) * 1024 +
         static_cast<size_t>(h * 32 + r) * 16 + (s & 1) * 8 + v * 4;
}


// 32 packed codes -> 32 signed integers, natural order (the formats of the public header).
template <int BITS>
__device__ __forceinline__ void decode_group(const uint32_t* w, int* q) {
  if constexpr (BITS == 8) {
#pragma unroll
    for (int j = 0; j < 32; ++j) q[j] = static_cast<int>(w[j / 4] << (24 - 8 * (j & 3))) >> 24;
  } else if constexpr (BITS == 4) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        q[8 * u + b] = static_cast<int>(w[u] << (24 - 8 * b)) >> 28;          // high nibble of byte b
        q[8 * u + 4 + b] = static_cast<int>(w[u] << (28 - 8 * b)) >> 28;      // low nibble
      }
  } else {
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int sh = 24 - 8 * b;
      q[b] = static_cast<int>(w[0] << sh) >> 29;
      q[4 + b] = static_cast<int>(w[0] << (sh + 3)) >> 29;
      q[8 + b] = static_cast<int>(w[1] << sh) >> 29;
      q[12 + b] = static_cast<int>(w[1] << (sh + 3)) >> 29;
      q[16 + b] = static_cast<int>(w[2] << sh) >> 29;
      q[20 + b] = static_cast<int>(w[2] << (sh + 3)) >> 29;
      const uint32_t t0 = (w[0] >> (8 * b)) & 3u, t1 = (w[1] >> (8 * b)) & 3u, lo = (w[2] >> (8 * b)) & 3u;
      q[24 + b] = static_cast<int>(((t0 << 1) | (lo & 1u)) << 29) >> 29;
      q[28 + b] = static_cast<int>(((t1 << 1) | (lo >> 1)) << 29) >> 29;
    }
  }
}

}  // namespace rptq
