// Device helpers shared by the LayerNorm / quantization kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rptq {

constexpr int kWave = 64;
constexpr int kMaxWaves = 16;   // 1024 threads

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
  return v;
}

// Row statistics of LayerNorm from exact fp64 sums of the bf16 inputs:
// mean = S1/d, var = (S2 - S1*S1/d)/d (biased), rstd = 1/sqrt(var+eps); both rounded once to fp32.
__device__ __forceinline__ void row_stats(double s1, double s2, int d, float eps, float* mu32, float* rstd32) {
  const double dd = static_cast<double>(d);
  const double mu = s1 / dd;
  double var = (s2 - s1 * mu) / dd;
  var = var < 0.0 ? 0.0 : var;
  const double rstd = 1.0 / sqrt(var + static_cast<double>(eps));
  *mu32 = static_cast<float>(mu);
  *rstd32 = static_cast<float>(rstd);
}

// The four separately rounded fp32 operations of the LayerNorm chain (no contraction).
__device__ __forceinline__ float ln_chain(float x, float mu, float rstd, float gamma, float beta) {
  const float t = __fsub_rn(x, mu);
  const float u = __fmul_rn(t, rstd);
  const float v = __fmul_rn(u, gamma);
  return __fadd_rn(v, beta);
}

// Order-preserving map between fp32 and uint32 (for atomic min/max on floats).
__device__ __forceinline__ uint32_t float_key(float f) {
  const uint32_t b = __float_as_uint(f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_float(uint32_t k) {
  const uint32_t b = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
  return __uint_as_float(b);
}

}  // namespace rptq
