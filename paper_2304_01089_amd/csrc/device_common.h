// Device helpers shared by the LayerNorm / quantization kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rptq {

constexpr int kWave = 64;
constexpr int kMaxWaves = 16;   // 1024 threads

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// ---- cross-lane sums on the DPP path (no LDS round trips) -------------------------------------
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_add(double v) {
  const uint32_t lo = static_cast<uint32_t>(__double_as_longlong(v));
  const uint32_t hi = static_cast<uint32_t>(__double_as_longlong(v) >> 32);
  // lanes outside ROW_MASK (or without a source) receive 0.0
  const uint32_t plo = __builtin_amdgcn_update_dpp(0u, lo, CTRL, ROW_MASK, 0xf, false);
  const uint32_t phi = __builtin_amdgcn_update_dpp(0u, hi, CTRL, ROW_MASK, 0xf, false);
  return v + __longlong_as_double(static_cast<long long>((static_cast<uint64_t>(phi) << 32) | plo));
}

// Sum over the 16 lanes of each DPP row; every lane of the row ends with the row's sum.
__device__ __forceinline__ double row16_sum(double v) {
  v = dpp_add<0xB1, 0xf>(v);     // quad_perm [1,0,3,2]
  v = dpp_add<0x4E, 0xf>(v);     // quad_perm [2,3,0,1]
  v = dpp_add<0x141, 0xf>(v);    // row_half_mirror
  v = dpp_add<0x140, 0xf>(v);    // row_mirror
  return v;
}

__device__ __forceinline__ double read_lane(double v, int lane) {
  const uint32_t lo = __builtin_amdgcn_readlane(static_cast<uint32_t>(__double_as_longlong(v)), lane);
  const uint32_t hi = __builtin_amdgcn_readlane(static_cast<uint32_t>(__double_as_longlong(v) >> 32), lane);
  return __longlong_as_double(static_cast<long long>((static_cast<uint64_t>(hi) << 32) | lo));
}

// Sum over the 64 lanes of the wave in a fixed order; the result is wave-uniform.
__device__ __forceinline__ double wave_sum(double v) {
  v = row16_sum(v);
  v = dpp_add<0x142, 0xa>(v);    // row_bcast15 into rows 1 and 3
  v = dpp_add<0x143, 0xc>(v);    // row_bcast31 into rows 2 and 3
  return read_lane(v, 63);
}

// Sum of per-wave partials p[0..nw) (nw <= 16) held in LDS, same order in every wave.
__device__ __forceinline__ double partials_sum(const double* p, int nw, int lane) {
  double v = (lane < nw) ? p[lane] : 0.0;
  v = row16_sum(v);
  return read_lane(v, 0);
}

// Row statistics of LayerNorm from exact fp64 sums of the bf16 inputs:
// mean = S1/d, var = (S2 - S1*mean)/d (biased), rstd = 1/sqrt(var+eps); both rounded once to fp32.
// The fp64 values are formed with a reciprocal of d and a Newton-refined reciprocal square root
// (a short dependent chain); they differ from the divide/sqrt forms by a few units in the last
// fp64 place, far inside the margin at which a row counts as having a fragile fp32 rounding.
__device__ __forceinline__ void row_stats(double s1, double s2, int d, float eps, float* mu32, float* rstd32) {
  const double inv_d = 1.0 / static_cast<double>(d);            // (uniform; hoisted out of row loops)
  const double mu = s1 * inv_d;
  double var = fma(-s1, mu, s2) * inv_d;
  var = var < 0.0 ? 0.0 : var;
  const double x = var + static_cast<double>(eps);
  double y = __builtin_amdgcn_rsq(x);                           // about 2^-26 relative
  y = y * fma(-0.5 * x * y, y, 1.5);                           // error about 1.5 e^2: 2^-51 after one step
  y = y * fma(-0.5 * x * y, y, 1.5);
  *mu32 = static_cast<float>(mu);
  *rstd32 = static_cast<float>(y);
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
