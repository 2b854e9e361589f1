// The reorder fused into LayerNorm the way Sec. 4.2 ("Avoid explicit reordering") words it:
// LayerNorm runs over the row in its original channel order, gamma and beta untouched, and
// every result is written to the address its reorder index gives it.  A scattered write has
// no unit smaller than a byte, so the codes leave as one int8 each into an [M, K_p] buffer in
// padded cluster order, and a second kernel packs them into the 3/4/8-bit formats.
//
// This is the comparison variant of rptq_ln_quant (which gathers through LDS and stores
// packed codes once): same arithmetic, bit-identical codes, measured beside it.
#include <hip/hip_runtime.h>

#include "device_common.h"
#include "rptq_internal.h"

namespace rptq {

// dst[c] = padded position of original channel c (the inverse of perm_pad)
__global__ void invert_perm_pad_kernel(const int32_t* perm_pad, int32_t k_padded, int32_t* dst) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= k_padded) return;
  const int c = perm_pad[j];
  if (c >= 0) dst[c] = j;
}

// kScChunk: 16-byte chunks of the input row per thread (4 up to 16384 channels, 8 beyond); at most
// 512 threads, so that a thread's constants fit the register file
template <bool LN, int kScChunk>
__global__ void __launch_bounds__(512) ln_scatter_kernel(const uint4* x, int64_t M, int32_t d, const float* gamma,
                                                          const float* beta, float eps, int32_t relu, const int32_t* dst,
                                                          ClusterGeom geom, QuantTab qt, int32_t qmin, int8_t* out) {
  __shared__ double red[2][2][kMaxWaves];
  __shared__ float t_inv[RPTQ_MAX_CLUSTERS], t_zb[RPTQ_MAX_CLUSTERS];
  const int tid = threadIdx.x, T = blockDim.x, lane = tid & 63, wid = tid >> 6, nw = T >> 6;
  const int chunks = d / 8;
  const float umax = static_cast<float>(-2 * qmin - 1);
  const float relu_floor = relu ? 0.0f : -__builtin_huge_valf();
  if (tid < RPTQ_MAX_CLUSTERS) {
    t_inv[tid] = qt.inv_s[tid];
    t_zb[tid] = static_cast<float>(qt.zb[tid]);
  }
  // a thread owns the same channels in every row: destination and cluster of each, once
  uint32_t where[kScChunk][8];                           // padded position | cluster << 24
#pragma unroll
  for (int c = 0; c < kScChunk; ++c) {
    const int idx = tid + c * T;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int pos = idx < chunks ? dst[idx * 8 + k] : 0;
      int ci = 0;
      for (int i = 1; i < geom.g; ++i) ci += (pos >= geom.pad_off[i]) ? 1 : 0;
      where[c][k] = static_cast<uint32_t>(pos) | (static_cast<uint32_t>(ci) << 24);
    }
  }
  __syncthreads();
  int parity = 0;
  for (int64_t row = blockIdx.x; row < M; row += gridDim.x, parity ^= 1) {
    uint4 v[kScChunk];
    double s1 = 0.0, s2 = 0.0;
#pragma unroll
    for (int c = 0; c < kScChunk; ++c) {
      // (no load under a lane-dependent branch: surplus lanes read a valid chunk again and add zeros)
      const int idx = tid + c * T;
      const bool ok = idx < chunks;
      v[c] = x[row * chunks + (ok ? idx : chunks - 1)];
      if (LN) {
        const uint32_t w[4] = {ok ? v[c].x : 0u, ok ? v[c].y : 0u, ok ? v[c].z : 0u, ok ? v[c].w : 0u};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const double lo = static_cast<double>(bf16_lo(w[k]));
          const double hi = static_cast<double>(bf16_hi(w[k]));
          s1 += lo;
          s2 = fma(lo, lo, s2);
          s1 += hi;
          s2 = fma(hi, hi, s2);
        }
      }
    }
    float mu = 0.0f, rstd = 1.0f;
    if (LN) {
      const double r1 = wave_sum(s1), r2 = wave_sum(s2);
      if (lane == 0) {
        red[parity][0][wid] = r1;
        red[parity][1][wid] = r2;
      }
      __syncthreads();
      const double t1 = partials_sum(red[parity][0], nw, lane);
      const double t2 = partials_sum(red[parity][1], nw, lane);
      row_stats(t1, t2, d, eps, &mu, &rstd);
    }
    int8_t* orow = out + row * geom.k_padded;
#pragma unroll
    for (int c = 0; c < kScChunk; ++c) {
      const int idx = tid + c * T;
      if (idx < chunks) {
        const uint32_t w[4] = {v[c].x, v[c].y, v[c].z, v[c].w};
        float gam[8], bet[8];
        if (LN) {                                          // gamma and beta stay in their original order
          const float4 g0 = *reinterpret_cast<const float4*>(gamma + idx * 8), g1 = *reinterpret_cast<const float4*>(gamma + idx * 8 + 4);
          const float4 b0 = *reinterpret_cast<const float4*>(beta + idx * 8), b1 = *reinterpret_cast<const float4*>(beta + idx * 8 + 4);
          gam[0] = g0.x; gam[1] = g0.y; gam[2] = g0.z; gam[3] = g0.w; gam[4] = g1.x; gam[5] = g1.y; gam[6] = g1.z; gam[7] = g1.w;
          bet[0] = b0.x; bet[1] = b0.y; bet[2] = b0.z; bet[3] = b0.w; bet[4] = b1.x; bet[5] = b1.y; bet[6] = b1.z; bet[7] = b1.w;
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const uint32_t wh = where[c][k];
          const int pos = static_cast<int>(wh & 0xffffffu), ci = static_cast<int>(wh >> 24);
          float y = (k & 1) ? bf16_hi(w[k / 2]) : bf16_lo(w[k / 2]);
          if (LN) y = ln_chain(y, mu, rstd, gam[k], bet[k]);
          y = fmaxf(y, relu_floor);
          const float r = __fmul_rn(y, t_inv[ci]);
          float b = __fadd_rn(rintf(r), t_zb[ci]);
          b = fminf(fmaxf(b, 0.0f), umax);
          orow[pos] = static_cast<int8_t>(static_cast<int>(b) + qmin);      // the reorder index offsets the write address
        }
      }
    }
  }
}

// int8 codes in padded cluster order -> the packed group formats (pad positions: code 0)
template <int BITS>
__global__ void __launch_bounds__(256) pack_codes_kernel(const int8_t* in, int64_t M, int32_t k_padded,
                                                         const int32_t* perm_pad, uint8_t* codes) {
  const int groups = k_padded / kGroup;
  const int64_t total = M * groups;
  for (int64_t gid = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; gid < total;
       gid += static_cast<int64_t>(gridDim.x) * blockDim.x) {
    const int64_t row = gid / groups;
    const int gi = static_cast<int>(gid % groups);
    const int8_t* src = in + row * k_padded + gi * kGroup;
    int q[32];
#pragma unroll
    for (int k4 = 0; k4 < 2; ++k4) {
      const uint4 v = reinterpret_cast<const uint4*>(src)[k4];
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int j = 0; j < 16; ++j) q[k4 * 16 + j] = static_cast<int8_t>(w[j / 4] >> (8 * (j & 3)));
    }
#pragma unroll
    for (int j = 0; j < 32; ++j)
      if (perm_pad[gi * kGroup + j] < 0) q[j] = 0;
    uint8_t* dstp = codes + (row * groups + gi) * (BITS * 4);
    if (BITS == 8) {
      uint32_t o[8];
#pragma unroll
      for (int j = 0; j < 32; ++j) {
        if ((j & 3) == 0) o[j / 4] = 0;
        o[j / 4] |= static_cast<uint32_t>(q[j] & 0xff) << (8 * (j & 3));
      }
      reinterpret_cast<uint4*>(dstp)[0] = make_uint4(o[0], o[1], o[2], o[3]);
      reinterpret_cast<uint4*>(dstp)[1] = make_uint4(o[4], o[5], o[6], o[7]);
    } else if (BITS == 4) {
      uint32_t o[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        o[u] = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) o[u] |= static_cast<uint32_t>(((q[8 * u + b] & 15) << 4) | (q[8 * u + 4 + b] & 15)) << (8 * b);
      }
      *reinterpret_cast<uint4*>(dstp) = make_uint4(o[0], o[1], o[2], o[3]);
    } else {
      uint32_t x0 = 0, x1 = 0, x2 = 0;
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const uint32_t f0 = q[b] & 7, f4 = q[4 + b] & 7, f8 = q[8 + b] & 7, f12 = q[12 + b] & 7, f16 = q[16 + b] & 7,
                       f20 = q[20 + b] & 7, f24 = q[24 + b] & 7, f28 = q[28 + b] & 7;
        x0 |= ((f0 << 5) | (f4 << 2) | (f24 >> 1)) << (8 * b);
        x1 |= ((f8 << 5) | (f12 << 2) | (f28 >> 1)) << (8 * b);
        x2 |= ((f16 << 5) | (f20 << 2) | ((f28 & 1) << 1) | (f24 & 1)) << (8 * b);
      }
      uint32_t* p = reinterpret_cast<uint32_t*>(dstp);
      p[0] = x0; p[1] = x1; p[2] = x2;
    }
  }
}

size_t ln_scatter_workspace_bytes(int64_t M, int32_t d, int32_t k_padded) {
  const size_t inv = (static_cast<size_t>(d) * sizeof(int32_t) + 255) / 256 * 256;
  return inv + static_cast<size_t>(M) * static_cast<size_t>(k_padded);
}

int32_t launch_ln_scatter(const void* x, int64_t M, int32_t d, const float* gamma, const float* beta, float eps,
                          int32_t relu, const int32_t* perm_pad, const ClusterGeom& geom, const QuantTab& qt, int32_t bits,
                          void* codes, void* workspace, hipStream_t st) {
  if (M == 0) return RPTQ_OK;
  int32_t* dst = static_cast<int32_t*>(workspace);
  int8_t* bytes = reinterpret_cast<int8_t*>(static_cast<unsigned char*>(workspace) +
                                           (static_cast<size_t>(d) * sizeof(int32_t) + 255) / 256 * 256);
  hipLaunchKernelGGL(invert_perm_pad_kernel, dim3((geom.k_padded + 255) / 256), dim3(256), 0, st, perm_pad, geom.k_padded, dst);
  RPTQ_HIP(hipGetLastError());
  const int chunks = d / 8;
  const int per_thread = chunks <= 512 * 4 ? 4 : 8;
  int threads = ((chunks + per_thread - 1) / per_thread + kWave - 1) / kWave * kWave;
  if (threads < 256) threads = std::min(256, (chunks + kWave - 1) / kWave * kWave);
  if (threads > 512) return RPTQ_ERR_SHAPE;
  int cus = 0;
  if (int32_t s = device_compute_units(st, &cus)) return s;
  const int grid = static_cast<int>(std::min<int64_t>(M, static_cast<int64_t>(cus) * 2));
  const int qmin = -(1 << (bits - 1));
  const uint4* xp = static_cast<const uint4*>(x);
  if (gamma && per_thread == 4) hipLaunchKernelGGL((ln_scatter_kernel<true, 4>), dim3(grid), dim3(threads), 0, st, xp, M, d, gamma, beta, eps, relu, dst, geom, qt, qmin, bytes);
  else if (gamma) hipLaunchKernelGGL((ln_scatter_kernel<true, 8>), dim3(grid), dim3(threads), 0, st, xp, M, d, gamma, beta, eps, relu, dst, geom, qt, qmin, bytes);
  else if (per_thread == 4) hipLaunchKernelGGL((ln_scatter_kernel<false, 4>), dim3(grid), dim3(threads), 0, st, xp, M, d, gamma, beta, eps, relu, dst, geom, qt, qmin, bytes);
  else hipLaunchKernelGGL((ln_scatter_kernel<false, 8>), dim3(grid), dim3(threads), 0, st, xp, M, d, gamma, beta, eps, relu, dst, geom, qt, qmin, bytes);
  RPTQ_HIP(hipGetLastError());
  const int64_t total = M * (geom.k_padded / kGroup);
  const int pgrid = static_cast<int>(std::min<int64_t>((total + 255) / 256, static_cast<int64_t>(cus) * 16));
  uint8_t* cp = static_cast<uint8_t*>(codes);
  if (bits == 3) hipLaunchKernelGGL(pack_codes_kernel<3>, dim3(pgrid), dim3(256), 0, st, bytes, M, geom.k_padded, perm_pad, cp);
  else if (bits == 4) hipLaunchKernelGGL(pack_codes_kernel<4>, dim3(pgrid), dim3(256), 0, st, bytes, M, geom.k_padded, perm_pad, cp);
  else hipLaunchKernelGGL(pack_codes_kernel<8>, dim3(pgrid), dim3(256), 0, st, bytes, M, geom.k_padded, perm_pad, cp);
  RPTQ_HIP(hipGetLastError());
  return RPTQ_OK;
}

}  // namespace rptq
