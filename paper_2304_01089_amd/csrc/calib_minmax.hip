// Per-channel minimum / maximum of a site's activation over calibration rows
// (Sec. 4.1, first displayed equation).  The activation is LayerNorm(x) computed with the
// same arithmetic as the online kernel (fp64 row sums, fp32 elementwise chain), or x
// itself at a non-LayerNorm site, optionally through max(.,0).
//
// Each thread owns up to 4 chunks of 8 channels for all rows of its workgroup and keeps
// running extrema in registers; workgroups merge through atomic min/max on an
// order-preserving integer image of the floats, so the result does not depend on order.
#include <hip/hip_runtime.h>

#include "device_common.h"
#include "rptq_internal.h"

namespace rptq {

constexpr int kCalChunk = 4;

__global__ void minmax_init_kernel(uint32_t* keys, int d) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < d) {
    keys[i] = 0xffffffffu;        // running minimum (as key)
    keys[d + i] = 0u;             // running maximum (as key)
  }
}

__global__ void minmax_final_kernel(const uint32_t* keys, int d, float* ch_min, float* ch_max) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < d) {
    ch_min[i] = key_float(keys[i]) + 0.0f;        // -0.0 -> +0.0
    ch_max[i] = key_float(keys[d + i]) + 0.0f;
  }
}

template <bool LN>
__global__ void __launch_bounds__(1024) minmax_kernel(const uint4* x, int64_t rows, int d, const float* gamma,
                                                      const float* beta, float eps, int relu, uint32_t* keys) {
  __shared__ double red[2][2][kMaxWaves];
  const int tid = threadIdx.x, T = blockDim.x, lane = tid & 63, wid = tid >> 6, nw = T >> 6;
  const int chunks = d / 8;

  float vmin[kCalChunk][8], vmax[kCalChunk][8];
#pragma unroll
  for (int c = 0; c < kCalChunk; ++c) {
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      vmin[c][k] = __builtin_huge_valf();
      vmax[c][k] = -__builtin_huge_valf();
    }
  }

  int parity = 0;
  for (int64_t row = blockIdx.x; row < rows; row += gridDim.x, parity ^= 1) {
    uint4 v[kCalChunk];
    double s1 = 0.0, s2 = 0.0;
#pragma unroll
    for (int c = 0; c < kCalChunk; ++c) {
      const int idx = tid + c * T;
      if (idx < chunks) {
        v[c] = x[row * chunks + idx];
        if (LN) {
          const uint32_t w[4] = {v[c].x, v[c].y, v[c].z, v[c].w};
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
#pragma unroll
    for (int c = 0; c < kCalChunk; ++c) {
      const int idx = tid + c * T;
      if (idx < chunks) {
        const uint32_t w[4] = {v[c].x, v[c].y, v[c].z, v[c].w};
        float gam[8], bet[8];
        if (LN) {
          // not kept in registers: calibration runs once, the extrema need the space
          const float4 g0 = *reinterpret_cast<const float4*>(gamma + idx * 8), g1 = *reinterpret_cast<const float4*>(gamma + idx * 8 + 4);
          const float4 b0 = *reinterpret_cast<const float4*>(beta + idx * 8), b1 = *reinterpret_cast<const float4*>(beta + idx * 8 + 4);
          gam[0] = g0.x; gam[1] = g0.y; gam[2] = g0.z; gam[3] = g0.w; gam[4] = g1.x; gam[5] = g1.y; gam[6] = g1.z; gam[7] = g1.w;
          bet[0] = b0.x; bet[1] = b0.y; bet[2] = b0.z; bet[3] = b0.w; bet[4] = b1.x; bet[5] = b1.y; bet[6] = b1.z; bet[7] = b1.w;
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          float y = (k & 1) ? bf16_hi(w[k / 2]) : bf16_lo(w[k / 2]);
          if (LN) y = ln_chain(y, mu, rstd, gam[k], bet[k]);
          if (relu) y = fmaxf(y, 0.0f);
          vmin[c][k] = fminf(vmin[c][k], y);
          vmax[c][k] = fmaxf(vmax[c][k], y);
        }
      }
    }
  }

  if (static_cast<int64_t>(blockIdx.x) < rows) {
#pragma unroll
    for (int c = 0; c < kCalChunk; ++c) {
      const int idx = tid + c * T;
      if (idx < chunks) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          atomicMin(&keys[idx * 8 + k], float_key(vmin[c][k]));
          atomicMax(&keys[d + idx * 8 + k], float_key(vmax[c][k]));
        }
      }
    }
  }
}

int32_t launch_channel_minmax(const void* const* x_batches, const int64_t* rows, int32_t n_batches, int32_t d,
                              const float* gamma, const float* beta, float eps, int32_t relu,
                              float* ch_min_dev, float* ch_max_dev, uint32_t* keys, hipStream_t st) {
  const int chunks = d / 8;
  int threads = ((chunks + kCalChunk - 1) / kCalChunk + kWave - 1) / kWave * kWave;
  if (threads < 256) threads = std::min(256, (chunks + kWave - 1) / kWave * kWave);
  if (threads > 1024) return RPTQ_ERR_SHAPE;
  hipLaunchKernelGGL(minmax_init_kernel, dim3((d + 255) / 256), dim3(256), 0, st, keys, d);
  RPTQ_HIP(hipGetLastError());
  for (int b = 0; b < n_batches; ++b) {
    if (rows[b] == 0) continue;
    const int grid = static_cast<int>(std::min<int64_t>(rows[b], 512));
    const uint4* xb = static_cast<const uint4*>(x_batches[b]);
    if (gamma) {
      hipLaunchKernelGGL(minmax_kernel<true>, dim3(grid), dim3(threads), 0, st, xb, rows[b], d, gamma, beta, eps, relu, keys);
    } else {
      hipLaunchKernelGGL(minmax_kernel<false>, dim3(grid), dim3(threads), 0, st, xb, rows[b], d, gamma, beta, eps, relu, keys);
    }
    RPTQ_HIP(hipGetLastError());
  }
  hipLaunchKernelGGL(minmax_final_kernel, dim3((d + 255) / 256), dim3(256), 0, st, keys, d, ch_min_dev, ch_max_dev);
  RPTQ_HIP(hipGetLastError());
  return RPTQ_OK;
}

}  // namespace rptq
