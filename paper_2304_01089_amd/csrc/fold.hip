// Offline folding of the reorder index (Sec. 4.2): LayerNorm parameters gathered into the
// padded cluster-order layout, weight columns permuted by the input reorder index (rows by
// the output reorder index when given), 4-bit Min-Max quantization per output channel
// (Eq. 1, Eq. 2 over the whole row), packing into the MFMA-fragment-major weight layout,
// and the per-cluster code sums the integer form of App. A.4 needs.
#include <hip/hip_runtime.h>

#include "device_common.h"
#include "pack_formats.h"
#include "rptq_internal.h"

namespace rptq {

// What the offline kernels report back: bit 0 = a weight is not finite, bit 1 = a row's Eq. 2
// scale is not a normal fp32 number.  One word per device; cleared and read by launch_fold.
__device__ int32_t g_fold_status;

__global__ void fold_status_clear_kernel() { g_fold_status = 0; }

__global__ void fold_ln_kernel(const float* gamma, const float* beta, const int32_t* perm_pad, int32_t k_padded,
                               float* gamma_pad, float* beta_pad) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= k_padded) return;
  const int c = perm_pad[j];
  gamma_pad[j] = c >= 0 ? gamma[c] : 0.0f;
  beta_pad[j] = c >= 0 ? beta[c] : 0.0f;
}

struct FoldArgs {
  const void* W;
  int32_t w_bf16;
  int32_t N;
  int32_t n_padded;
  int32_t has_perm_out;          // the caller's output index was uploaded into zW[0..N)
  const int32_t* perm_pad;
  uint8_t* Wq;
  float* sW;
  int32_t* zW;
  int32_t* wsum;
  float* colterm;
};

struct ScaleTab {
  double sz[RPTQ_MAX_CLUSTERS];     // sX_i * zX_i
};

__global__ void __launch_bounds__(256) fold_weight_kernel(FoldArgs a, ClusterGeom geom, ScaleTab tab) {
  __shared__ float red_min[4], red_max[4];
  __shared__ float sh_inv;
  __shared__ int32_t sh_z;
  __shared__ int32_t sh_wsum[RPTQ_MAX_CLUSTERS];
  const int o = blockIdx.x;
  const int tid = threadIdx.x;
  const int n_units = geom.k_padded / 8;

  if (o >= a.N) {                                  // rows added by rounding N up: all-zero codes
    for (int u = tid; u < n_units; u += blockDim.x)
      *reinterpret_cast<uint32_t*>(a.Wq + weight_dword_offset(o, u, geom.k_padded)) = 0u;
    return;
  }
  // (zW[o] carries the validated source row of output o until this workgroup overwrites it with
  // the row's zero point: every thread reads it here, thread 0 writes behind a barrier)
  const int64_t src_row = a.has_perm_out ? a.zW[o] : o;
  if (src_row < 0) {                               // a pad row of the output layout: weights 0, s = 1, z = 0
    for (int u = tid; u < n_units; u += blockDim.x)
      *reinterpret_cast<uint32_t*>(a.Wq + weight_dword_offset(o, u, geom.k_padded)) = 0u;
    if (tid < geom.g) a.wsum[static_cast<int64_t>(o) * geom.g + tid] = 0;
    __syncthreads();
    if (tid == 0) {
      a.sW[o] = 1.0f;
      a.zW[o] = 0;
      a.colterm[o] = 0.0f;
    }
    return;
  }
  const uint16_t* wb = static_cast<const uint16_t*>(a.W) + src_row * geom.k;
  const float* wf = static_cast<const float*>(a.W) + src_row * geom.k;
  auto wval = [&](int c) -> float { return a.w_bf16 ? __uint_as_float(static_cast<uint32_t>(wb[c]) << 16) : wf[c]; };

  // ---- Eq. 2 over the whole row ---------------------------------------------------------
  float lo = __builtin_huge_valf(), hi = -__builtin_huge_valf();
  bool bad = false;
  for (int c = tid; c < geom.k; c += blockDim.x) {
    const float w = wval(c);
    bad |= !(fabsf(w) <= 3.4028234664e38f);         // NaN or infinity (min/max would skip a NaN)
    lo = fminf(lo, w);
    hi = fmaxf(hi, w);
  }
  if (bad) atomicOr(&g_fold_status, 1);
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) {
    lo = fminf(lo, __shfl_xor(lo, m, kWave));
    hi = fmaxf(hi, __shfl_xor(hi, m, kWave));
  }
  if ((tid & 63) == 0) {
    red_min[tid >> 6] = lo;
    red_max[tid >> 6] = hi;
  }
  if (tid < geom.g) sh_wsum[tid] = 0;
  __syncthreads();
  if (tid == 0) {
    const double l = fminf(fminf(red_min[0], red_min[1]), fminf(red_min[2], red_min[3])) + 0.0f;
    const double h = fmaxf(fmaxf(red_max[0], red_max[1]), fmaxf(red_max[2], red_max[3])) + 0.0f;
    double s64, zz;
    if (h == l) {
      s64 = 1.0;
      zz = -rint(l);
    } else {
      s64 = (h - l) / 16.0;
      zz = -rint((h + l) / (2.0 * s64));
    }
    const float s32 = static_cast<float>(s64);
    if (!(s32 >= 1.17549435e-38f && s32 <= 3.4028234664e38f)) atomicOr(&g_fold_status, 2);
    sh_inv = static_cast<float>(1.0 / static_cast<double>(s32));
    sh_z = static_cast<int32_t>(zz);
    a.sW[o] = s32;
    a.zW[o] = sh_z;
  }
  __syncthreads();
  const float inv = sh_inv;
  const float zf = static_cast<float>(sh_z);

  // ---- Eq. 1 per weight, pack eight codes per dword ----------------------------------------
  for (int u = tid; u < n_units; u += blockDim.x) {
    int q[8];
    int sum = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int c = a.perm_pad[u * 8 + e];
      int code = 0;
      if (c >= 0) {
        const float r = __fmul_rn(wval(c), inv);
        float b = __fadd_rn(rintf(r), zf);
        b = fminf(fmaxf(b, -8.0f), 7.0f);
        code = static_cast<int>(b);
      }
      q[e] = code;
      sum += code;
    }
    uint32_t word = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) word |= static_cast<uint32_t>(((q[b] & 15) << 4) | (q[4 + b] & 15)) << (8 * b);
    *reinterpret_cast<uint32_t*>(a.Wq + weight_dword_offset(o, u, geom.k_padded)) = word;
    int ci = 0;
    for (int i = 1; i < geom.g; ++i) ci += (u * 8 >= geom.pad_off[i]) ? 1 : 0;
    atomicAdd(&sh_wsum[ci], sum);
  }
  __syncthreads();
  if (tid < geom.g) a.wsum[static_cast<int64_t>(o) * geom.g + tid] = sh_wsum[tid];
  if (tid == 0) {
    double acc = 0.0;
    for (int i = 0; i < geom.g; ++i) acc += tab.sz[i] * static_cast<double>(sh_wsum[i]);
    a.colterm[o] = static_cast<float>(acc);
  }
}


// ---- App. A.4 as printed: one Eq. 2 pair per (output channel, input cluster) ------------------
struct FoldCwArgs {
  const void* W;
  int32_t w_bf16;
  int32_t N;
  int32_t n_padded;
  int32_t has_perm_out;
  const int32_t* perm_pad;
  uint8_t* Wq;
  float* sW;            // [N, g]
  int32_t* zW;          // [N, g]; row o's first entry carries the source row until it is overwritten
  int32_t* wsum;        // [N, g]
  float* scale_tab;     // [g, n_padded]: sX_i * sW[o,i]
  float* cross_tab;     // [n_padded, g2], position of cluster i: (i & 1) * g2/2 + i/2; holds -sW[o,i] * zW[o,i]
  float* colterm;       // [N]: sum_i sX_i sW[o,i] zX_i wsum[o,i]
  int32_t g2;
};

struct ScaleTabCw {
  double sx[RPTQ_MAX_CLUSTERS];
  double zx[RPTQ_MAX_CLUSTERS];
};

__global__ void __launch_bounds__(256) fold_weight_cw_kernel(FoldCwArgs a, ClusterGeom geom, ScaleTabCw tab) {
  __shared__ uint32_t k_lo[RPTQ_MAX_CLUSTERS], k_hi[RPTQ_MAX_CLUSTERS];
  __shared__ float sh_inv[RPTQ_MAX_CLUSTERS], sh_s[RPTQ_MAX_CLUSTERS];
  __shared__ int32_t sh_z[RPTQ_MAX_CLUSTERS], sh_wsum[RPTQ_MAX_CLUSTERS];
  const int o = blockIdx.x;
  const int tid = threadIdx.x;
  const int n_units = geom.k_padded / 8;
  const int g = geom.g;

  for (int i = tid; i < a.g2; i += blockDim.x) a.cross_tab[static_cast<int64_t>(o) * a.g2 + i] = 0.0f;
  const int64_t src_row = (o < a.N) ? (a.has_perm_out ? a.zW[static_cast<int64_t>(o) * g] : o) : -1;
  if (src_row < 0) {                               // a pad row: weights 0, every scale 1, every zero point 0
    for (int u = tid; u < n_units; u += blockDim.x)
      *reinterpret_cast<uint32_t*>(a.Wq + weight_dword_offset(o, u, geom.k_padded)) = 0u;
    __syncthreads();
    if (tid < g) {
      a.scale_tab[static_cast<int64_t>(tid) * a.n_padded + o] = static_cast<float>(tab.sx[tid]);
      if (o < a.N) {
        a.wsum[static_cast<int64_t>(o) * g + tid] = 0;
        a.sW[static_cast<int64_t>(o) * g + tid] = 1.0f;
        a.zW[static_cast<int64_t>(o) * g + tid] = 0;
      }
    }
    if (tid == 0 && o < a.N) a.colterm[o] = 0.0f;
    return;
  }
  const uint16_t* wb = static_cast<const uint16_t*>(a.W) + src_row * geom.k;
  const float* wf = static_cast<const float*>(a.W) + src_row * geom.k;
  auto wval = [&](int c) -> float { return a.w_bf16 ? __uint_as_float(static_cast<uint32_t>(wb[c]) << 16) : wf[c]; };

  if (tid < g) {
    k_lo[tid] = 0xffffffffu;
    k_hi[tid] = 0u;
    sh_wsum[tid] = 0;
  }
  __syncthreads();
  // ---- minimum and maximum of every cluster block of the row (order-free: integer images of the floats)
  bool bad = false;
  for (int u = tid; u < n_units; u += blockDim.x) {
    int ci = 0;
    for (int i = 1; i < g; ++i) ci += (u * 8 >= geom.pad_off[i]) ? 1 : 0;
    float lo = __builtin_huge_valf(), hi = -__builtin_huge_valf();
    bool any = false;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int c = a.perm_pad[u * 8 + e];
      if (c >= 0) {
        const float w = wval(c);
        bad |= !(fabsf(w) <= 3.4028234664e38f);
        lo = fminf(lo, w);
        hi = fmaxf(hi, w);
        any = true;
      }
    }
    if (any) {
      atomicMin(&k_lo[ci], float_key(lo));
      atomicMax(&k_hi[ci], float_key(hi));
    }
  }
  if (bad) atomicOr(&g_fold_status, 1);
  __syncthreads();
  if (tid < g) {                                   // Eq. 2 for block (o, tid)
    const double l = key_float(k_lo[tid]) + 0.0f, h = key_float(k_hi[tid]) + 0.0f;
    double s64, zz;
    if (h == l) {
      s64 = 1.0;
      zz = -rint(l);
    } else {
      s64 = (h - l) / 16.0;
      zz = -rint((h + l) / (2.0 * s64));
    }
    const float s32 = static_cast<float>(s64);
    // (a block that lies far from zero relative to its width has a large zero point: at most
    // 8 * 2 * 2^24 for fp32 extrema that differ, so it always fits an int32)
    if (!(s32 >= 1.17549435e-38f && s32 <= 3.4028234664e38f) || !(fabs(zz) <= 1073741824.0)) atomicOr(&g_fold_status, 2);
    sh_s[tid] = s32;
    sh_inv[tid] = static_cast<float>(1.0 / static_cast<double>(s32));
    sh_z[tid] = static_cast<int32_t>(zz);
  }
  __syncthreads();
  // ---- Eq. 1 per weight with its block's pair, pack eight codes per dword
  for (int u = tid; u < n_units; u += blockDim.x) {
    int ci = 0;
    for (int i = 1; i < g; ++i) ci += (u * 8 >= geom.pad_off[i]) ? 1 : 0;
    const float inv = sh_inv[ci];
    const double zd = static_cast<double>(sh_z[ci]);
    int q[8];
    int sum = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int c = a.perm_pad[u * 8 + e];
      int code = 0;
      if (c >= 0) {
        const float r = __fmul_rn(wval(c), inv);           // one fp32 rounding, as everywhere
        double b = rint(static_cast<double>(r)) + zd;      // the zero point of a block may exceed fp32's exact integers
        b = fmin(fmax(b, -8.0), 7.0);
        code = static_cast<int>(b);
      }
      q[e] = code;
      sum += code;
    }
    uint32_t word = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) word |= static_cast<uint32_t>(((q[b] & 15) << 4) | (q[4 + b] & 15)) << (8 * b);
    *reinterpret_cast<uint32_t*>(a.Wq + weight_dword_offset(o, u, geom.k_padded)) = word;
    atomicAdd(&sh_wsum[ci], sum);
  }
  __syncthreads();
  if (tid < g) {
    const int64_t k = static_cast<int64_t>(o) * g + tid;
    a.wsum[k] = sh_wsum[tid];
    a.sW[k] = sh_s[tid];
    a.zW[k] = sh_z[tid];
    a.scale_tab[static_cast<int64_t>(tid) * a.n_padded + o] = static_cast<float>(tab.sx[tid] * static_cast<double>(sh_s[tid]));
    a.cross_tab[static_cast<int64_t>(o) * a.g2 + (tid & 1) * (a.g2 / 2) + (tid >> 1)] =
        static_cast<float>(-static_cast<double>(sh_s[tid]) * static_cast<double>(sh_z[tid]));
  }
  if (tid == 0) {
    double acc = 0.0;
    for (int i = 0; i < g; ++i)
      acc += tab.sx[i] * static_cast<double>(sh_s[i]) * tab.zx[i] * static_cast<double>(sh_wsum[i]);
    a.colterm[o] = static_cast<float>(acc);
  }
}

__global__ void unpack_weights_kernel(const uint8_t* Wq, int N, ClusterGeom geom, int8_t* out) {
  const int o = blockIdx.x;
  if (o >= N) return;
  for (int j = threadIdx.x; j < geom.k; j += blockDim.x) {
    int ci = 0;
    for (int i = 1; i < geom.g; ++i) ci += (j >= geom.off[i]) ? 1 : 0;
    const int pos = geom.pad_off[ci] + (j - geom.off[ci]);
    const int u = pos >> 3, e = pos & 7;
    const uint8_t byte = Wq[weight_dword_offset(o, u, geom.k_padded) + (e & 3)];
    const int nib = (e < 4) ? (byte >> 4) : (byte & 15);
    out[static_cast<int64_t>(o) * geom.k + j] = static_cast<int8_t>((nib ^ 8) - 8);
  }
}

int32_t launch_fold(const float* gamma, const float* beta, const int32_t* perm_pad_host, const ClusterGeom& geom,
                    const float* sX, const int32_t* zX, const void* W, int32_t w_dtype, int32_t N,
                    const int32_t* perm_out_host, int32_t* perm_pad, float* gamma_pad, float* beta_pad,
                    void* Wq_packed, float* sW, int32_t* zW, int32_t* wsum, float* colterm, hipStream_t st) {
  // the index arrays were validated on the host; they are uploaded from there, so what the
  // kernels read is what was checked
  RPTQ_HIP(hipMemcpyAsync(perm_pad, perm_pad_host, sizeof(int32_t) * geom.k_padded, hipMemcpyHostToDevice, st));
  if (gamma) {
    hipLaunchKernelGGL(fold_ln_kernel, dim3((geom.k_padded + 255) / 256), dim3(256), 0, st, gamma, beta, perm_pad,
                       geom.k_padded, gamma_pad, beta_pad);
    RPTQ_HIP(hipGetLastError());
  }
  if (!W) {
    RPTQ_HIP(hipStreamSynchronize(st));            // perm_pad_host belongs to the caller's frame
    return RPTQ_OK;
  }
  if (perm_out_host) RPTQ_HIP(hipMemcpyAsync(zW, perm_out_host, sizeof(int32_t) * N, hipMemcpyHostToDevice, st));
  FoldArgs a;
  a.W = W;
  a.w_bf16 = (w_dtype == RPTQ_DTYPE_BF16);
  a.N = N;
  a.n_padded = (N + RPTQ_N_ALIGN - 1) / RPTQ_N_ALIGN * RPTQ_N_ALIGN;
  a.has_perm_out = perm_out_host != nullptr;
  a.perm_pad = perm_pad;
  a.Wq = static_cast<uint8_t*>(Wq_packed);
  a.sW = sW;
  a.zW = zW;
  a.wsum = wsum;
  a.colterm = colterm;
  ScaleTab tab;
  for (int i = 0; i < RPTQ_MAX_CLUSTERS; ++i)
    tab.sz[i] = i < geom.g ? static_cast<double>(sX[i]) * static_cast<double>(zX[i]) : 0.0;
  hipLaunchKernelGGL(fold_status_clear_kernel, dim3(1), dim3(1), 0, st);
  RPTQ_HIP(hipGetLastError());
  hipLaunchKernelGGL(fold_weight_kernel, dim3(a.n_padded), dim3(256), 0, st, a, geom, tab);
  RPTQ_HIP(hipGetLastError());
  int32_t status = 0;
  RPTQ_HIP(hipMemcpyFromSymbolAsync(&status, HIP_SYMBOL(g_fold_status), sizeof(status), 0, hipMemcpyDeviceToHost, st));
  RPTQ_HIP(hipStreamSynchronize(st));
  return status ? RPTQ_ERR_RANGE : RPTQ_OK;
}


int32_t launch_fold_cw(const int32_t* perm_pad_host, const ClusterGeom& geom, const float* sX, const int32_t* zX,
                       const void* W, int32_t w_dtype, int32_t N, const int32_t* perm_out_host, int32_t* perm_pad,
                       void* Wq_packed, float* sW, int32_t* zW, int32_t* wsum, float* scale_tab, float* cross_tab,
                       float* colterm, hipStream_t st) {
  RPTQ_HIP(hipMemcpyAsync(perm_pad, perm_pad_host, sizeof(int32_t) * geom.k_padded, hipMemcpyHostToDevice, st));
  // the validated source rows travel in the first zero-point entry of every output row
  if (perm_out_host)
    RPTQ_HIP(hipMemcpy2DAsync(zW, sizeof(int32_t) * geom.g, perm_out_host, sizeof(int32_t), sizeof(int32_t), N,
                              hipMemcpyHostToDevice, st));
  FoldCwArgs a;
  a.W = W;
  a.w_bf16 = (w_dtype == RPTQ_DTYPE_BF16);
  a.N = N;
  a.n_padded = (N + RPTQ_N_ALIGN - 1) / RPTQ_N_ALIGN * RPTQ_N_ALIGN;
  a.has_perm_out = perm_out_host != nullptr;
  a.perm_pad = perm_pad;
  a.Wq = static_cast<uint8_t*>(Wq_packed);
  a.sW = sW;
  a.zW = zW;
  a.wsum = wsum;
  a.scale_tab = scale_tab;
  a.cross_tab = cross_tab;
  a.colterm = colterm;
  a.g2 = geom.g <= 32 ? 32 : 64;
  ScaleTabCw tab;
  for (int i = 0; i < RPTQ_MAX_CLUSTERS; ++i) {
    tab.sx[i] = i < geom.g ? static_cast<double>(sX[i]) : 0.0;
    tab.zx[i] = i < geom.g ? static_cast<double>(zX[i]) : 0.0;
  }
  hipLaunchKernelGGL(fold_status_clear_kernel, dim3(1), dim3(1), 0, st);
  RPTQ_HIP(hipGetLastError());
  hipLaunchKernelGGL(fold_weight_cw_kernel, dim3(a.n_padded), dim3(256), 0, st, a, geom, tab);
  RPTQ_HIP(hipGetLastError());
  int32_t status = 0;
  RPTQ_HIP(hipMemcpyFromSymbolAsync(&status, HIP_SYMBOL(g_fold_status), sizeof(status), 0, hipMemcpyDeviceToHost, st));
  RPTQ_HIP(hipStreamSynchronize(st));
  return status ? RPTQ_ERR_RANGE : RPTQ_OK;
}

int32_t launch_unpack_weights(const void* Wq, int32_t N, const ClusterGeom& geom, int8_t* out, hipStream_t st) {
  hipLaunchKernelGGL(unpack_weights_kernel, dim3(N), dim3(256), 0, st, static_cast<const uint8_t*>(Wq), N, geom, out);
  RPTQ_HIP(hipGetLastError());
  return RPTQ_OK;
}

}  // namespace rptq
