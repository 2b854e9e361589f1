// LayerNorm emitted in cluster order + per-cluster asymmetric quantization + bit packing
// (Sec. 4.2 "fuse the reorder into layer norm"; Eq. 1; App. A.4 first equation).
//
// One workgroup owns whole rows and walks them in a grid-stride loop.  Each thread owns
// the same output units (8 codes, or 16 for 3-bit) for every row, so everything that does
// not depend on the row - source channel, gamma', beta', the cluster's quantizer constants
// - is loaded once into registers.  Per row: coalesced 16-byte loads of the bf16 row,
// exact fp64 row sums, one workgroup reduction (one barrier), then a gather of the row
// through LDS in cluster order, the fp32 LayerNorm chain, round/offset/clamp, packing and
// a coalesced store.  The next row's loads are issued before the gather of the current one.
#include <hip/hip_runtime.h>

#include "device_common.h"
#include "rptq_internal.h"

namespace rptq {

struct LnQuantArgs {
  const uint4* x;          // bf16 [M, d], 8 values per uint4
  int64_t M;
  int32_t d;
  int32_t chunks;          // d / 8
  const float* gamma_pad;
  const float* beta_pad;
  float eps;
  int32_t relu;
  const int32_t* perm_pad;
  uint8_t* codes;
  float* rowterm;
  int32_t n_units;         // K_p / codes-per-unit
  int32_t row_bytes;       // K_p * bits / 8
};

constexpr int kMaxChunk = 4;   // 16-byte chunks of the input row per thread

template <int BITS>
struct Unit {
  static constexpr int kCodes = (BITS == 3) ? 16 : 8;
};

// Position inside its 32-group of local code e of a 3-bit unit with the given role.
// role 0 carries codes 0..7, 24..27, 16..19; role 1 carries 8..15, 28..31, 20..23.
__device__ __forceinline__ int pos3(int role, int e) {
  if (e < 8) return role * 8 + e;
  if (e < 12) return 24 + role * 4 + (e - 8);
  return 16 + role * 4 + (e - 12);
}

template <int BITS, int NUNIT, bool LN>
__global__ void __launch_bounds__(1024) ln_quant_kernel(LnQuantArgs a, ClusterGeom geom, QuantTab qt) {
  constexpr int UC = Unit<BITS>::kCodes;
  constexpr int ND = UC / 4;                       // dwords of biased code bytes per unit
  constexpr float kUMax = static_cast<float>((1 << BITS) - 1);
  constexpr int kQMin = -(1 << (BITS - 1));

  extern __shared__ __align__(16) unsigned char smem[];
  const int rowbuf_bytes = a.d * 2;
  double* red = reinterpret_cast<double*>(smem + 2 * rowbuf_bytes);      // [2][kMaxWaves][3]

  const int tid = threadIdx.x;
  const int T = blockDim.x;
  const int lane = tid & (kWave - 1);
  const int wid = tid >> 6;
  const int nw = T >> 6;

  // ---- per-thread constants, loaded once ---------------------------------------
  uint32_t src[NUNIT][UC / 2];       // LDS byte offsets of the source channels, two per register
  float gam[LN ? NUNIT : 1][LN ? UC : 1];
  float bet[LN ? NUNIT : 1][LN ? UC : 1];
  float inv_s[NUNIT], zbf[NUNIT];
  double sdq[NUNIT];                 // cluster scale, for the de-quantized row sum
  int32_t usum_fix[NUNIT];           // turns the sum of biased bytes into sum of (q - z) over real codes
  uint32_t keep[NUNIT][ND], fill[NUNIT][ND];
  bool has_pad[NUNIT];
  int64_t out_off[NUNIT];

#pragma unroll
  for (int n = 0; n < NUNIT; ++n) {
    const int u = tid + n * T;
    const bool valid = u < a.n_units;
    const int uu = valid ? u : 0;
    int gbase, role = 0;
    if (BITS == 3) {
      gbase = (uu >> 1) * kGroup;
      role = uu & 1;
      out_off[n] = static_cast<int64_t>(uu >> 1) * 12 + role * 4;
    } else {
      gbase = uu * 8;
      out_off[n] = static_cast<int64_t>(uu) * BITS;
    }
    if (!valid) out_off[n] = -1;
    int ci = 0;
    for (int i = 1; i < geom.g; ++i) ci += (gbase >= geom.pad_off[i]) ? 1 : 0;
    inv_s[n] = qt.inv_s[ci];
    zbf[n] = static_cast<float>(qt.zb[ci]);
    sdq[n] = static_cast<double>(qt.s[ci]);
    int n_real = 0;
    has_pad[n] = false;
#pragma unroll
    for (int w = 0; w < ND; ++w) { keep[n][w] = 0xffffffffu; fill[n][w] = 0u; }
#pragma unroll
    for (int e = 0; e < UC; ++e) {
      const int pos = (BITS == 3) ? gbase + pos3(role, e) : gbase + e;
      const int c = a.perm_pad[pos];
      const bool real = c >= 0;
      n_real += real ? 1 : 0;
      const uint32_t off = real ? static_cast<uint32_t>(c) * 2u : 0u;
      if (e & 1) src[n][e / 2] |= off << 16; else src[n][e / 2] = off;
      if (LN) {
        gam[n][e] = real ? a.gamma_pad[pos] : 0.0f;
        bet[n][e] = real ? a.beta_pad[pos] : 0.0f;
      }
      if (!real) {                               // pad position: force code 0 (biased byte = -qmin)
        has_pad[n] = true;
        keep[n][e / 4] &= ~(0xffu << (8 * (e & 3)));
        fill[n][e / 4] |= static_cast<uint32_t>(-kQMin) << (8 * (e & 3));
      }
    }
    usum_fix[n] = UC * kQMin - n_real * qt.z[ci];
  }

  // ---- row loop ------------------------------------------------------------------
  uint4 nxt[kMaxChunk];
  auto load_row = [&](int64_t row) {
    const uint4* p = a.x + row * a.chunks;
#pragma unroll
    for (int c = 0; c < kMaxChunk; ++c) {
      const int idx = tid + c * T;
      if (idx < a.chunks) nxt[c] = p[idx];
    }
  };

  int64_t row = blockIdx.x;
  if (row < a.M) load_row(row);
  int parity = 0;
  double rt_prev = 0.0;            // this thread's share of the previous row's de-quantized sum
  int64_t prev_row = -1;

  for (; row < a.M; row += gridDim.x, parity ^= 1) {
    unsigned char* rowbuf = smem + parity * rowbuf_bytes;
    double s1 = 0.0, s2 = 0.0;
#pragma unroll
    for (int c = 0; c < kMaxChunk; ++c) {
      const int idx = tid + c * T;
      if (idx < a.chunks) {
        const uint4 v = nxt[c];
        *reinterpret_cast<uint4*>(rowbuf + idx * 16) = v;
        if (LN) {
          const uint32_t w[4] = {v.x, v.y, v.z, v.w};
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
    const int64_t next_row = row + gridDim.x;
    if (next_row < a.M) load_row(next_row);

    // one reduction carries the row sums and the previous row's de-quantized sum
    double* slot = red + parity * (kMaxWaves * 3);        // [3][kMaxWaves]
    {
      const double r1 = wave_sum(s1), r2 = wave_sum(s2), r3 = wave_sum(rt_prev);
      if (lane == 0) {
        slot[0 * kMaxWaves + wid] = r1;
        slot[1 * kMaxWaves + wid] = r2;
        slot[2 * kMaxWaves + wid] = r3;
      }
    }
    __syncthreads();
    const double t1 = partials_sum(slot + 0 * kMaxWaves, nw, lane);
    const double t2 = partials_sum(slot + 1 * kMaxWaves, nw, lane);
    const double t3 = partials_sum(slot + 2 * kMaxWaves, nw, lane);
    if (tid == 0 && prev_row >= 0 && a.rowterm) a.rowterm[prev_row] = static_cast<float>(t3);
    float mu = 0.0f, rstd = 1.0f;
    if (LN) row_stats(t1, t2, a.d, a.eps, &mu, &rstd);

    // ---- gather in cluster order, normalize, quantize, pack ------------------------
    double rt = 0.0;
    uint8_t* out_row = a.codes + row * a.row_bytes;
#pragma unroll
    for (int n = 0; n < NUNIT; ++n) {
      if (out_off[n] < 0) continue;
      uint32_t D[ND];
#pragma unroll
      for (int w = 0; w < ND; ++w) D[w] = 0u;
#pragma unroll
      for (int e = 0; e < UC; ++e) {
        const uint32_t off = (e & 1) ? (src[n][e / 2] >> 16) : (src[n][e / 2] & 0xffffu);
        const uint32_t h = *reinterpret_cast<const uint16_t*>(rowbuf + off);
        float y = __uint_as_float(h << 16);
        if (LN) y = ln_chain(y, mu, rstd, gam[n][e], bet[n][e]);
        if (a.relu) y = fmaxf(y, 0.0f);
        const float r = __fmul_rn(y, inv_s[n]);
        float b = __fadd_rn(rintf(r), zbf[n]);          // round, then add the zero point (biased by -qmin)
        if (BITS < 8) b = fminf(b, kUMax);              // upper clamp; the conversion saturates at 0 and 255
        D[e / 4] = __builtin_amdgcn_cvt_pk_u8_f32(b, e & 3, D[e / 4]);
      }
      if (has_pad[n]) {
#pragma unroll
        for (int w = 0; w < ND; ++w) D[w] = (D[w] & keep[n][w]) | fill[n][w];
      }
      uint32_t usum = 0;
#pragma unroll
      for (int w = 0; w < ND; ++w) usum = __builtin_amdgcn_sad_u8(D[w], 0u, usum);
      rt += sdq[n] * static_cast<double>(static_cast<int32_t>(usum) + usum_fix[n]);

      if (BITS == 8) {
        uint2 o;
        o.x = D[0] ^ 0x80808080u;
        o.y = D[1] ^ 0x80808080u;
        *reinterpret_cast<uint2*>(out_row + out_off[n]) = o;
      } else if (BITS == 4) {
        *reinterpret_cast<uint32_t*>(out_row + out_off[n]) = ((D[0] << 4) | D[1]) ^ 0x88888888u;
      } else {
        // role 0 -> x0 and its half of x2; role 1 -> x1 and its half of x2 (partner = lane ^ 1)
        const uint32_t w1 = ((D[0] << 5) | (D[1] << 2) | ((D[2] >> 1) & 0x03030303u)) ^ 0x80808080u ^ 0x10101010u ^ 0x02020202u;
        const int role = tid & 1;
        const uint32_t mine = role ? (((D[3] << 2) ^ 0x10101010u) | ((D[2] & 0x01010101u) << 1))
                                   : (((D[3] << 5) ^ 0x80808080u) | (D[2] & 0x01010101u));
        const uint32_t other = __shfl_xor(mine, 1, kWave);
        if (role == 0) {
          *reinterpret_cast<uint32_t*>(out_row + out_off[n]) = w1;
        } else {
          uint32_t* p = reinterpret_cast<uint32_t*>(out_row + out_off[n]);
          p[0] = w1;
          p[1] = mine | other;
        }
      }
    }
    rt_prev = rt;
    prev_row = row;
  }

  // flush the last row's de-quantized sum
  if (prev_row >= 0 && a.rowterm) {
    double* slot = red + parity * (kMaxWaves * 3);
    const double r3 = wave_sum(rt_prev);
    if (lane == 0) slot[2 * kMaxWaves + wid] = r3;
    __syncthreads();
    const double t3 = partials_sum(slot + 2 * kMaxWaves, nw, lane);
    if (tid == 0) a.rowterm[prev_row] = static_cast<float>(t3);
  }
}

// Per-cluster sums of the packed codes (verification output of rptq_ln_quant).
template <int BITS>
__device__ __forceinline__ int code_at(const uint8_t* row, int pos) {
  const int grp = pos >> 5, j = pos & 31;
  if (BITS == 8) return static_cast<int8_t>(row[pos]);
  if (BITS == 4) {
    const uint8_t* g4 = row + grp * 16;
    const int u = j >> 3, b = j & 3, hi = ((j & 7) < 4);
    const uint8_t byte = g4[u * 4 + b];
    const int nib = hi ? (byte >> 4) : (byte & 15);
    return (nib ^ 8) - 8;
  }
  const uint8_t* g3 = row + grp * 12;
  const int b = j & 3;
  int f;
  if (j < 24) {
    const uint8_t byte = g3[(j >> 3) * 4 + b];
    f = ((j & 7) < 4) ? (byte >> 5) : ((byte >> 2) & 7);
  } else {
    const int which = (j - 24) >> 2;                       // 0: codes 24..27, 1: codes 28..31
    const int top = g3[which * 4 + b] & 3;
    const int low = (g3[8 + b] >> which) & 1;
    f = (top << 1) | low;
  }
  return (f ^ 4) - 4;
}

template <int BITS>
__global__ void xsum_kernel(const uint8_t* codes, int64_t M, int32_t row_bytes, ClusterGeom geom, int32_t* xsum) {
  const int64_t row = blockIdx.x;
  const int i = threadIdx.x;
  if (row >= M || i >= geom.g) return;
  const uint8_t* r = codes + row * row_bytes;
  int acc = 0;
  const int n = geom.off[i + 1] - geom.off[i];
  for (int j = 0; j < n; ++j) acc += code_at<BITS>(r, geom.pad_off[i] + j);
  xsum[row * geom.g + i] = acc;
}

template <int BITS>
__global__ void unpack_codes_kernel(const uint8_t* codes, int64_t rows, int32_t row_bytes, ClusterGeom geom, int8_t* out) {
  const int64_t row = blockIdx.x;
  if (row >= rows) return;
  const uint8_t* r = codes + row * row_bytes;
  for (int j = threadIdx.x; j < geom.k; j += blockDim.x) {
    int ci = 0;
    for (int i = 1; i < geom.g; ++i) ci += (j >= geom.off[i]) ? 1 : 0;
    out[row * geom.k + j] = static_cast<int8_t>(code_at<BITS>(r, geom.pad_off[ci] + (j - geom.off[ci])));
  }
}

// ---------------------------------------------------------------------------------------
template <int BITS, int NUNIT>
static int32_t launch_one(const LnQuantArgs& a, const ClusterGeom& geom, const QuantTab& qt, bool ln, int threads,
                          int grid, size_t shmem, hipStream_t st) {
  auto k_ln = ln_quant_kernel<BITS, NUNIT, true>;
  auto k_plain = ln_quant_kernel<BITS, NUNIT, false>;
  if (shmem > 64 * 1024) {
    RPTQ_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(ln ? k_ln : k_plain),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(shmem)));
  }
  if (ln) {
    hipLaunchKernelGGL(k_ln, dim3(grid), dim3(threads), shmem, st, a, geom, qt);
  } else {
    hipLaunchKernelGGL(k_plain, dim3(grid), dim3(threads), shmem, st, a, geom, qt);
  }
  RPTQ_HIP(hipGetLastError());
  return RPTQ_OK;
}

template <int BITS>
static int32_t launch_bits(const LnQuantArgs& a, const ClusterGeom& geom, const QuantTab& qt, bool ln, int nunit,
                           int threads, int grid, size_t shmem, hipStream_t st) {
  switch (nunit) {
    case 1: return launch_one<BITS, 1>(a, geom, qt, ln, threads, grid, shmem, st);
    case 2: return launch_one<BITS, 2>(a, geom, qt, ln, threads, grid, shmem, st);
    case 3: return launch_one<BITS, 3>(a, geom, qt, ln, threads, grid, shmem, st);
    default: return launch_one<BITS, 4>(a, geom, qt, ln, threads, grid, shmem, st);
  }
}

int32_t launch_ln_quant(const void* x, int64_t M, int32_t d, const float* gamma_pad, const float* beta_pad,
                        float eps, int32_t relu, const int32_t* perm_pad, const ClusterGeom& geom,
                        const QuantTab& qt, int32_t bits, void* codes, int32_t* xsum, float* rowterm,
                        hipStream_t st) {
  if (M == 0) return RPTQ_OK;
  LnQuantArgs a;
  a.x = static_cast<const uint4*>(x);
  a.M = M;
  a.d = d;
  a.chunks = d / 8;
  a.gamma_pad = gamma_pad;
  a.beta_pad = beta_pad;
  a.eps = eps;
  a.relu = relu;
  a.perm_pad = perm_pad;
  a.codes = static_cast<uint8_t*>(codes);
  a.rowterm = rowterm;
  const int uc = (bits == 3) ? 16 : 8;
  a.n_units = geom.k_padded / uc;
  a.row_bytes = geom.k_padded * bits / 8;

  // Threads: enough for the input chunks (<= kMaxChunk per thread) and the units (<= 4 per
  // thread), a multiple of the wave size, as few idle lanes in the unit phase as possible.
  const bool ln = gamma_pad != nullptr;
  // register budget at 1024 threads: per-unit constants of more units than this would spill
  const int max_nunit = ln ? (bits == 3 ? 1 : 2) : (bits == 3 ? 2 : 4);
  int best_t = 0, best_n = 0;
  double best_waste = 1e30;
  for (int nunit = 1; nunit <= max_nunit; ++nunit) {
    int t = (a.n_units + nunit - 1) / nunit;
    t = (t + kWave - 1) / kWave * kWave;
    const int t_chunks = ((a.chunks + kMaxChunk - 1) / kMaxChunk + kWave - 1) / kWave * kWave;
    if (t < t_chunks) t = t_chunks;
    if (t > 1024) continue;
    if (t < 256 && nunit > 1) continue;
    const double waste = static_cast<double>(t) * nunit / a.n_units;
    if (waste < best_waste - 1e-9) {
      best_waste = waste;
      best_t = t;
      best_n = nunit;
    }
  }
  if (best_t == 0) return RPTQ_ERR_SHAPE;

  int dev = 0, cus = 256;
  RPTQ_HIP(hipGetDevice(&dev));
  RPTQ_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  const size_t shmem = static_cast<size_t>(d) * 4 + 2 * kMaxWaves * 3 * sizeof(double);
  if (shmem > 160 * 1024) return RPTQ_ERR_SHAPE;
  int per_cu = static_cast<int>(std::min<size_t>(1024 / best_t, (160 * 1024) / shmem));
  if (per_cu < 1) per_cu = 1;
  const int64_t grid64 = std::min<int64_t>(M, static_cast<int64_t>(cus) * per_cu);
  const int grid = static_cast<int>(grid64);

  int32_t stt;
  if (bits == 3) stt = launch_bits<3>(a, geom, qt, ln, best_n, best_t, grid, shmem, st);
  else if (bits == 4) stt = launch_bits<4>(a, geom, qt, ln, best_n, best_t, grid, shmem, st);
  else stt = launch_bits<8>(a, geom, qt, ln, best_n, best_t, grid, shmem, st);
  if (stt) return stt;

  if (xsum) {
    const int thr = (geom.g + kWave - 1) / kWave * kWave;
    if (bits == 3) hipLaunchKernelGGL(xsum_kernel<3>, dim3(static_cast<unsigned>(M)), dim3(thr), 0, st, a.codes, M, a.row_bytes, geom, xsum);
    else if (bits == 4) hipLaunchKernelGGL(xsum_kernel<4>, dim3(static_cast<unsigned>(M)), dim3(thr), 0, st, a.codes, M, a.row_bytes, geom, xsum);
    else hipLaunchKernelGGL(xsum_kernel<8>, dim3(static_cast<unsigned>(M)), dim3(thr), 0, st, a.codes, M, a.row_bytes, geom, xsum);
    RPTQ_HIP(hipGetLastError());
  }
  return RPTQ_OK;
}

int32_t launch_unpack_codes(const void* codes, int64_t rows, const ClusterGeom& geom, int32_t bits, int8_t* out,
                            hipStream_t st) {
  if (rows == 0) return RPTQ_OK;
  const uint8_t* c = static_cast<const uint8_t*>(codes);
  const int32_t row_bytes = geom.k_padded * bits / 8;
  const dim3 grid(static_cast<unsigned>(rows)), block(256);
  if (bits == 3) hipLaunchKernelGGL(unpack_codes_kernel<3>, grid, block, 0, st, c, rows, row_bytes, geom, out);
  else if (bits == 4) hipLaunchKernelGGL(unpack_codes_kernel<4>, grid, block, 0, st, c, rows, row_bytes, geom, out);
  else hipLaunchKernelGGL(unpack_codes_kernel<8>, grid, block, 0, st, c, rows, row_bytes, geom, out);
  RPTQ_HIP(hipGetLastError());
  return RPTQ_OK;
}

}  // namespace rptq
