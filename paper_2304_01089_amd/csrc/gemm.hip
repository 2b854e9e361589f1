// Cluster-wise integer product (App. A.4, second method) on int8 MFMA.
//
// K runs over the padded cluster-order layout in slices of 32 codes, so a cluster always
// ends on a slice boundary.  Packed 3/4/8-bit activation codes and packed 4-bit weight
// codes are loaded from global memory, turned into sign-carrying int8 (code << 5, << 4 or
// << 0; weights << 4) with one shift/mask per four codes, and written to LDS in the order
// the 32x32x32 int8 MFMA reads its operands.  When the last slice of cluster i has been
// accumulated, the int32 accumulators hold 2^shift * P_i; they are converted, scaled by
// sX_i / 2^shift, added to the fp32 result and cleared.  The zero-point terms of App. A.4
// are applied once at the end from per-row and per-column vectors.
#include <hip/hip_runtime.h>

#include "device_common.h"
#include "rptq_internal.h"

namespace rptq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

struct GemmArgs {
  const uint8_t* codes;      // packed activation codes, row-major
  int64_t M;
  int32_t row_bytes;         // K_p * bits / 8
  const uint8_t* Wq;         // packed weights, fragment-major
  int32_t N;
  int32_t slices;            // K_p / 32
  int32_t used_slices;       // slices up to the end of the last cluster
  const float* sW;
  const int32_t* zW;
  const float* colterm;
  const float* rowterm;
  void* y;
  // verification mode
  const int32_t* xsum;
  const int32_t* wsum;
  int32_t* yq;
};

struct GemmTab {
  int32_t g;
  int32_t slice_end[RPTQ_MAX_CLUSTERS];   // first slice after cluster i
  float scale[RPTQ_MAX_CLUSTERS];         // sX_i / 2^shift
  int32_t zx[RPTQ_MAX_CLUSTERS];
  int32_t n[RPTQ_MAX_CLUSTERS];           // channels in cluster i
};

constexpr int kStepSlices = 4;            // slices per K step (128 codes)
constexpr int kSlicePad = 32;             // bytes added to a slice's LDS stride (bank spread on writes)

template <int BITS>
struct ActFmt {
  static constexpr int kGroupBytes = BITS * 4;             // bytes of 32 packed codes
  static constexpr int kShift = (BITS == 8) ? 0 : (BITS == 4 ? 4 : 5);
};

// 16 bytes of 4-bit codes (32 codes) -> 32 int8 values (code << 4), natural order.
__device__ __forceinline__ void unpack4(const uint4 p, uint4* lo, uint4* hi) {
  lo->x = p.x & 0xf0f0f0f0u;
  lo->y = (p.x << 4) & 0xf0f0f0f0u;
  lo->z = p.y & 0xf0f0f0f0u;
  lo->w = (p.y << 4) & 0xf0f0f0f0u;
  hi->x = p.z & 0xf0f0f0f0u;
  hi->y = (p.z << 4) & 0xf0f0f0f0u;
  hi->z = p.w & 0xf0f0f0f0u;
  hi->w = (p.w << 4) & 0xf0f0f0f0u;
}

// 12 bytes of 3-bit codes (32 codes) -> 32 int8 values (code << 5), natural order.
__device__ __forceinline__ void unpack3(uint32_t x0, uint32_t x1, uint32_t x2, uint4* lo, uint4* hi) {
  lo->x = x0 & 0xe0e0e0e0u;
  lo->y = (x0 << 3) & 0xe0e0e0e0u;
  lo->z = x1 & 0xe0e0e0e0u;
  lo->w = (x1 << 3) & 0xe0e0e0e0u;
  hi->x = x2 & 0xe0e0e0e0u;
  hi->y = (x2 << 3) & 0xe0e0e0e0u;
  hi->z = ((x0 << 6) & 0xc0c0c0c0u) | ((x2 << 5) & 0x20202020u);
  hi->w = ((x1 << 6) & 0xc0c0c0c0u) | ((x2 << 4) & 0x20202020u);
}

template <int BITS, int WGM, int WGN, int WM, int WN, bool PARTIALS, bool YF32>
__global__ void __launch_bounds__(256) cluster_gemm_kernel(GemmArgs a, GemmTab tab) {
  constexpr int BM = WGM * WM * 32;
  constexpr int BN = WGN * WN * 32;
  constexpr int A_SLICE = 2 * BM * 16 + kSlicePad;       // [half][row][16 B]
  constexpr int B_SLICE = 2 * BN * 16 + kSlicePad;
  constexpr int A_STAGE = kStepSlices * A_SLICE;
  constexpr int B_STAGE = kStepSlices * B_SLICE;
  constexpr int A_UNITS = BM * kStepSlices;              // (row, slice) units per K step
  constexpr int B_UNITS = (BN / 32) * kStepSlices * 32;  // 16-byte units per K step
  constexpr int A_PER = (A_UNITS + 255) / 256;
  constexpr int B_PER = (B_UNITS + 255) / 256;
  constexpr int GB = ActFmt<BITS>::kGroupBytes;
  constexpr int A_REGS = GB / 4;                          // dwords per A unit

  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* sA = smem;                               // [2][A_STAGE]
  unsigned char* sB = smem + 2 * A_STAGE;                 // [2][B_STAGE]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int64_t m0 = static_cast<int64_t>(blockIdx.y) * BM;
  const int n0 = blockIdx.x * BN;

  // ---- global -> register staging ------------------------------------------------------
  uint32_t ra[A_PER][A_REGS];
  uint4 rb[B_PER];
  const uint8_t* a_ptr[A_PER];
  const uint8_t* b_ptr[B_PER];
  int a_lds[A_PER], b_lds[B_PER];
#pragma unroll
  for (int i = 0; i < A_PER; ++i) {
    const int unit = tid + i * 256;
    const int row = unit / kStepSlices, s = unit % kStepSlices;
    int64_t grow = m0 + row;
    if (grow >= a.M) grow = a.M - 1;                       // clamp: loads stay in bounds, rows never stored
    a_ptr[i] = a.codes + grow * a.row_bytes + s * GB;
    a_lds[i] = s * A_SLICE + row * 16;
    if (unit >= A_UNITS) a_lds[i] = -1;
  }
#pragma unroll
  for (int i = 0; i < B_PER; ++i) {
    const int unit = tid + i * 256;
    const int blk = unit / 32, p = unit % 32;
    const int rbl = blk / kStepSlices, s = blk % kStepSlices;
    b_ptr[i] = a.Wq + ((static_cast<size_t>(n0 / 32 + rbl) * a.slices + s) * 64) * 8 + p * 16;
    const int h = p / 16, r = (2 * p) % 32;
    b_lds[i] = s * B_SLICE + h * (BN * 16) + (rbl * 32 + r) * 16;
    if (unit >= B_UNITS) b_lds[i] = -1;
  }

  auto load_global = [&](int step) {
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
      if (a_lds[i] < 0) continue;
      const uint32_t* p = reinterpret_cast<const uint32_t*>(a_ptr[i] + static_cast<size_t>(step) * kStepSlices * GB);
#pragma unroll
      for (int k = 0; k < A_REGS; ++k) ra[i][k] = p[k];
    }
#pragma unroll
    for (int i = 0; i < B_PER; ++i) {
      if (b_lds[i] < 0) continue;
      rb[i] = *reinterpret_cast<const uint4*>(b_ptr[i] + static_cast<size_t>(step) * kStepSlices * 512);
    }
  };

  auto store_lds = [&](int buf) {
    unsigned char* dA = sA + buf * A_STAGE;
    unsigned char* dB = sB + buf * B_STAGE;
#pragma unroll
    for (int i = 0; i < A_PER; ++i) {
      if (a_lds[i] < 0) continue;
      uint4 lo, hi;
      if (BITS == 8) {
        lo = make_uint4(ra[i][0], ra[i][1], ra[i][2], ra[i][3]);
        hi = make_uint4(ra[i][4 % A_REGS], ra[i][5 % A_REGS], ra[i][6 % A_REGS], ra[i][7 % A_REGS]);
      } else if (BITS == 4) {
        unpack4(make_uint4(ra[i][0], ra[i][1], ra[i][2], ra[i][3]), &lo, &hi);
      } else {
        unpack3(ra[i][0], ra[i][1], ra[i][2], &lo, &hi);
      }
      *reinterpret_cast<uint4*>(dA + a_lds[i]) = lo;
      *reinterpret_cast<uint4*>(dA + a_lds[i] + BM * 16) = hi;
    }
#pragma unroll
    for (int i = 0; i < B_PER; ++i) {
      if (b_lds[i] < 0) continue;
      uint4 r0, r1;                                        // rows r and r+1 of the same k half
      unpack4(rb[i], &r0, &r1);
      *reinterpret_cast<uint4*>(dB + b_lds[i]) = r0;
      *reinterpret_cast<uint4*>(dB + b_lds[i] + 16) = r1;
    }
  };

  // ---- accumulators -----------------------------------------------------------------------
  v16i acc[WM][WN];
  float facc[PARTIALS ? 1 : WM][PARTIALS ? 1 : WN][16];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        acc[i][j][r] = 0;
        if (!PARTIALS) facc[i][j][r] = 0.0f;
      }
    }

  const int a_frag = (lane >> 5) * (BM * 16) + (wm * WM * 32 + (lane & 31)) * 16;
  const int b_frag = (lane >> 5) * (BN * 16) + (wn * WN * 32 + (lane & 31)) * 16;

  int ci = 0;
  int next_end = tab.slice_end[0];
  const int steps = (a.used_slices + kStepSlices - 1) / kStepSlices;

  load_global(0);
  for (int step = 0; step < steps; ++step) {
    const int buf = step & 1;
    store_lds(buf);
    __syncthreads();
    if (step + 1 < steps) load_global(step + 1);
    const unsigned char* cA = sA + buf * A_STAGE;
    const unsigned char* cB = sB + buf * B_STAGE;
#pragma unroll
    for (int s = 0; s < kStepSlices; ++s) {
      v4i fa[WM], fb[WN];
#pragma unroll
      for (int i = 0; i < WM; ++i) fa[i] = *reinterpret_cast<const v4i*>(cA + s * A_SLICE + a_frag + i * 32 * 16);
#pragma unroll
      for (int j = 0; j < WN; ++j) fb[j] = *reinterpret_cast<const v4i*>(cB + s * B_SLICE + b_frag + j * 32 * 16);
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);

      const int gs = step * kStepSlices + s + 1;           // slices accumulated so far
      if (gs == next_end) {                                  // cluster ci is complete (uniform branch)
        const float sc = tab.scale[ci];
        if (PARTIALS) {
          const int zx = tab.zx[ci], nn = tab.n[ci];
#pragma unroll
          for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int j = 0; j < WN; ++j) {
              const int n = n0 + (wn * WN + j) * 32 + (lane & 31);
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                const int64_t t = m0 + (wm * WM + i) * 32 + (r / 4) * 8 + (lane >> 5) * 4 + (r % 4);
                if (t < a.M && n < a.N) {
                  const int p = acc[i][j][r] >> (ActFmt<BITS>::kShift + 4);
                  const int zw = a.zW[n];
                  const int v = p - zx * a.wsum[static_cast<int64_t>(n) * tab.g + ci] -
                                zw * a.xsum[t * tab.g + ci] + nn * zx * zw;
                  a.yq[(static_cast<int64_t>(ci) * a.M + t) * a.N + n] = v;
                }
                acc[i][j][r] = 0;
              }
            }
        } else {
#pragma unroll
          for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int j = 0; j < WN; ++j)
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                facc[i][j][r] = fmaf(static_cast<float>(acc[i][j][r]), sc, facc[i][j][r]);
                acc[i][j][r] = 0;
              }
        }
        ++ci;
        next_end = ci < tab.g ? tab.slice_end[ci] : -1;
      }
    }
  }

  // ---- zero-point terms and output scale ---------------------------------------------------
  if (!PARTIALS) {
#pragma unroll
    for (int j = 0; j < WN; ++j) {
      const int n = n0 + (wn * WN + j) * 32 + (lane & 31);
      const bool n_ok = n < a.N;
      const float sw = n_ok ? a.sW[n] : 0.0f;
      const float ct = n_ok ? a.colterm[n] : 0.0f;
      const float zw = n_ok ? static_cast<float>(a.zW[n]) : 0.0f;
#pragma unroll
      for (int i = 0; i < WM; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int64_t t = m0 + (wm * WM + i) * 32 + (r / 4) * 8 + (lane >> 5) * 4 + (r % 4);
          if (t < a.M && n_ok) {
            const float v = sw * ((facc[i][j][r] - ct) - zw * a.rowterm[t]);
            if (YF32) {
              static_cast<float*>(a.y)[t * a.N + n] = v;
            } else {
              const uint32_t bits = __float_as_uint(v);
              const uint32_t rounded = bits + 0x7fffu + ((bits >> 16) & 1u);   // round to nearest even
              static_cast<uint16_t*>(a.y)[t * a.N + n] = static_cast<uint16_t>(rounded >> 16);
            }
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
template <int BITS, int WGM, int WGN, int WM, int WN, bool PARTIALS, bool YF32>
static int32_t launch_cfg(const GemmArgs& a, const GemmTab& tab, hipStream_t st) {
  constexpr int BM = WGM * WM * 32, BN = WGN * WN * 32;
  constexpr size_t shmem = 2 * kStepSlices * ((2 * BM * 16 + kSlicePad) + (2 * BN * 16 + kSlicePad));
  auto kern = cluster_gemm_kernel<BITS, WGM, WGN, WM, WN, PARTIALS, YF32>;
  if (shmem > 64 * 1024) RPTQ_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(shmem)));
  const dim3 grid((a.N + BN - 1) / BN, static_cast<unsigned>((a.M + BM - 1) / BM));
  hipLaunchKernelGGL(kern, grid, dim3(256), shmem, st, a, tab);
  RPTQ_HIP(hipGetLastError());
  return RPTQ_OK;
}

template <int BITS, bool PARTIALS, bool YF32>
static int32_t launch_shape(const GemmArgs& a, const GemmTab& tab, hipStream_t st) {
  if (a.M <= 32) return launch_cfg<BITS, 1, 4, 1, 1, PARTIALS, YF32>(a, tab, st);
  return launch_cfg<BITS, 2, 2, 2, 2, PARTIALS, YF32>(a, tab, st);
}

template <int BITS>
static int32_t launch_bits(const GemmArgs& a, const GemmTab& tab, bool partials, bool yf32, hipStream_t st) {
  if (partials) return launch_shape<BITS, true, true>(a, tab, st);
  if (yf32) return launch_shape<BITS, false, true>(a, tab, st);
  return launch_shape<BITS, false, false>(a, tab, st);
}

int32_t launch_gemm(const void* codes, int64_t M, int32_t bits, const void* Wq, int32_t N,
                    const ClusterGeom& geom, const float* sX, const float* sW, const int32_t* zW,
                    const float* colterm, const float* rowterm, void* y, int32_t y_dtype,
                    const int32_t* zX, const int32_t* xsum, const int32_t* wsum, int32_t* yq, hipStream_t st) {
  if (M == 0) return RPTQ_OK;
  GemmArgs a;
  a.codes = static_cast<const uint8_t*>(codes);
  a.M = M;
  a.row_bytes = geom.k_padded * bits / 8;
  a.Wq = static_cast<const uint8_t*>(Wq);
  a.N = N;
  a.slices = geom.k_padded / kGroup;
  a.used_slices = geom.pad_off[geom.g] / kGroup;
  a.sW = sW;
  a.zW = zW;
  a.colterm = colterm;
  a.rowterm = rowterm;
  a.y = y;
  a.xsum = xsum;
  a.wsum = wsum;
  a.yq = yq;
  GemmTab tab;
  tab.g = geom.g;
  const int shift = (bits == 8 ? 0 : (bits == 4 ? 4 : 5)) + 4;
  for (int i = 0; i < RPTQ_MAX_CLUSTERS; ++i) {
    const bool in = i < geom.g;
    tab.slice_end[i] = in ? geom.pad_off[i + 1] / kGroup : -1;
    tab.scale[i] = (in && sX) ? sX[i] / static_cast<float>(1 << shift) : 0.0f;
    tab.zx[i] = (in && zX) ? zX[i] : 0;
    tab.n[i] = in ? geom.off[i + 1] - geom.off[i] : 0;
  }
  const bool partials = yq != nullptr;
  const bool yf32 = y_dtype == RPTQ_DTYPE_F32;
  if (bits == 3) return launch_bits<3>(a, tab, partials, yf32, st);
  if (bits == 4) return launch_bits<4>(a, tab, partials, yf32, st);
  return launch_bits<8>(a, tab, partials, yf32, st);
}

}  // namespace rptq
