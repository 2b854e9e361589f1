// First method of App. A.4 ("de-quantize, concatenate, multiply in floating point") as the
// comparison variant of the cluster-wise integer product: both operands are de-quantized to
// bf16 (x_hat = s (x_q - z), the line under Eq. 1) in the padded cluster-order layout, pad
// positions zero, and multiplied on the bf16 matrix cores with fp32 accumulation.  One
// accumulator set, no per-cluster work in the product; the price is twice the bytes per
// operand element of int8 (four times those of packed 4-bit weights), half the matrix rate
// and the rounding of every operand to eight significant bits.
#include <hip/hip_runtime.h>

#include "device_common.h"
#include "pack_formats.h"
#include "rptq_internal.h"

namespace rptq {

typedef float f2v __attribute__((ext_vector_type(2)));
typedef __bf16 b2v __attribute__((ext_vector_type(2)));
typedef __bf16 b8v __attribute__((ext_vector_type(8)));
typedef float v16f32 __attribute__((ext_vector_type(16)));
typedef unsigned u4v __attribute__((ext_vector_type(4)));    // 16 bytes as a plain vector value (a uint4 copy is a memcpy the optimizer leaves in memory)

// s * n for an integer-valued n (exact in fp32), rounded once to fp32 and once to bf16 (ties to even); two at a time
__device__ __forceinline__ uint32_t dequant_pair(float s0, float n0, float s1, float n1) {
  const f2v pr = {__fmul_rn(s0, n0), __fmul_rn(s1, n1)};
  const b2v cv = __builtin_convertvector(pr, b2v);
  return *reinterpret_cast<const uint32_t*>(&cv);
}

struct DequantTab {
  float s[RPTQ_MAX_CLUSTERS];
  float zf[RPTQ_MAX_CLUSTERS];
};

// Activation codes [M, K_p * bits / 8] -> bf16 [M, K_p].  One thread per 32-code group.
template <int BITS>
__global__ void __launch_bounds__(256) dequant_codes_kernel(const uint8_t* codes, int64_t M, int32_t row_bytes,
                                                            ClusterGeom geom, DequantTab tab, uint16_t* out) {
  constexpr int GB = BITS * 4;
  const int groups = geom.k_padded / kGroup;
  const int64_t total = M * groups;
  for (int64_t gid = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; gid < total;
       gid += static_cast<int64_t>(gridDim.x) * blockDim.x) {
    const int64_t row = gid / groups;
    const int gi = static_cast<int>(gid % groups);
    int ci = 0;
    for (int i = 1; i < geom.g; ++i) ci += (gi * kGroup >= geom.pad_off[i]) ? 1 : 0;
    int n_real = (geom.off[ci + 1] - geom.off[ci]) - (gi * kGroup - geom.pad_off[ci]);      // real codes of the group
    n_real = n_real < 0 ? 0 : (n_real > kGroup ? kGroup : n_real);
    const float s = tab.s[ci], zf = tab.zf[ci];
    uint32_t w[GB / 4];
    const uint32_t* p = reinterpret_cast<const uint32_t*>(codes + row * row_bytes + static_cast<int64_t>(gi) * GB);
#pragma unroll
    for (int k = 0; k < GB / 4; ++k) w[k] = p[k];
    int q[32];
    decode_group<BITS>(w, q);
    uint32_t o[16];
#pragma unroll
    for (int j = 0; j < 32; j += 2) {
      const float n0 = j < n_real ? static_cast<float>(q[j]) - zf : 0.0f;          // pad positions: 0
      const float n1 = (j + 1) < n_real ? static_cast<float>(q[j + 1]) - zf : 0.0f;
      o[j / 2] = dequant_pair(s, n0, s, n1);
    }
    uint4* dst = reinterpret_cast<uint4*>(out + row * geom.k_padded + static_cast<int64_t>(gi) * kGroup);
#pragma unroll
    for (int k = 0; k < 4; ++k) dst[k] = make_uint4(o[4 * k], o[4 * k + 1], o[4 * k + 2], o[4 * k + 3]);
  }
}

// Packed 4-bit weights (MFMA-lane-major blocks) -> bf16 [N, K_p], w_hat = sW[o] (w_q - zW[o]), pad positions zero.
// One thread per (output row, 8 columns): one dword in, 16 bytes out.
__global__ void __launch_bounds__(256) dequant_weights_kernel(const uint8_t* Wq, int32_t N, ClusterGeom geom, const float* sW,
                                                              const int32_t* zW, uint16_t* out) {
  const int units = geom.k_padded / 8;
  const int64_t total = static_cast<int64_t>(N) * units;
  for (int64_t id = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; id < total;
       id += static_cast<int64_t>(gridDim.x) * blockDim.x) {
    const int o = static_cast<int>(id / units), u = static_cast<int>(id % units);
    int ci = 0;
    for (int i = 1; i < geom.g; ++i) ci += (u * 8 >= geom.pad_off[i]) ? 1 : 0;
    int n_real = (geom.off[ci + 1] - geom.off[ci]) - (u * 8 - geom.pad_off[ci]);
    n_real = n_real < 0 ? 0 : (n_real > 8 ? 8 : n_real);
    const float s = sW[o], zf = static_cast<float>(zW[o]);
    const uint32_t word = *reinterpret_cast<const uint32_t*>(Wq + weight_dword_offset(o, u, geom.k_padded));
    float n[8];
#pragma unroll
    for (int b = 0; b < 4; ++b) {                   // byte b: high nibble = column 8u + b, low nibble = column 8u + 4 + b
      const int hi = static_cast<int>(word << (24 - 8 * b)) >> 28;
      const int lo = static_cast<int>(word << (28 - 8 * b)) >> 28;
      n[b] = b < n_real ? static_cast<float>(hi) - zf : 0.0f;
      n[4 + b] = (4 + b) < n_real ? static_cast<float>(lo) - zf : 0.0f;
    }
    *reinterpret_cast<uint4*>(out + static_cast<int64_t>(o) * geom.k_padded + u * 8) =
        make_uint4(dequant_pair(s, n[0], s, n[1]), dequant_pair(s, n[2], s, n[3]), dequant_pair(s, n[4], s, n[5]),
                   dequant_pair(s, n[6], s, n[7]));
  }
}

// Y[t, n] = sum_k xh[t, k] wh[n, k], bf16 operands, fp32 accumulation (v_mfma_f32_32x32x16_bf16).
// Workgroup tile 128 tokens x 128 channels, four waves of 64 x 64; K steps of 64 through two LDS
// stages, one barrier per step; the next step's operands travel global -> registers while this
// step's MFMAs run.  The weights are the first operand, so a lane holds one token and runs of four
// consecutive channels: 16-byte stores.
constexpr int kM1Tile = 128;
constexpr int kM1Step = 64;                                 // K per step
constexpr int kM1Operand = kM1Tile * kM1Step * 2;           // bytes of one operand tile of a step

// The MFMAs of one K step: operand fragments from the LDS stage at `stage` (weights, then activations).
__device__ __forceinline__ void m1_compute(const unsigned char* stage, int wch, int wtok, int frag, v16f32 (&acc)[2][2]) {
  const unsigned char* wb = stage;
  const unsigned char* xb = stage + kM1Operand;
#pragma unroll
  for (int s = 0; s < kM1Step / 16; ++s) {
    b8v wf[2], xf[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) wf[i] = *reinterpret_cast<const b8v*>(wb + s * 2 * kM1Tile * 16 + (wch + i * 32) * 16 + frag);
#pragma unroll
    for (int j = 0; j < 2; ++j) xf[j] = *reinterpret_cast<const b8v*>(xb + s * 2 * kM1Tile * 16 + (wtok + j * 32) * 16 + frag);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], xf[j], acc[i][j], 0, 0, 0);
  }
}

template <bool YF32>
__global__ void __launch_bounds__(256, 2) gemm_bf16_kernel(const uint16_t* xh, const uint16_t* wh, int64_t M, int32_t N,
                                                           int32_t K, void* y, int32_t tiles_m, int32_t tiles_n) {
  extern __shared__ __align__(16) unsigned char smem[];      // [2 stages][weights | activations]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // Workgroups are dealt round robin to the 8 XCDs: each XCD gets a contiguous range of tiles, walked in
  // blocks of 8 token tiles x 8 channel tiles, so that the 64 workgroups resident on an XCD share 16
  // operand strips in its L2 (bf16 operands are four to five times the bytes of the packed codes).
  const int total = tiles_m * tiles_n;
  int lin = blockIdx.x;
  if (total % 8 == 0) lin = (lin & 7) * (total >> 3) + (lin >> 3);
  int tm = lin % tiles_m, tn = lin / tiles_m;
  if (tiles_m % 8 == 0) {
    const int group = lin / (8 * tiles_m), rem = lin % (8 * tiles_m);
    const int wg = (tiles_n - 8 * group) < 8 ? (tiles_n - 8 * group) : 8;
    const int chunk = rem / (8 * wg), r = rem % (8 * wg);
    tm = chunk * 8 + r / wg;
    tn = 8 * group + r % wg;
  }
  const int64_t m0 = static_cast<int64_t>(tm) * kM1Tile;
  const int n0 = tn * kM1Tile;
  const int steps = K / kM1Step;

  // this thread's four 16-byte chunks of each operand tile: rows clamped into the tensor (what a
  // clamped row contributes is never stored)
  const u4v* wsrc[4];
  const u4v* xsrc[4];
  int lds_off[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int q = tid + 256 * j, row = q >> 3, c = q & 7;    // chunk c = columns 8c .. 8c+7 of the step
    const int64_t wr = (n0 + row) < N ? (n0 + row) : (N - 1);
    const int64_t xr = (m0 + row) < M ? (m0 + row) : (M - 1);
    wsrc[j] = reinterpret_cast<const u4v*>(wh + wr * K) + c;
    xsrc[j] = reinterpret_cast<const u4v*>(xh + xr * K) + c;
    // a 16-column slice s = c >> 1 keeps its two 8-column halves apart: [s][half][row][16 bytes] is the
    // order the MFMA operand is read in (lane = half * 32 + row)
    lds_off[j] = (((c >> 1) * 2 + (c & 1)) * kM1Tile + row) * 16;
  }
  // Three register sets hold the operands of the next three steps on their way from memory (one step of
  // MFMAs is far shorter than a loaded memory latency).  Loops are written out where they are used:
  // register arrays handed to helper lambdas ended up in scratch memory.
  struct OperandRegs {
    u4v w0, w1, w2, w3, x0, x1, x2, x3;
  } ra, rb, rc;
#define RPTQ_M1_FETCH(r_, step_)                                                                                  \
  {                                                                                                               \
    const int fs_ = ((step_) < steps ? (step_) : (steps - 1)) * (kM1Step / 8); /* past the end: the last step again */ \
    r_.w0 = wsrc[0][fs_]; r_.x0 = xsrc[0][fs_]; r_.w1 = wsrc[1][fs_]; r_.x1 = xsrc[1][fs_];                         \
    r_.w2 = wsrc[2][fs_]; r_.x2 = xsrc[2][fs_]; r_.w3 = wsrc[3][fs_]; r_.x3 = xsrc[3][fs_];                         \
  }
#define RPTQ_M1_STASH(r_, stage_)                                                                                 \
  {                                                                                                               \
    unsigned char* base_ = smem + (stage_) * 2 * kM1Operand;                                                      \
    *reinterpret_cast<u4v*>(base_ + lds_off[0]) = r_.w0; *reinterpret_cast<u4v*>(base_ + kM1Operand + lds_off[0]) = r_.x0; \
    *reinterpret_cast<u4v*>(base_ + lds_off[1]) = r_.w1; *reinterpret_cast<u4v*>(base_ + kM1Operand + lds_off[1]) = r_.x1; \
    *reinterpret_cast<u4v*>(base_ + lds_off[2]) = r_.w2; *reinterpret_cast<u4v*>(base_ + kM1Operand + lds_off[2]) = r_.x2; \
    *reinterpret_cast<u4v*>(base_ + lds_off[3]) = r_.w3; *reinterpret_cast<u4v*>(base_ + kM1Operand + lds_off[3]) = r_.x3; \
  }

  v16f32 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const int wch = (wave & 1) * 64, wtok = (wave >> 1) * 64;    // this wave's channels and tokens inside the tile
  const int frag = ((lane >> 5) * kM1Tile + (lane & 31)) * 16;

  // one step: the MFMAs of step k from LDS stage k & 1; then the registers that hold step k + 1 go to the other
  // stage and are refilled with step k + 4
#define RPTQ_M1_STEP(k_, set_)               \
  {                                          \
    m1_compute(smem + ((k_) & 1) * 2 * kM1Operand, wch, wtok, frag, acc); \
    RPTQ_M1_STASH(set_, ((k_) & 1) ^ 1)      \
    RPTQ_M1_FETCH(set_, (k_) + 4)            \
    __syncthreads();                         \
  }

  RPTQ_M1_FETCH(ra, 0)
  RPTQ_M1_STASH(ra, 0)
  RPTQ_M1_FETCH(rb, 1)                        // step j travels in set j % 3 (ra, rb, rc)
  RPTQ_M1_FETCH(rc, 2)
  RPTQ_M1_FETCH(ra, 3)
  __syncthreads();
  int step = 0;
  for (; step + 2 < steps; step += 3) {
    RPTQ_M1_STEP(step, rb)
    RPTQ_M1_STEP(step + 1, rc)
    RPTQ_M1_STEP(step + 2, ra)
  }
  if (step < steps) RPTQ_M1_STEP(step, rb)
  if (step + 1 < steps) RPTQ_M1_STEP(step + 1, rc)
#undef RPTQ_M1_STEP
#undef RPTQ_M1_FETCH
#undef RPTQ_M1_STASH

  // D[channel][token]: lane & 31 = token, register quad q4 = channels 8 q4 + 4 (lane >> 5) .. + 3
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int64_t t = m0 + wtok + j * 32 + (lane & 31);
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int n = n0 + wch + i * 32 + q4 * 8 + (lane >> 5) * 4;
        if (t < M && n + 3 < N) {
          if (YF32) {
            *reinterpret_cast<float4*>(static_cast<float*>(y) + t * N + n) =
                make_float4(acc[i][j][q4 * 4], acc[i][j][q4 * 4 + 1], acc[i][j][q4 * 4 + 2], acc[i][j][q4 * 4 + 3]);
          } else {
            const f2v p0 = {acc[i][j][q4 * 4], acc[i][j][q4 * 4 + 1]}, p1 = {acc[i][j][q4 * 4 + 2], acc[i][j][q4 * 4 + 3]};
            const b2v c0 = __builtin_convertvector(p0, b2v), c1 = __builtin_convertvector(p1, b2v);
            *reinterpret_cast<uint2*>(static_cast<uint16_t*>(y) + t * N + n) =
                make_uint2(*reinterpret_cast<const uint32_t*>(&c0), *reinterpret_cast<const uint32_t*>(&c1));
          }
        }
      }
    }
}

int32_t launch_dequant_codes(const void* codes, int64_t M, const ClusterGeom& geom, int32_t bits, const float* sX,
                             const int32_t* zX, void* out, hipStream_t st) {
  if (M == 0) return RPTQ_OK;
  DequantTab tab;
  for (int i = 0; i < RPTQ_MAX_CLUSTERS; ++i) {
    tab.s[i] = i < geom.g ? sX[i] : 0.0f;
    tab.zf[i] = i < geom.g ? static_cast<float>(zX[i]) : 0.0f;
  }
  int cus = 0;
  if (int32_t s = device_compute_units(st, &cus)) return s;
  const int64_t total = M * (geom.k_padded / kGroup);
  const dim3 grid(static_cast<unsigned>(std::min<int64_t>((total + 255) / 256, static_cast<int64_t>(cus) * 32))), block(256);
  const uint8_t* c = static_cast<const uint8_t*>(codes);
  const int32_t row_bytes = geom.k_padded * bits / 8;
  uint16_t* o = static_cast<uint16_t*>(out);
  if (bits == 3) hipLaunchKernelGGL(dequant_codes_kernel<3>, grid, block, 0, st, c, M, row_bytes, geom, tab, o);
  else if (bits == 4) hipLaunchKernelGGL(dequant_codes_kernel<4>, grid, block, 0, st, c, M, row_bytes, geom, tab, o);
  else hipLaunchKernelGGL(dequant_codes_kernel<8>, grid, block, 0, st, c, M, row_bytes, geom, tab, o);
  RPTQ_HIP(hipGetLastError());
  return RPTQ_OK;
}

int32_t launch_dequant_weights(const void* Wq, int32_t N, const ClusterGeom& geom, const float* sW, const int32_t* zW,
                               void* out, hipStream_t st) {
  int cus = 0;
  if (int32_t s = device_compute_units(st, &cus)) return s;
  const int64_t total = static_cast<int64_t>(N) * (geom.k_padded / 8);
  const dim3 grid(static_cast<unsigned>(std::min<int64_t>((total + 255) / 256, static_cast<int64_t>(cus) * 32))), block(256);
  hipLaunchKernelGGL(dequant_weights_kernel, grid, block, 0, st, static_cast<const uint8_t*>(Wq), N, geom, sW, zW,
                     static_cast<uint16_t*>(out));
  RPTQ_HIP(hipGetLastError());
  return RPTQ_OK;
}

int32_t launch_gemm_bf16(const void* xh, const void* wh, int64_t M, int32_t N, int32_t K, void* y, int32_t y_f32,
                         hipStream_t st) {
  if (M == 0) return RPTQ_OK;
  const size_t shmem = 2 * 2 * kM1Operand;                    // 64 KiB
  const int tiles_m = static_cast<int>((M + kM1Tile - 1) / kM1Tile), tiles_n = (N + kM1Tile - 1) / kM1Tile;
  const dim3 grid(static_cast<unsigned>(tiles_m) * static_cast<unsigned>(tiles_n)), block(256);
  const uint16_t* x = static_cast<const uint16_t*>(xh);
  const uint16_t* w = static_cast<const uint16_t*>(wh);
  if (y_f32) {
    static LdsGrant granted;
    if (int32_t s = ensure_dynamic_lds(reinterpret_cast<const void*>(gemm_bf16_kernel<true>), shmem, &granted, st)) return s;
    hipLaunchKernelGGL(gemm_bf16_kernel<true>, grid, block, shmem, st, x, w, M, N, K, y, tiles_m, tiles_n);
  } else {
    static LdsGrant granted;
    if (int32_t s = ensure_dynamic_lds(reinterpret_cast<const void*>(gemm_bf16_kernel<false>), shmem, &granted, st)) return s;
    hipLaunchKernelGGL(gemm_bf16_kernel<false>, grid, block, shmem, st, x, w, M, N, K, y, tiles_m, tiles_n);
  }
  RPTQ_HIP(hipGetLastError());
  return RPTQ_OK;
}

}  // namespace rptq
