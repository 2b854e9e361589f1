// Key / value cache codes (Sec. 5.1: the W4A4KV, W4A3KV and W3A3KV settings quantize only the
// key and value caches; one reorder index per attention head, shared by queries and keys,
// Sec. 4.2) - writing: per head, channels in cluster order, Eq. 1 with the cluster's Eq. 2
// pair, packed at 3, 4 or 8 bits; reading: x_hat = s (x_q - z) as bf16 in cluster order.
//
// The cache layout is dense (no padding of clusters: the cache is what the method saves
// memory on), so the quantizer constants are per position, in a device table built once.
// A reorder index never moves a channel out of its head, so the gather is local: one wave
// owns a tile of 1024 consecutive channels (whole heads) of a row, stages its 2 KiB through
// a private piece of LDS and needs no workgroup barrier.
#include <hip/hip_runtime.h>

#include "device_common.h"
#include "pack_formats.h"
#include "rptq_internal.h"

namespace rptq {

constexpr int kKvTile = 1024;                  // channels per wave tile
constexpr int kKvLaneCodes = 16;               // codes per lane

// position of local code e of a lane inside the wave tile
template <int BITS>
__device__ __forceinline__ int kv_local_pos(int lane, int e) {
  if (BITS == 3) {
    // lanes 2g, 2g+1 share the 32-code group g: lane 2g carries codes 0..7, 24..27, 16..19,
    // lane 2g+1 codes 8..15, 28..31, 20..23 (so that each owns whole dwords of the group)
    const int role = lane & 1, gbase = (lane >> 1) * kGroup;
    if (e < 8) return gbase + role * 8 + e;
    if (e < 12) return gbase + 24 + role * 4 + (e - 8);
    return gbase + 16 + role * 4 + (e - 12);
  }
  return lane * kKvLaneCodes + e;
}

template <int BITS>
__global__ void __launch_bounds__(256) kv_quant_kernel(const uint4* x, int64_t T, int32_t d, const KvPos* pos,
                                                       uint8_t* codes, int32_t segs, int32_t row_groups) {
  constexpr int kQMin = -(1 << (BITS - 1));
  constexpr float kUMax = static_cast<float>((1 << BITS) - 1);
  __shared__ __align__(16) unsigned char lds[4][kKvTile * 2];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int seg = blockIdx.x % segs, rg = blockIdx.x / segs;
  const int base_ch = seg * kKvTile;
  const int n_here = (d - base_ch) < kKvTile ? (d - base_ch) : kKvTile;      // channels of this tile (multiple of 32)
  unsigned char* my = lds[wave];

  // per-lane constants: source offset inside the tile, 1/s and the biased zero point of each code
  uint32_t src[kKvLaneCodes];
  float inv_s[kKvLaneCodes], zbf[kKvLaneCodes];
#pragma unroll
  for (int e = 0; e < kKvLaneCodes; ++e) {
    const int lp = kv_local_pos<BITS>(lane, e);
    const KvPos kp = pos[base_ch + (lp < n_here ? lp : 0)];
    src[e] = static_cast<uint32_t>(kp.src - base_ch) * 2u;
    inv_s[e] = kp.inv_s;
    zbf[e] = static_cast<float>(kp.z - kQMin);
  }
  const bool lane_ok = (BITS == 3) ? ((lane >> 1) * kGroup < n_here) : (lane * kKvLaneCodes < n_here);
  // this lane's two 16-byte chunks of the tile's input (clamped inside the tile; surplus data is never gathered)
  const int chunks_here = n_here / 8;
  const int64_t row_chunks = d / 8;
  const int64_t stride = static_cast<int64_t>(row_groups) * 4;
  int64_t row = static_cast<int64_t>(rg) * 4 + wave;
  if (row >= T) return;
  const int64_t out_row_bytes = static_cast<int64_t>(d) * BITS / 8;
  const int64_t out_tile = static_cast<int64_t>(base_ch) * BITS / 8;

  // (scalars, not arrays handed to a helper by pointer: those ended up in scratch memory, re-written
  // every row)
  const int ch0 = lane < chunks_here ? lane : (chunks_here - 1);
  const int ch1 = (64 + lane) < chunks_here ? (64 + lane) : (chunks_here - 1);
  auto row_ptr = [&](int64_t r) {
    if (r >= T) r = T - 1;
    return x + r * row_chunks + base_ch / 8;
  };
  const uint4* p0 = row_ptr(row);
  uint4 cur0 = p0[ch0], cur1 = p0[ch1];
  const uint4* p1 = row_ptr(row + stride);
  uint4 nxt0 = p1[ch0], nxt1 = p1[ch1];
  for (; row < T; row += stride) {
    *reinterpret_cast<uint4*>(my + lane * 16) = cur0;
    *reinterpret_cast<uint4*>(my + (64 + lane) * 16) = cur1;
    cur0 = nxt0;
    cur1 = nxt1;
    const uint4* p2 = row_ptr(row + 2 * stride);
    nxt0 = p2[ch0];
    nxt1 = p2[ch1];
    __builtin_amdgcn_wave_barrier();                 // (one wave: LDS executes its instructions in order)
    uint32_t D[4] = {0u, 0u, 0u, 0u};                // biased codes, one byte each
#pragma unroll
    for (int e = 0; e < kKvLaneCodes; ++e) {
      const uint32_t h = *reinterpret_cast<const uint16_t*>(my + src[e]);
      const float y = __uint_as_float(h << 16);
      const float r = __fmul_rn(y, inv_s[e]);
      float b = __fadd_rn(rintf(r), zbf[e]);         // round, then add the zero point (biased by -qmin)
      if (BITS < 8) b = fminf(b, kUMax);             // upper clamp; the conversion saturates at 0 and 255
      D[e / 4] = __builtin_amdgcn_cvt_pk_u8_f32(b, e & 3, D[e / 4]);
    }
    __builtin_amdgcn_wave_barrier();
    uint8_t* out = codes + row * out_row_bytes + out_tile;
    if (BITS == 8) {
      const uint4 o = make_uint4(D[0] ^ 0x80808080u, D[1] ^ 0x80808080u, D[2] ^ 0x80808080u, D[3] ^ 0x80808080u);
      if (lane_ok) *reinterpret_cast<uint4*>(out + lane * 16) = o;
    } else if (BITS == 4) {
      uint2 o;
      o.x = ((D[0] << 4) | D[1]) ^ 0x88888888u;
      o.y = ((D[2] << 4) | D[3]) ^ 0x88888888u;
      if (lane_ok) *reinterpret_cast<uint2*>(out + lane * 8) = o;
    } else {
      const int role = lane & 1;
      const uint32_t w1 = ((D[0] << 5) | (D[1] << 2) | ((D[2] >> 1) & 0x03030303u)) ^ 0x80808080u ^ 0x10101010u ^ 0x02020202u;
      const uint32_t mine = role ? (((D[3] << 2) ^ 0x10101010u) | ((D[2] & 0x01010101u) << 1))
                                 : (((D[3] << 5) ^ 0x80808080u) | (D[2] & 0x01010101u));
      const uint32_t other = __shfl_xor(mine, 1, kWave);
      if (lane_ok) {
        uint32_t* p = reinterpret_cast<uint32_t*>(out + (lane >> 1) * 12 + role * 4);
        p[0] = w1;
        if (role) p[1] = mine | other;
      }
    }
  }
}

template <int BITS>
__global__ void __launch_bounds__(128) kv_dequant_kernel(const uint8_t* codes, int64_t T, int32_t d, const KvPos* pos,
                                                         uint16_t* out, int32_t blocks_per_row) {
  typedef float f2 __attribute__((ext_vector_type(2)));
  typedef __bf16 b2 __attribute__((ext_vector_type(2)));
  constexpr int GB = BITS * 4;                         // bytes of a 32-code group
  const int groups = d / kGroup;
  const int gi = (blockIdx.x % blocks_per_row) * 128 + threadIdx.x;       // this thread's group, the same for every row
  if (gi >= groups) return;
  float s[32], zf[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const KvPos kp = pos[gi * kGroup + j];
    s[j] = kp.s;
    zf[j] = static_cast<float>(kp.z);
  }
  const int64_t row_bytes = static_cast<int64_t>(d) * BITS / 8;
  const int64_t stride = gridDim.x / blocks_per_row;
  // the next row's codes are requested before this row is expanded (rows past the end: the last row again)
  auto load_row = [&](int64_t row, uint32_t (&w)[GB / 4]) {
    if (row >= T) row = T - 1;
    const uint32_t* p = reinterpret_cast<const uint32_t*>(codes + row * row_bytes + static_cast<int64_t>(gi) * GB);
    if constexpr (BITS == 3) {
      w[0] = p[0]; w[1] = p[1]; w[2] = p[2];
    } else {
#pragma unroll
      for (int k = 0; k < GB / 16; ++k) {
        const uint4 v = reinterpret_cast<const uint4*>(p)[k];
        w[4 * k] = v.x; w[4 * k + 1] = v.y; w[4 * k + 2] = v.z; w[4 * k + 3] = v.w;
      }
    }
  };
  uint32_t w[GB / 4], wn[GB / 4];
  int64_t row = blockIdx.x / blocks_per_row;
  load_row(row, w);
  for (; row < T; row += stride) {
    load_row(row + stride, wn);
    int q[32];
    decode_group<BITS>(w, q);
    uint32_t o[16];
#pragma unroll
    for (int j = 0; j < 32; j += 2) {
      // s (x_q - z): the integer difference is exact in fp32, one rounded product, then bf16 (ties to even)
      const f2 pr = {__fmul_rn(s[j], static_cast<float>(q[j]) - zf[j]), __fmul_rn(s[j + 1], static_cast<float>(q[j + 1]) - zf[j + 1])};
      const b2 cv = __builtin_convertvector(pr, b2);
      o[j / 2] = *reinterpret_cast<const uint32_t*>(&cv);
    }
    uint4* dst = reinterpret_cast<uint4*>(out + row * d + static_cast<int64_t>(gi) * kGroup);
#pragma unroll
    for (int k = 0; k < 4; ++k) dst[k] = make_uint4(o[4 * k], o[4 * k + 1], o[4 * k + 2], o[4 * k + 3]);
#pragma unroll
    for (int k = 0; k < GB / 4; ++k) w[k] = wn[k];
  }
}

int32_t launch_kv_quant(const void* x, int64_t T, int32_t d, const KvPos* pos, int32_t bits, void* codes, hipStream_t st) {
  if (T == 0) return RPTQ_OK;
  int cus = 0;
  if (int32_t s = device_compute_units(st, &cus)) return s;
  const int segs = (d + kKvTile - 1) / kKvTile;
  // about eight workgroups of four waves per compute unit, but at least 32 rows per wave while the
  // batch allows (a wave's per-lane constants cost as much as eight rows of input); every workgroup
  // keeps one tile column
  int64_t row_groups = (static_cast<int64_t>(cus) * 8 + segs - 1) / segs;
  row_groups = std::min<int64_t>(row_groups, std::max<int64_t>((T + 127) / 128, (static_cast<int64_t>(cus) * 2 + segs - 1) / segs));
  row_groups = std::min<int64_t>(std::max<int64_t>(row_groups, 1), (T + 3) / 4);
  const dim3 grid(static_cast<unsigned>(segs * row_groups)), block(256);
  const uint4* xp = static_cast<const uint4*>(x);
  uint8_t* cp = static_cast<uint8_t*>(codes);
  if (bits == 3) hipLaunchKernelGGL(kv_quant_kernel<3>, grid, block, 0, st, xp, T, d, pos, cp, segs, static_cast<int>(row_groups));
  else if (bits == 4) hipLaunchKernelGGL(kv_quant_kernel<4>, grid, block, 0, st, xp, T, d, pos, cp, segs, static_cast<int>(row_groups));
  else hipLaunchKernelGGL(kv_quant_kernel<8>, grid, block, 0, st, xp, T, d, pos, cp, segs, static_cast<int>(row_groups));
  RPTQ_HIP(hipGetLastError());
  return RPTQ_OK;
}

int32_t launch_kv_dequant(const void* codes, int64_t T, int32_t d, const KvPos* pos, int32_t bits, void* out, hipStream_t st) {
  if (T == 0) return RPTQ_OK;
  int cus = 0;
  if (int32_t s = device_compute_units(st, &cus)) return s;
  const int blocks_per_row = (d / kGroup + 127) / 128;
  // (a thread's constants are 512 bytes: at least 16 rows per thread while the batch allows)
  int64_t rows_par = (static_cast<int64_t>(cus) * 16 + blocks_per_row - 1) / blocks_per_row;
  rows_par = std::min<int64_t>(rows_par, std::max<int64_t>((T + 15) / 16, (static_cast<int64_t>(cus) * 4 + blocks_per_row - 1) / blocks_per_row));
  rows_par = std::min<int64_t>(std::max<int64_t>(rows_par, 1), T);
  const dim3 grid(static_cast<unsigned>(blocks_per_row * rows_par)), block(128);
  const uint8_t* cp = static_cast<const uint8_t*>(codes);
  uint16_t* op = static_cast<uint16_t*>(out);
  if (bits == 3) hipLaunchKernelGGL(kv_dequant_kernel<3>, grid, block, 0, st, cp, T, d, pos, op, blocks_per_row);
  else if (bits == 4) hipLaunchKernelGGL(kv_dequant_kernel<4>, grid, block, 0, st, cp, T, d, pos, op, blocks_per_row);
  else hipLaunchKernelGGL(kv_dequant_kernel<8>, grid, block, 0, st, cp, T, d, pos, op, blocks_per_row);
  RPTQ_HIP(hipGetLastError());
  return RPTQ_OK;
}

}  // namespace rptq
