// LayerNorm emitted in cluster order + per-cluster asymmetric quantization + bit packing
// (Sec. 4.2 "fuse the reorder into layer norm"; Eq. 1; App. A.4 first equation).
//
// One workgroup owns whole rows and walks them in a grid-stride loop.  Its last wave is the
// statistics wave, all others are unit waves: a unit thread owns the same output units
// (8 codes, or 16 for 3-bit) for every row, so everything that does not depend on the row -
// source channel, gamma', beta', the cluster's quantizer constants - sits in registers.
// The loop is pipelined over rows with one barrier per row.  Before the barrier the unit
// threads put the next row into LDS (coalesced 16-byte loads, issued one iteration earlier)
// and leave their exact fp64 partial sums there.  After it the statistics wave turns those
// into the next row's mean and 1/std while the unit waves gather the current row through LDS
// in cluster order, run the fp32 LayerNorm chain, round/offset/clamp, pack and store.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "device_common.h"
#include "pack_formats.h"
#include "rptq_internal.h"

namespace rptq {

// 16 bytes as a plain vector value (copies of the runtime's uint4 struct are memory copies, which can keep
// register arrays in scratch memory)
typedef unsigned u4v __attribute__((ext_vector_type(4)));

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
  int32_t ring;            // row buffers in LDS: 3, or 2 (one more barrier per row) when three do not fit
};

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

// LDS: `ring` row buffers (bf16 row + a 16-byte slot for surplus lanes), then per parity the
// partial sums of the unit threads ({S1, S2} and the de-quantized row sum), then per parity
// {mean, 1/std}.
struct LnLds {
  int rowbuf_bytes;
  int part12, part3, bcast;          // byte offsets
};
// Row-buffer stride of the kernels with compile-time buffer offsets: the offset of the third
// buffer still fits the 16-bit offset field of an LDS instruction.
constexpr int kFixedStride = 32752;
__host__ __device__ inline LnLds ln_lds_layout(int d, int ring, int tu, bool fixed = false) {
  LnLds l;
  l.rowbuf_bytes = fixed ? kFixedStride : d * 2 + 16;
  l.part12 = ring * l.rowbuf_bytes;
  l.part3 = l.part12 + 2 * tu * 16;
  l.bcast = l.part3 + 2 * tu * 8;
  return l;
}

// No load of this kernel sits under a lane-dependent branch: indices are clamped and what a
// surplus lane computes is masked or never stored.  (A load under a divergent branch makes
// the compiler wait for every load in flight at each such branch, which serializes them.)
//
// FIXED (wide LayerNorm rows, three row buffers at the constant stride kFixedStride): the row loop
// is unrolled over the three buffers, so a gather read carries its buffer's offset in the
// instruction instead of adding it to the address, and the 16-bit reads land in the upper half of
// their registers (the bf16 value as fp32, no shift).  Two vector instructions less per element.
template <int BITS, int NUNIT, int NCH, bool LN, bool FIXED = false>
__global__ void __launch_bounds__(1024) ln_quant_kernel(LnQuantArgs a, ClusterGeom geom, QuantTab qt) {
  constexpr int UC = Unit<BITS>::kCodes;
  constexpr int ND = UC / 4;                       // dwords of biased code bytes per unit
  constexpr float kUMax = static_cast<float>((1 << BITS) - 1);
  constexpr int kQMin = -(1 << (BITS - 1));

  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wid = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform by construction
  const int TU = static_cast<int>(blockDim.x) - kWave;          // unit threads; the last wave does the statistics
  const int nwu = TU >> 6;
  const bool stats_wave = wid == nwu;
  const LnLds lds = ln_lds_layout(a.d, a.ring, TU, FIXED);
  double* part12 = reinterpret_cast<double*>(smem + lds.part12);   // [2][TU][2]
  double* part3 = reinterpret_cast<double*>(smem + lds.part3);     // [2][TU]
  float* bcast = reinterpret_cast<float*>(smem + lds.bcast);       // [2][2]

  const int64_t row0 = blockIdx.x;
  const int64_t stride = gridDim.x;
  const int n_rows = static_cast<int>((a.M - row0 + stride - 1) / stride);   // >= 1: the grid has at most M workgroups

  // Sum of the unit threads' partials in a fixed order: per lane over the waves, then over the lanes.
  // One pass of the statistics wave: {S1, S2} of the row staged last (parity pb_stats) and the
  // de-quantized sum of the row stored last (parity pb_rt) are reduced together, so that the
  // three dependent chains overlap; fixed summation order (per lane over the unit waves, then
  // over the lanes).
  auto finalize = [&](bool do_stats, int pb_stats, bool do_rt, int pb_rt, int64_t rt_row) {
    double s1 = 0.0, s2 = 0.0, s3 = 0.0;
    const double* p12 = part12 + (static_cast<size_t>(pb_stats) * TU + lane) * 2;
    const double* p3 = part3 + static_cast<size_t>(pb_rt) * TU + lane;
    for (int j = 0; j < nwu; j += 4) {                            // four reads in flight; surplus slots re-read wave 0
      double2 v[4];
      double r[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int jj = (j + k) < nwu ? (j + k) : 0;
        v[k] = *reinterpret_cast<const double2*>(p12 + jj * 128);
        r[k] = p3[jj * 64];
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const bool in = (j + k) < nwu;
        s1 += in ? v[k].x : 0.0;
        s2 += in ? v[k].y : 0.0;
        s3 += in ? r[k] : 0.0;
      }
    }
    const double t1 = wave_sum(s1), t2 = wave_sum(s2), t3 = wave_sum(s3);
    if (LN && do_stats) {
      float mu, rstd;
      row_stats(t1, t2, a.d, a.eps, &mu, &rstd);
      if (lane == 0) {
        bcast[pb_stats * 2 + 0] = mu;
        bcast[pb_stats * 2 + 1] = rstd;
      }
    }
    if (do_rt && lane == 0 && a.rowterm) a.rowterm[rt_row] = static_cast<float>(t3);
  };

  if (stats_wave) {
    // ---- statistics wave ---------------------------------------------------------------------
    // Its dependent chain per row must stay shorter than the unit waves' work on a row: it
    // issues ahead of the unit waves that share its SIMD.
    __builtin_amdgcn_s_setprio(3);
    __syncthreads();                                           // row 0 staged
    finalize(true, 0, false, 0, 0);
    for (int i = 0; i < n_rows; ++i) {
      __syncthreads();                                         // row i+1 staged, row i-1 stored
      finalize(true, (i + 1) & 1, i >= 1, (i - 1) & 1, row0 + (i - 1) * stride);
      if (a.ring == 2) __syncthreads();
    }
    __syncthreads();
    finalize(false, 0, true, (n_rows - 1) & 1, row0 + (n_rows - 1) * stride);
    return;
  }

  // ---- this thread's 16-byte chunks of an input row ---------------------------------------
  int ch_idx[NCH];                   // chunk index, clamped for surplus lanes
  int ch_lds[NCH];                   // LDS byte offset inside a row buffer (surplus lanes: the spare slot)
  bool ch_ok[NCH];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int idx = tid + c * TU;
    ch_ok[c] = idx < a.chunks;
    ch_idx[c] = ch_ok[c] ? idx : a.chunks - 1;
    ch_lds[c] = ch_ok[c] ? idx * 16 : a.d * 2;
  }
  // Two register sets hold input rows on their way from HBM: the row staged in iteration i
  // (row i+1) was requested two iterations earlier, so that two rows per workgroup are in
  // flight at any time (with one, the bytes in flight per compute unit bound the kernel at
  // about 3 TB/s: one row of 24 KB per 2 us of loaded-memory latency).
  // (with four chunks per thread a second set does not fit the 128 registers: one row in flight)
  constexpr bool kDeep = NCH <= 2;
  u4v nxa[NCH], nxb[kDeep ? NCH : 1];
  auto fetch_row = [&](int k, u4v* dst) {          // k-th row of this workgroup; past the end: a valid row again
    int64_t row = row0 + k * stride;
    if (row >= a.M) row = a.M - 1;
    const u4v* p = reinterpret_cast<const u4v*>(a.x + row * a.chunks);
#pragma unroll
    for (int c = 0; c < NCH; ++c) dst[c] = p[ch_idx[c]];
  };
  // the first rows are requested before anything else, so that their latency runs under the
  // loads of the per-thread constants below instead of after them
  fetch_row(0, nxa);
  if (kDeep) fetch_row(1, nxb);

  // ---- unit waves: per-thread constants, loaded once -----------------------------------------
  uint32_t src[NUNIT][UC];           // LDS byte offsets of the source channels inside a row buffer
  float gam[LN ? NUNIT : 1][LN ? UC : 1];
  float bet[LN ? NUNIT : 1][LN ? UC : 1];
  float inv_s[NUNIT], zbf[NUNIT];
  double sdq[NUNIT];                 // cluster scale, for the de-quantized row sum
  int32_t usum_fix[NUNIT];           // turns the sum of biased bytes into sum of (q - z) over real codes
  uint32_t keep[NUNIT][ND], fill[NUNIT][ND];
  bool unit_ok[NUNIT];
  int64_t out_off[NUNIT];

#pragma unroll
  for (int n = 0; n < NUNIT; ++n) {
    const int u = tid + n * TU;
    unit_ok[n] = u < a.n_units;
    const int uu = unit_ok[n] ? u : 0;             // surplus lanes redo unit 0 and store nothing
    int gbase, role = 0;
    if (BITS == 3) {
      gbase = (uu >> 1) * kGroup;
      role = uu & 1;
      out_off[n] = static_cast<int64_t>(uu >> 1) * 12 + role * 4;
    } else {
      gbase = uu * 8;
      out_off[n] = static_cast<int64_t>(uu) * BITS;
    }
    int ci = 0;
    for (int i = 1; i < geom.g; ++i) ci += (gbase >= geom.pad_off[i]) ? 1 : 0;
    inv_s[n] = qt.inv_s[ci];
    zbf[n] = static_cast<float>(qt.zb[ci]);
    sdq[n] = static_cast<double>(qt.s[ci]);
    // the unit's positions are runs of four consecutive padded positions: 16-byte loads
    int32_t pc[UC];
    float pg[UC], pb[UC];
#pragma unroll
    for (int v = 0; v < UC / 4; ++v) {
      const int pos = (BITS == 3) ? gbase + pos3(role, v * 4) : gbase + v * 4;
      const int4 c4 = *reinterpret_cast<const int4*>(a.perm_pad + pos);
      pc[v * 4 + 0] = c4.x; pc[v * 4 + 1] = c4.y; pc[v * 4 + 2] = c4.z; pc[v * 4 + 3] = c4.w;
      if (LN) {
        const float4 g4 = *reinterpret_cast<const float4*>(a.gamma_pad + pos);
        const float4 b4 = *reinterpret_cast<const float4*>(a.beta_pad + pos);
        pg[v * 4 + 0] = g4.x; pg[v * 4 + 1] = g4.y; pg[v * 4 + 2] = g4.z; pg[v * 4 + 3] = g4.w;
        pb[v * 4 + 0] = b4.x; pb[v * 4 + 1] = b4.y; pb[v * 4 + 2] = b4.z; pb[v * 4 + 3] = b4.w;
      }
    }
    int n_real = 0;
#pragma unroll
    for (int w = 0; w < ND; ++w) { keep[n][w] = 0xffffffffu; fill[n][w] = 0u; }
#pragma unroll
    for (int e = 0; e < UC; ++e) {
      const bool real = pc[e] >= 0;
      n_real += real ? 1 : 0;
      const uint32_t off = real ? static_cast<uint32_t>(pc[e]) * 2u : 0u;
      src[n][e] = off;
      if (LN) {
        gam[n][e] = real ? pg[e] : 0.0f;
        bet[n][e] = real ? pb[e] : 0.0f;
      }
      if (!real) {                                 // pad position: force code 0 (biased byte = -qmin)
        keep[n][e / 4] &= ~(0xffu << (8 * (e & 3)));
        fill[n][e / 4] |= static_cast<uint32_t>(-kQMin) << (8 * (e & 3));
      }
    }
    usum_fix[n] = UC * kQMin - n_real * qt.z[ci];
  }

  // registers -> row buffer, exact fp64 sums of this thread's elements -> partials
  auto stage_row = [&](const u4v* regs, unsigned char* rowbuf, int pb) {
    double s1 = 0.0, s2 = 0.0;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      u4v v = regs[c];
      *reinterpret_cast<u4v*>(rowbuf + ch_lds[c]) = v;
      if (LN) {
        if (!ch_ok[c]) v = u4v{0u, 0u, 0u, 0u};              // surplus lane: contributes nothing
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
    if (LN) *reinterpret_cast<double2*>(part12 + (static_cast<size_t>(pb) * TU + tid) * 2) = make_double2(s1, s2);
  };

  // ReLU commutes with the rounding and with the (monotonic, exact) addition of the zero point:
  // max(y, 0) before Eq. 1 equals a lower clamp of the biased code at the biased zero point, which
  // shares one median-of-three instruction with the upper clamp.
  float code_floor[NUNIT];
#pragma unroll
  for (int n = 0; n < NUNIT; ++n) code_floor[n] = a.relu ? fminf(zbf[n], kUMax) : -__builtin_huge_valf();   // (zero points beyond the range: floor at the top code)

  // ---- pipelined row loop --------------------------------------------------------------------
  int b_cur = 0, b_next = lds.rowbuf_bytes, b_spare = (a.ring == 3) ? 2 * lds.rowbuf_bytes : 0;
  stage_row(nxa, smem + b_cur, 0);
  fetch_row(kDeep ? 2 : 1, nxa);
  __syncthreads();                                             // row 0 staged

  // one iteration: stage row i+1 from `regs`, request the next row they will hold (i+3, or
  // i+2 with one set), then gather row i
  // destination registers of the upper-half LDS reads (FIXED): only those reads ever write them
  uint32_t hreg[FIXED ? NUNIT : 1][FIXED ? UC : 1];
#pragma unroll
  for (int n = 0; n < (FIXED ? NUNIT : 1); ++n)
#pragma unroll
    for (int e = 0; e < (FIXED ? UC : 1); ++e) hreg[n][e] = 0u;

  // bc_tag: the row buffer that holds row i when it is known at compile time (FIXED), else -1
  auto row_iter = [&](int i, u4v* regs, auto bc_tag) {
    constexpr int BC = decltype(bc_tag)::value;
    const int cur_off = BC >= 0 ? BC * kFixedStride : b_cur;
    const int next_off = BC >= 0 ? ((BC + 1) % 3) * kFixedStride : b_next;
    stage_row(regs, smem + next_off, (i + 1) & 1);
    fetch_row(i + (kDeep ? 3 : 2), regs);
    __syncthreads();                                           // row i+1 staged; {mean, 1/std} of row i published
    const unsigned char* rowbuf = smem + cur_off;
    float mu = 0.0f, rstd = 1.0f;
    if (LN) {
      const float2 ms = *reinterpret_cast<const float2*>(bcast + (i & 1) * 2);
      mu = ms.x;
      rstd = ms.y;
    }
    if constexpr (BC >= 0) {
      // all of this thread's source values at once; the wait below also ties every later use of
      // the registers to the reads' completion
#pragma unroll
      for (int n = 0; n < NUNIT; ++n)
#pragma unroll
        for (int e = 0; e < UC; ++e)
          asm volatile("ds_read_u16_d16_hi %0, %1 offset:%2" : "+v"(hreg[n][e]) : "v"(src[n][e]), "n"(BC * kFixedStride));
      static_assert(!FIXED || NUNIT * UC == 16, "sixteen source values per thread");
      uint32_t(&h)[FIXED ? NUNIT : 1][FIXED ? UC : 1] = hreg;
      constexpr int U = FIXED ? UC : 1;
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(h[0 / U][0 % U]), "+v"(h[1 / U][1 % U]), "+v"(h[2 / U][2 % U]), "+v"(h[3 / U][3 % U]),
                     "+v"(h[4 / U][4 % U]), "+v"(h[5 / U][5 % U]), "+v"(h[6 / U][6 % U]), "+v"(h[7 / U][7 % U]),
                     "+v"(h[8 / U][8 % U]), "+v"(h[9 / U][9 % U]), "+v"(h[10 / U][10 % U]), "+v"(h[11 / U][11 % U]),
                     "+v"(h[12 / U][12 % U]), "+v"(h[13 / U][13 % U]), "+v"(h[14 / U][14 % U]), "+v"(h[15 / U][15 % U]));
    }
    const int64_t row = row0 + i * stride;

    // ---- gather in cluster order, normalize, quantize, pack ------------------------
    double rt = 0.0;
    uint8_t* out_row = a.codes + row * a.row_bytes;
#pragma unroll
    for (int n = 0; n < NUNIT; ++n) {
      uint32_t D[ND];
#pragma unroll
      for (int w = 0; w < ND; ++w) D[w] = 0u;
#pragma unroll
      for (int e = 0; e < UC; ++e) {
        float y;
        if constexpr (BC >= 0) {
          y = __uint_as_float(hreg[n][e]);
        } else {
          const uint32_t h = *reinterpret_cast<const uint16_t*>(rowbuf + src[n][e]);
          y = __uint_as_float(h << 16);
        }
        if (LN) y = ln_chain(y, mu, rstd, gam[n][e], bet[n][e]);
        const float r = __fmul_rn(y, inv_s[n]);
        float b = __fadd_rn(rintf(r), zbf[n]);          // round, then add the zero point (biased by -qmin)
        // ReLU floor (or -inf) and upper clamp; the conversion saturates at 0 and 255
        b = (BITS < 8) ? __builtin_amdgcn_fmed3f(b, code_floor[n], kUMax) : fmaxf(b, code_floor[n]);
        D[e / 4] = __builtin_amdgcn_cvt_pk_u8_f32(b, e & 3, D[e / 4]);
      }
#pragma unroll
      for (int w = 0; w < ND; ++w) D[w] = (D[w] & keep[n][w]) | fill[n][w];      // pad positions: code 0
      uint32_t usum = 0;
#pragma unroll
      for (int w = 0; w < ND; ++w) usum = __builtin_amdgcn_sad_u8(D[w], 0u, usum);
      const double part = sdq[n] * static_cast<double>(static_cast<int32_t>(usum) + usum_fix[n]);
      rt += unit_ok[n] ? part : 0.0;

      if (BITS == 8) {
        uint2 o;
        o.x = D[0] ^ 0x80808080u;
        o.y = D[1] ^ 0x80808080u;
        if (unit_ok[n]) *reinterpret_cast<uint2*>(out_row + out_off[n]) = o;
      } else if (BITS == 4) {
        const uint32_t o = ((D[0] << 4) | D[1]) ^ 0x88888888u;
        if (unit_ok[n]) *reinterpret_cast<uint32_t*>(out_row + out_off[n]) = o;
      } else {
        // role 0 -> x0 and its half of x2; role 1 -> x1 and its half of x2 (partner = lane ^ 1)
        const uint32_t w1 = ((D[0] << 5) | (D[1] << 2) | ((D[2] >> 1) & 0x03030303u)) ^ 0x80808080u ^ 0x10101010u ^ 0x02020202u;
        const int role = tid & 1;
        const uint32_t mine = role ? (((D[3] << 2) ^ 0x10101010u) | ((D[2] & 0x01010101u) << 1))
                                   : (((D[3] << 5) ^ 0x80808080u) | (D[2] & 0x01010101u));
        const uint32_t other = __shfl_xor(mine, 1, kWave);
        if (unit_ok[n]) {
          uint32_t* p = reinterpret_cast<uint32_t*>(out_row + out_off[n]);
          p[0] = w1;
          if (role) p[1] = mine | other;
        }
      }
    }
    part3[static_cast<size_t>(i & 1) * TU + tid] = rt;
    if (BC >= 0) return;
    if (a.ring == 2) {
      __syncthreads();                                         // two row buffers only: all gathers done before the next staging
      const int t = b_cur; b_cur = b_next; b_next = t;
    } else {
      const int t = b_cur; b_cur = b_next; b_next = b_spare; b_spare = t;
    }
  };
  using B0 = std::integral_constant<int, 0>;
  using B1 = std::integral_constant<int, 1>;
  using B2 = std::integral_constant<int, 2>;
  using BR = std::integral_constant<int, -1>;
  if (kDeep) {
    int i = 0;
    if (FIXED) {                                               // six rows per pass: 2 register sets x 3 buffers
      for (; i + 5 < n_rows; i += 6) {
        row_iter(i, nxb, B0());
        row_iter(i + 1, nxa, B1());
        row_iter(i + 2, nxb, B2());
        row_iter(i + 3, nxa, B0());
        row_iter(i + 4, nxb, B1());
        row_iter(i + 5, nxa, B2());
      }
      // (the last rows take the run-time offsets below, which start at buffer 0 again)
    }
    for (; i + 1 < n_rows; i += 2) {                           // row i+1 waits in nxb, row i+2 in nxa
      row_iter(i, nxb, BR());
      row_iter(i + 1, nxa, BR());
    }
    if (i < n_rows) row_iter(i, nxb, BR());
  } else {
    for (int i = 0; i < n_rows; ++i) row_iter(i, nxa, BR());
  }
  __syncthreads();                                             // last row's partial sums are in LDS
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

// De-quantized row sum of every cluster, rtc[t, i] = sX_i (sum_{c in i} xq[t,c] - n_i zX_i): what the
// zero-point cross term of App. A.4 needs per (token, cluster) when the weights carry one
// zero point per (output, cluster).  One wave per row; a 32-code group lies inside one
// cluster, so a lane adds whole groups into the cluster's integer sum (exact, order-free).
// Output position of cluster i in a row of g2 floats: (i & 1) * g2/2 + i/2 (the operand order
// of the 32x32x2 fp32 MFMA that consumes it).
struct RowSumTab {
  double s[RPTQ_MAX_CLUSTERS];
  double nz[RPTQ_MAX_CLUSTERS];        // n_i * zX_i
};

template <int BITS>
__global__ void __launch_bounds__(256) cluster_rowsums_kernel(const uint8_t* codes, int64_t M, int32_t row_bytes,
                                                              ClusterGeom geom, RowSumTab tab, float* rtc, int32_t g2) {
  constexpr int GB = BITS * 4;
  __shared__ int32_t acc[4][RPTQ_MAX_CLUSTERS];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + wave;
  if (lane < RPTQ_MAX_CLUSTERS) acc[wave][lane] = 0;
  __builtin_amdgcn_wave_barrier();
  if (row < M) {
    const int groups = geom.pad_off[geom.g] / kGroup;
    for (int gi = lane; gi < groups; gi += kWave) {
      const uint32_t* p = reinterpret_cast<const uint32_t*>(codes + row * row_bytes + static_cast<int64_t>(gi) * GB);
      uint32_t w[GB / 4];
#pragma unroll
      for (int k = 0; k < GB / 4; ++k) w[k] = p[k];
      int q[32];
      decode_group<BITS>(w, q);
      int sum = 0;
#pragma unroll
      for (int j = 0; j < 32; ++j) sum += q[j];
      int ci = 0;
      for (int i = 1; i < geom.g; ++i) ci += (gi * kGroup >= geom.pad_off[i]) ? 1 : 0;
      atomicAdd(&acc[wave][ci], sum);
    }
  }
  __builtin_amdgcn_wave_barrier();
  if (row < M && lane < g2) {
    float v = 0.0f;
    if (lane < geom.g) v = static_cast<float>(tab.s[lane] * (static_cast<double>(acc[wave][lane]) - tab.nz[lane]));
    rtc[row * g2 + (lane & 1) * (g2 / 2) + (lane >> 1)] = v;
  }
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
constexpr int kMaxChunk = 4;   // 16-byte chunks of the input row per unit thread
constexpr int kMaxUnitThreads = 1024 - kWave;

template <int BITS, int NUNIT, int NCH, bool LN, bool FIXED = false>
static int32_t launch_kernel(const LnQuantArgs& a, const ClusterGeom& geom, const QuantTab& qt, int threads,
                             int64_t want_grid, int lds_per_cu, size_t shmem, hipStream_t st) {
  auto kern = ln_quant_kernel<BITS, NUNIT, NCH, LN, FIXED>;
  static LdsGrant lds_granted;
  if (int32_t st_lds = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), shmem, &lds_granted, st)) return st_lds;
  // workgroups resident per compute unit (registers, threads, LDS); the grid is one full round
  static OccupancyMemo occupancy;
  int per_cu = 1;
  if (int32_t st_occ = resident_workgroups(reinterpret_cast<const void*>(kern), threads, shmem, &occupancy, st, &per_cu))
    return st_occ;
  (void)lds_per_cu;
  const int64_t grid = std::min<int64_t>(a.M, want_grid * per_cu);
  hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(grid)), dim3(threads), shmem, st, a, geom, qt);
  RPTQ_HIP(hipGetLastError());
  return RPTQ_OK;
}

template <int BITS, int NUNIT, bool LN>
static int32_t launch_chunks(const LnQuantArgs& a, const ClusterGeom& geom, const QuantTab& qt, int nch, int threads,
                             int64_t cus, int lds_per_cu, size_t shmem, hipStream_t st) {
  if constexpr (LN && BITS == 3 && NUNIT == 1) {       // (the 4- and 8-bit kernels with two units per thread would spill)
    // wide LayerNorm rows (one workgroup per compute unit either way): the variant with compile-time
    // row-buffer offsets, when its three buffers at the fixed stride fit
    const int rowbuf = a.d * 2 + 16;
    const LnLds lay = ln_lds_layout(a.d, 3, threads - kWave, true);
    const size_t shmem_fixed = static_cast<size_t>(lay.bcast) + 16;
    if (a.ring == 3 && nch <= 2 && rowbuf > kFixedStride / 2 && rowbuf <= kFixedStride &&
        shmem_fixed <= static_cast<size_t>(lds_per_cu)) {
      if (nch <= 1) return launch_kernel<BITS, NUNIT, 1, true, true>(a, geom, qt, threads, cus, lds_per_cu, shmem_fixed, st);
      return launch_kernel<BITS, NUNIT, 2, true, true>(a, geom, qt, threads, cus, lds_per_cu, shmem_fixed, st);
    }
  }
  if (nch <= 1) return launch_kernel<BITS, NUNIT, 1, LN>(a, geom, qt, threads, cus, lds_per_cu, shmem, st);
  if (nch == 2) return launch_kernel<BITS, NUNIT, 2, LN>(a, geom, qt, threads, cus, lds_per_cu, shmem, st);
  return launch_kernel<BITS, NUNIT, kMaxChunk, LN>(a, geom, qt, threads, cus, lds_per_cu, shmem, st);
}

// With LayerNorm a thread keeps gamma' and beta' of its units in registers: at most two units
// (one of 16 codes at 3 bits); without, up to four (two).
template <int BITS>
static int32_t launch_bits(const LnQuantArgs& a, const ClusterGeom& geom, const QuantTab& qt, bool ln, int nunit,
                           int nch, int threads, int64_t cus, int lds_per_cu, size_t shmem, hipStream_t st) {
  if constexpr (BITS == 3) {
    if (ln) return launch_chunks<3, 1, true>(a, geom, qt, nch, threads, cus, lds_per_cu, shmem, st);
    if (nunit == 1) return launch_chunks<3, 1, false>(a, geom, qt, nch, threads, cus, lds_per_cu, shmem, st);
    return launch_chunks<3, 2, false>(a, geom, qt, nch, threads, cus, lds_per_cu, shmem, st);
  } else {
    if (ln) {
      if (nunit == 1) return launch_chunks<BITS, 1, true>(a, geom, qt, nch, threads, cus, lds_per_cu, shmem, st);
      return launch_chunks<BITS, 2, true>(a, geom, qt, nch, threads, cus, lds_per_cu, shmem, st);
    }
    if (nunit == 1) return launch_chunks<BITS, 1, false>(a, geom, qt, nch, threads, cus, lds_per_cu, shmem, st);
    if (nunit == 2) return launch_chunks<BITS, 2, false>(a, geom, qt, nch, threads, cus, lds_per_cu, shmem, st);
    return launch_chunks<BITS, 4, false>(a, geom, qt, nch, threads, cus, lds_per_cu, shmem, st);
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

  // Unit threads: enough for the units (<= max_nunit per thread) and the input chunks
  // (<= kMaxChunk per thread), a multiple of the wave size, as few idle lanes as possible.
  const bool ln = gamma_pad != nullptr;
  // register budget: per-unit constants of more units than this would spill
  const int max_nunit = ln ? (bits == 3 ? 1 : 2) : (bits == 3 ? 2 : 4);
  int best_t = 0, best_n = 0;
  double best_waste = 1e30;
  for (int nunit = 1; nunit <= max_nunit; ++nunit) {
    if (nunit == 3) continue;                      // instantiated: 1, 2, 4
    int t = (a.n_units + nunit - 1) / nunit;
    t = (t + kWave - 1) / kWave * kWave;
    const int t_chunks = ((a.chunks + kMaxChunk - 1) / kMaxChunk + kWave - 1) / kWave * kWave;
    if (t < t_chunks) t = t_chunks;
    if (t > kMaxUnitThreads) continue;
    if (t < 256 && nunit > 1) continue;
    const double waste = static_cast<double>(t) * nunit / a.n_units;
    if (waste < best_waste - 1e-9) {
      best_waste = waste;
      best_t = t;
      best_n = nunit;
    }
  }
  if (best_t == 0) return RPTQ_ERR_SHAPE;
  const int nch = (a.chunks + best_t - 1) / best_t;          // 1, 2 or 3..4 (run as 4)

  int cus = 0;                                     // compute units of the current device
  if (int32_t st_cu = device_compute_units(st, &cus)) return st_cu;
  const int lds_cu = 160 * 1024;
  a.ring = 3;
  LnLds lay = ln_lds_layout(d, 3, best_t);
  size_t shmem = static_cast<size_t>(lay.bcast) + 16;
  if (shmem > static_cast<size_t>(lds_cu)) {
    a.ring = 2;
    lay = ln_lds_layout(d, 2, best_t);
    shmem = static_cast<size_t>(lay.bcast) + 16;
  }
  if (shmem > static_cast<size_t>(lds_cu)) return RPTQ_ERR_SHAPE;
  const int threads = best_t + kWave;

  int32_t stt;
  if (bits == 3) stt = launch_bits<3>(a, geom, qt, ln, best_n, nch, threads, cus, lds_cu, shmem, st);
  else if (bits == 4) stt = launch_bits<4>(a, geom, qt, ln, best_n, nch, threads, cus, lds_cu, shmem, st);
  else stt = launch_bits<8>(a, geom, qt, ln, best_n, nch, threads, cus, lds_cu, shmem, st);
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

int32_t launch_cluster_rowsums(const void* codes, int64_t M, const ClusterGeom& geom, int32_t bits, const float* sX,
                               const int32_t* zX, float* rtc, hipStream_t st) {
  if (M == 0) return RPTQ_OK;
  RowSumTab tab;
  for (int i = 0; i < RPTQ_MAX_CLUSTERS; ++i) {
    const bool in = i < geom.g;
    tab.s[i] = in ? static_cast<double>(sX[i]) : 0.0;
    tab.nz[i] = in ? static_cast<double>(geom.off[i + 1] - geom.off[i]) * static_cast<double>(zX[i]) : 0.0;
  }
  const int g2 = geom.g <= 32 ? 32 : 64;
  const uint8_t* c = static_cast<const uint8_t*>(codes);
  const int32_t row_bytes = geom.k_padded * bits / 8;
  const dim3 grid(static_cast<unsigned>((M + 3) / 4)), block(256);
  if (bits == 3) hipLaunchKernelGGL(cluster_rowsums_kernel<3>, grid, block, 0, st, c, M, row_bytes, geom, tab, rtc, g2);
  else if (bits == 4) hipLaunchKernelGGL(cluster_rowsums_kernel<4>, grid, block, 0, st, c, M, row_bytes, geom, tab, rtc, g2);
  else hipLaunchKernelGGL(cluster_rowsums_kernel<8>, grid, block, 0, st, c, M, row_bytes, geom, tab, rtc, g2);
  RPTQ_HIP(hipGetLastError());
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
