// Cluster-wise integer product (App. A.4, second method) on int8 MFMA.
//
// K runs over the padded cluster-order layout in slices of 32 codes, so a cluster always
// ends on a slice boundary.  Activation codes (3/4/8 bit, packed) go global -> registers ->
// int8 in LDS (code << 5, << 4 or << 0, one shift/mask per four codes) in the order the
// 32x32x32 int8 MFMA reads its operand.  Weight codes (4 bit, packed in MFMA-lane order) go
// global -> registers and are expanded to int8 (code << 4) in registers right before use:
// they never touch LDS, which would otherwise be the bandwidth limit of this kernel.
// The int32 accumulators hold 2^shift * P_i of the current cluster only: when the last slice
// of cluster i has been accumulated they are converted, scaled by sX_i / 2^shift, added to
// the fp32 result and cleared.  (Letting them run on as sums over clusters 1..i and adding
// (sX_i - sX_{i+1}) * sum saves the clearing, but the fp32 result then passes through
// intermediate values sX_{i+1} * sum that can be hundreds of times larger than the result
// when a late cluster has a large scale: at K = 20480 that cost three decimal digits.)
// The zero-point terms of App. A.4 are applied once at the end from per-row and per-column
// vectors.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "device_common.h"
#include "rptq_internal.h"
#include "gemm_common.h"

namespace rptq {

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

// OUT: what the output stage writes - kOutBf16 / kOutF32: Y; 3, 4 or 8: the next site's packed
// codes of that many bits (ReLU optional) and the partial row sums its product needs.
constexpr int kOutBf16 = 0, kOutF32 = 1;
// CWISE: the weights carry one (s, z) per (output channel, input cluster), as App. A.4 prints the
// scheme: the rescale of a finished cluster multiplies every output column by its own
// sX_i sW[o,i] (a table of the tile's columns in LDS), and the zero-point cross term
// sum_i sW[o,i] zW[o,i] * sX_i (xsum[t,i] - n_i zX_i) is a rank-g update of the fp32 tile, done
// on the matrix cores (32x32x2 fp32 MFMA) before the output stage.
template <int BITS, int WGM, int WGN, int WM, int WN, bool PARTIALS, int OUT, bool CWISE>
__global__ void __launch_bounds__(256, 2) cluster_gemm_kernel(GemmArgs a, GemmTab tab, GemmQuantOut qo) {
  constexpr bool YF32 = OUT == kOutF32;
  constexpr bool QOUT = OUT >= 2;
  constexpr int BM = WGM * WM * 32;
  constexpr int BN = WGN * WN * 32;
  constexpr int A_SLICE = 2 * BM * 16 + kSlicePad;       // [half][row][16 B]
  constexpr int A_STAGE = kStepSlices * A_SLICE;
  constexpr int A_UNITS = BM * kStepSlices;              // (row, slice) units per K step
  constexpr int A_PER = (A_UNITS + 255) / 256;
  constexpr int GB = ActFmt<BITS>::kGroupBytes;
  constexpr int A_REGS = GB / 4;                          // dwords per A unit

  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* sA = smem;                               // [2][A_STAGE]
  // behind the pipeline buffers / the output tile (they share the front of the LDS): the
  // per-channel and per-row terms of the output stage, fetched in the prologue
  constexpr int kStageBytes = PARTIALS ? 0 : BM * (BN + 4) * 4;
  constexpr int kConstOff = (2 * A_STAGE > kStageBytes) ? 2 * A_STAGE : kStageBytes;
  float* c_sw = reinterpret_cast<float*>(smem + kConstOff);   // [BN]
  float* c_ct = c_sw + BN;                                     // [BN]
  float* c_zw = c_ct + BN;                                     // [BN]
  float* c_rt = c_zw + BN;                                     // [BM]
  // CWISE: per-cluster scales of the tile's columns, [g][BN].  They are read during the main loop
  // only, so they live between the pipeline buffers and the vectors above when that gap (which
  // the output tile reuses afterwards) holds 32 clusters, else behind the vectors.
  constexpr int kCwBytes = 32 * BN * 4;
  constexpr bool kCwInGap = kConstOff - 2 * A_STAGE >= kCwBytes;
  float* c_sc = reinterpret_cast<float*>(smem + (kCwInGap ? 2 * A_STAGE : kConstOff + (3 * BN + BM) * 4));

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): give every XCD a
  // contiguous band of output columns, all row tiles of one column tile back to back.
  const int tiles_m = a.tiles_m, tiles_n = a.tiles_n;
  const int total = tiles_m * tiles_n;
  int lin = blockIdx.x;
  if (total % 8 == 0) lin = (lin & 7) * (total >> 3) + (lin >> 3);
  // The workgroups resident on an XCD at one time (64 with two per compute unit) should share
  // operands in its L2: blocks of grp_m row tiles x grp_n column tiles (16 x 4 tiles: 5 MB + 6.7 MB of
  // operands at K = 12288) rather than 64 row tiles x 1 column tile (20 MB + 1.7 MB).
  int tm = lin % tiles_m, tn = lin / tiles_m;
  const int GM = a.grp_m, GN = a.grp_n;
  if (GM > 0) {
    const int group = lin / (GN * tiles_m), rem = lin % (GN * tiles_m);
    const int wg = (tiles_n - GN * group) < GN ? (tiles_n - GN * group) : GN;      // column tiles of this group
    const int chunk = rem / (GM * wg), r = rem % (GM * wg);
    tm = chunk * GM + r / wg;
    tn = GN * group + r % wg;
  }
  const int64_t m0 = static_cast<int64_t>(tm) * BM;
  const int n0 = tn * BN;

  // ---- global -> register staging ------------------------------------------------------
  uint32_t ra[2][A_PER][A_REGS];                          // two staging sets: loads run ahead of use
  uint4 wreg[WN][kStepSlices / 2];                        // this lane's weight bytes of one K step: [block][slice pair]
  // Operands are read with buffer loads (a resource descriptor per workgroup, a 32-bit offset
  // per lane): next to a busy matrix pipe this path sustains about twice the bytes per clock of
  // loads that carry a 64-bit address per lane.
  typedef unsigned u4v __attribute__((ext_vector_type(4)));
  typedef unsigned u3v __attribute__((ext_vector_type(3)));
  constexpr int kRsrcFlags = 0x00020000;                   // raw buffer, 32-bit data format
  int a_off[A_PER], w_off[WN];                             // byte offsets inside the workgroup's operand windows
  int a_lds[A_PER];
  const int64_t rows_here = (a.M - m0) < BM ? (a.M - m0) : BM;             // rows of this tile that exist (>= 1)
#pragma unroll
  for (int i = 0; i < A_PER; ++i) {
    // surplus threads repeat a valid unit (same bytes to the same LDS address): no divergent
    // branches around the loads, so all of a step's loads are in flight together
    const int unit = (tid + i * 256) % A_UNITS;
    const int row = unit / kStepSlices, s = unit % kStepSlices;
    const int lrow = row < rows_here ? row : static_cast<int>(rows_here) - 1;   // clamp: rows past M are never stored
    a_off[i] = lrow * a.row_bytes + s * GB;
    a_lds[i] = s * A_SLICE + row * 16;
  }
  const int wblocks = a.slices / (kWBlockCols / kGroup);   // packed weight blocks per 32-row band
#pragma unroll
  for (int j = 0; j < WN; ++j) w_off[j] = (wn * WN + j) * wblocks * 2048 + lane * 16;
  const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(a.codes) + m0 * a.row_bytes, 0, static_cast<int>(rows_here) * a.row_bytes, kRsrcFlags);
  const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(a.Wq) + static_cast<size_t>(n0 / 32) * wblocks * 2048, 0, (BN / 32) * wblocks * 2048, kRsrcFlags);

  auto load_a_unit = [&](int step, int q, int i) {
    const int soff = step * (kStepSlices * GB);
    if (A_REGS == 3) {
      const u3v r = __builtin_amdgcn_raw_buffer_load_b96(a_rsrc, a_off[i], soff, 0);
#pragma unroll
      for (int k = 0; k < 3; ++k) ra[q][i][k % A_REGS] = r[k];
    } else {
#pragma unroll
      for (int h = 0; h < A_REGS / 4; ++h) {
        const u4v r = __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, a_off[i] + h * 16, soff, 0);
#pragma unroll
        for (int k = 0; k < 4; ++k) ra[q][i][(h * 4 + k) % A_REGS] = r[k];
      }
    }
  };
  auto load_a = [&](int step, int q) {
#pragma unroll
    for (int i = 0; i < A_PER; ++i) load_a_unit(step, q, i);
  };
  // one slice pair (32 bytes per lane) of weight block j
  auto load_w_pair = [&](int step, int j, int pi) {
    // (a wave's load of a slice pair is 1 KiB contiguous: eight whole cache lines)
    const u4v r = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, w_off[j],
                                                        (step * (kStepSlices / 4) + (pi >> 1)) * 2048 + (pi & 1) * 1024, 0);
    wreg[j][pi] = make_uint4(r[0], r[1], r[2], r[3]);
  };
  auto load_w = [&](int step) {
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int pi = 0; pi < kStepSlices / 2; ++pi) load_w_pair(step, j, pi);
  };

  // unpack one half (16 codes) of a staged unit to int8 and write it to LDS stage `buf`
  auto store_a_half = [&](int buf, int q, int i, int half) {
    unsigned char* dA = sA + buf * A_STAGE;
    uint4 v;
    if (BITS == 8) {
      v = half ? make_uint4(ra[q][i][4 % A_REGS], ra[q][i][5 % A_REGS], ra[q][i][6 % A_REGS], ra[q][i][7 % A_REGS])
               : make_uint4(ra[q][i][0], ra[q][i][1], ra[q][i][2], ra[q][i][3]);
    } else if (BITS == 4) {
      const uint32_t x = ra[q][i][half * 2], y = ra[q][i][half * 2 + 1];
      v = make_uint4(x & 0xf0f0f0f0u, (x << 4) & 0xf0f0f0f0u, y & 0xf0f0f0f0u, (y << 4) & 0xf0f0f0f0u);
    } else {
      const uint32_t x0 = ra[q][i][0], x1 = ra[q][i][1], x2 = ra[q][i][2];
      if (half == 0) {
        v = make_uint4(x0 & 0xe0e0e0e0u, (x0 << 3) & 0xe0e0e0e0u, x1 & 0xe0e0e0e0u, (x1 << 3) & 0xe0e0e0e0u);
      } else {
        v = make_uint4(x2 & 0xe0e0e0e0u, (x2 << 3) & 0xe0e0e0e0u,
                       ((x0 << 6) & 0xc0c0c0c0u) | ((x2 << 5) & 0x20202020u),
                       ((x1 << 6) & 0xc0c0c0c0u) | ((x2 << 4) & 0x20202020u));
      }
    }
    *reinterpret_cast<uint4*>(dA + a_lds[i] + half * (BM * 16)) = v;
  };

  // ---- accumulators -----------------------------------------------------------------------
  v16i acc[WM][WN];                                         // 2^shift * P_i of the cluster being accumulated
  v16f facc[PARTIALS ? 1 : WM][PARTIALS ? 1 : WN];          // sum over finished clusters of sX_i P_i
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

  // cluster tables live in one register each (lane i holds cluster i): a boundary reads them
  // with a lane read, no memory access inside the loop
  const float tab_scale = tab.scale[lane];
  const int tab_end = tab.slice_end[lane];
  const int tab_zx = PARTIALS ? tab.zx[lane] : 0, tab_n = PARTIALS ? tab.n[lane] : 0;
  int ci = 0;
  int next_end = __builtin_amdgcn_readlane(tab_end, 0);
  const int steps = (a.used_slices + kStepSlices - 1) / kStepSlices;

  // Pipeline.  Activations: LDS holds two stages; while stage p feeds the MFMAs of K step
  // `step`, the registers loaded earlier are unpacked into stage p^1 between those MFMAs.
  // Weights: one register set holds a step; a slice pair is refilled with the next step's bytes
  // right after its last use, seven slices before it is needed again.  Activation staging
  // registers are refilled after use with the data of step+3.
  // (step indices are clamped to the last step instead of guarding the loads: a load that is
  // always issued lets the compiler count outstanding loads exactly, and the surplus data of
  // the tail is never used)
  const int last = steps - 1;
  __builtin_amdgcn_s_setprio(2);
  load_a(0, 0);
  load_w(0);
  load_a(min(1, last), 1);
  // output-stage terms of this tile (thread i: channel n0 + i, token m0 + i; reads past the end
  // of a vector return 0 and belong to outputs that are never stored)
  float p_sw = 0.0f, p_ct = 0.0f, p_zw = 0.0f, p_rt = 0.0f;
  if (!PARTIALS) {
    const __amdgpu_buffer_rsrc_t sw_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.sW), 0, a.N * 4, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t ct_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.colterm), 0, a.N * 4, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t zw_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t*>(a.zW), 0, a.N * 4, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rt_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(a.rowterm) + m0, 0, static_cast<int>(rows_here) * 4, kRsrcFlags);
    const int ci = tid % BN, ri = tid % BM;
    p_sw = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(sw_rsrc, (n0 + ci) * 4, 0, 0));
    p_ct = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(ct_rsrc, (n0 + ci) * 4, 0, 0));
    p_zw = static_cast<float>(static_cast<int32_t>(__builtin_amdgcn_raw_buffer_load_b32(zw_rsrc, (n0 + ci) * 4, 0, 0)));
    p_rt = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rt_rsrc, ri * 4, 0, 0));
  }
#pragma unroll
  for (int u = 0; u < A_PER; ++u) {
    store_a_half(0, 0, u, 0);
    store_a_half(0, 0, u, 1);
  }
  // every prologue load has landed before the loop starts: the loop's own waits then count
  // only the loads of the steady state (vmcnt(0); the other counters are left alone)
  __builtin_amdgcn_s_waitcnt(0x0F70);
  if (!PARTIALS) {                                          // (threads beyond BN / BM repeat a valid entry)
    c_sw[tid % BN] = p_sw;
    c_ct[tid % BN] = p_ct;
    c_zw[tid % BN] = p_zw;
    c_rt[tid % BM] = p_rt;
  }
  if (CWISE && !PARTIALS) {                                 // scale table of this tile's columns (n_padded covers the tile)
    for (int k = tid; k < tab.g * BN; k += 256) c_sc[k] = a.scale_tab[static_cast<int64_t>(k / BN) * a.n_padded + n0 + (k % BN)] * a.cw_prescale;
  }
  __syncthreads();
  load_a(min(2, last), 0);

  v4i fb[2][WN];                                            // weight fragments (code << 4), one slice ahead
  auto unpack_w = [&](int q, int s, int j) {                // fb[q][j] <- slice s of the staged weights
    const uint4 w = wreg[j][s >> 1];
    const uint32_t x = (s & 1) ? w.z : w.x, y = (s & 1) ? w.w : w.y;
    fb[q][j][0] = static_cast<int>(x & 0xf0f0f0f0u);
    fb[q][j][1] = static_cast<int>((x << 4) & 0xf0f0f0f0u);
    fb[q][j][2] = static_cast<int>(y & 0xf0f0f0f0u);
    fb[q][j][3] = static_cast<int>((y << 4) & 0xf0f0f0f0u);
  };
#pragma unroll
  for (int j = 0; j < WN; ++j) unpack_w(0, 0, j);

  // Clears one tile's accumulators.  (Written as instructions the optimizer cannot see through:
  // a known zero would be folded into the next MFMA's C operand, which needs a second copy of
  // every slice body and measured 7 % slower; 8 two-register moves per tile.)
  auto clear_tile = [&](int i, int j) {
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
      unsigned long long zz;
      asm volatile("v_mov_b64 %0, 0" : "=v"(zz));
      acc[i][j][r] = static_cast<int>(zz);
      acc[i][j][r + 1] = static_cast<int>(zz >> 32);
    }
  };

  auto k_step = [&](int step, auto parity) {
    constexpr int buf = decltype(parity)::value;            // LDS stage / weight set read by this step
    const unsigned char* cA = sA + buf * A_STAGE;
    v4i fa[2][WM];                                          // activation fragments, one slice ahead
    auto load_frags = [&](int s, int q) {
#pragma unroll
      for (int i = 0; i < WM; ++i) fa[q][i] = *reinterpret_cast<const v4i*>(cA + s * A_SLICE + a_frag + i * 32 * 16);
    };
    load_frags(0, 0);
    const int w_step = min(step + 1, last), a_step = min(step + 3, last);
    auto do_slice = [&](auto s_tag) {
      constexpr int s = decltype(s_tag)::value;
      // One basic block per slice: the MFMAs of this slice with, between them, everything else
      // that is due - next slice's activation fragments (LDS reads), next slice's weight
      // fragments (register unpack) and a share of the next stage's activation unpack + LDS
      // write - so that the matrix pipe never waits for a burst of other instructions.
      {
        constexpr int NM = WM * WN;
        // the step's A units are spread evenly over its slices
        constexpr int u_lo = (s * A_PER + kStepSlices - 1) / kStepSlices;          // first unit of this slice
        constexpr int u_hi = ((s + 1) * A_PER + kStepSlices - 1) / kStepSlices;    // one past its last unit
        constexpr int NP = WN + 2 * (u_hi - u_lo);
        if (s + 1 < kStepSlices) load_frags(s + 1, (s + 1) & 1);
        auto piece = [&](int k) {
          if (k < WN) {
            // (on the last step the "next" data is stale and its results are never used)
            if (s + 1 < kStepSlices) unpack_w((s + 1) & 1, s + 1, k);
            else unpack_w(0, 0, k);              // pair 0 already holds the next step
          } else {
            const int h = k - WN;
            store_a_half(buf ^ 1, buf ^ 1, u_lo + (h >> 1), h & 1);
          }
        };
#pragma unroll
        for (int m = 0; m < NM; ++m) {
          const int i = m / WN, j = m % WN;
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[s & 1][j], fa[s & 1][i], acc[i][j], 0, 0, 0);
#pragma unroll
          for (int k = m; k < NP; k += NM) piece(k);
        }
        // refill the staging registers this slice has finished with
        if ((s & 1) == 0) {                                // pair s/2: its second slice was expanded just above
#pragma unroll
          for (int j = 0; j < WN; ++j) load_w_pair(w_step, j, s >> 1);
        }
#pragma unroll
        for (int u = u_lo; u < u_hi; ++u) load_a_unit(a_step, buf ^ 1, u);
        // pin the order: LDS reads first, then one MFMA followed by its share of the rest
        __builtin_amdgcn_sched_group_barrier(0x100, WM, 0);
#pragma unroll
        for (int m = 0; m < NM; ++m) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
          __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
        }
      }

      const int gs = step * kStepSlices + s + 1;           // slices accumulated so far
      if (gs == next_end) {                                  // cluster ci is complete (uniform branch)
        if (PARTIALS) {
          const int zx = __builtin_amdgcn_readlane(tab_zx, ci), nn = __builtin_amdgcn_readlane(tab_n, ci);
#pragma unroll
          for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int j = 0; j < WN; ++j) {
              const int64_t t = m0 + (wm * WM + i) * 32 + (lane & 31);
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                const int n = n0 + (wn * WN + j) * 32 + (r / 4) * 8 + (lane >> 5) * 4 + (r % 4);
                if (t < a.M && n < a.N) {
                  const int p = acc[i][j][r] >> (ActFmt<BITS>::kShift + 4);
                  const int zw = CWISE ? a.zW[static_cast<int64_t>(n) * tab.g + ci] : a.zW[n];
                  // (64-bit: the zero point of a weight block far from zero can reach 2^28; the stored
                  // value is the integer modulo 2^32)
                  const int64_t v = static_cast<int64_t>(p) - static_cast<int64_t>(zx) * a.wsum[static_cast<int64_t>(n) * tab.g + ci] -
                                    static_cast<int64_t>(zw) * a.xsum[t * tab.g + ci] + static_cast<int64_t>(nn) * zx * zw;
                  a.yq[(static_cast<int64_t>(ci) * a.M + t) * a.N + n] = static_cast<int32_t>(v);
                }
              }
              clear_tile(i, j);
            }
        } else {
          // (while this wave works through the instructions of the rescale it feeds the matrix
          // pipe nothing: the other wave of the SIMD gets the issue slots first)
          const float sc = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, tab_scale), ci));
          __builtin_amdgcn_s_setprio(0);
#pragma unroll
          for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int j = 0; j < WN; ++j) {
              if (CWISE) {                                   // every output column has its own scale for this cluster
                const float* scp = c_sc + ci * BN + (wn * WN + j) * 32 + (lane >> 5) * 4;
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                  const float4 s4 = *reinterpret_cast<const float4*>(scp + q4 * 8);
                  facc[i][j][q4 * 4 + 0] = fmaf(static_cast<float>(acc[i][j][q4 * 4 + 0]), s4.x, facc[i][j][q4 * 4 + 0]);
                  facc[i][j][q4 * 4 + 1] = fmaf(static_cast<float>(acc[i][j][q4 * 4 + 1]), s4.y, facc[i][j][q4 * 4 + 1]);
                  facc[i][j][q4 * 4 + 2] = fmaf(static_cast<float>(acc[i][j][q4 * 4 + 2]), s4.z, facc[i][j][q4 * 4 + 2]);
                  facc[i][j][q4 * 4 + 3] = fmaf(static_cast<float>(acc[i][j][q4 * 4 + 3]), s4.w, facc[i][j][q4 * 4 + 3]);
                }
              } else {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                  facc[i][j][r] = fmaf(static_cast<float>(acc[i][j][r]), sc, facc[i][j][r]);
              }
              clear_tile(i, j);
            }
          __builtin_amdgcn_s_setprio(2);
        }
        ++ci;
        next_end = __builtin_amdgcn_readlane(tab_end, ci & 63);
      }
    };
    do_slice(std::integral_constant<int, 0>());
    do_slice(std::integral_constant<int, 1>());
    do_slice(std::integral_constant<int, 2>());
    do_slice(std::integral_constant<int, 3>());
    do_slice(std::integral_constant<int, 4>());
    do_slice(std::integral_constant<int, 5>());
    do_slice(std::integral_constant<int, 6>());
    do_slice(std::integral_constant<int, 7>());
    static_assert(kStepSlices == 8, "eight slices per K step");
    __syncthreads();
  };
  // (pairs of steps in the loop, an odd last step after it: with no branch around a step inside
  // the loop, the count of loads in flight at the loop head is the same on every path)
  int step = 0;
  for (; step + 1 < steps; step += 2) {
    k_step(step, std::integral_constant<int, 0>());
    k_step(step + 1, std::integral_constant<int, 1>());
  }
  if (step < steps) k_step(step, std::integral_constant<int, 0>());
  __builtin_amdgcn_s_setprio(0);                             // the output stage yields to a co-resident main loop

  if (CWISE && !PARTIALS) {
    // Zero-point cross term, fp32 tile += (-sW zW)[n, i] * rtc[t, i] over the clusters i: per
    // 32 x 32 block g2/2 MFMAs of depth 2.  Lane l supplies row / column l & 31 and depth index
    // l >> 5; both tables are stored so that a lane's values for all its MFMAs are contiguous.
    const __amdgpu_buffer_rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(a.cross_tab), 0, a.n_padded * a.g2 * 4, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t r_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float*>(a.rtc) + m0 * a.g2, 0, static_cast<int>(rows_here) * a.g2 * 4, kRsrcFlags);
    const int half = a.g2 / 2;
    for (int k0 = 0; k0 < half; k0 += 4) {                   // four depth pairs per 16-byte load
      u4v av[WN], bv[WM];
#pragma unroll
      for (int j = 0; j < WN; ++j)
        av[j] = __builtin_amdgcn_raw_buffer_load_b128(
            x_rsrc, ((n0 + (wn * WN + j) * 32 + (lane & 31)) * a.g2 + (lane >> 5) * half + k0) * 4, 0, 0);
#pragma unroll
      for (int i = 0; i < WM; ++i)                           // (rows past M read 0: their outputs are never stored)
        bv[i] = __builtin_amdgcn_raw_buffer_load_b128(
            r_rsrc, (((wm * WM + i) * 32 + (lane & 31)) * a.g2 + (lane >> 5) * half + k0) * 4, 0, 0);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
          for (int j = 0; j < WN; ++j)
            facc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(av[j][kk]), __uint_as_float(bv[i][kk]),
                                                              facc[i][j], 0, 0, 0);
    }
  }

  // ---- zero-point terms, output scale, store ----------------------------------------------------
  // D[n][t]: a lane holds one token (lane & 31) and, per register quad, four consecutive output
  // channels.  The fp32 sums go through an LDS tile of the whole workgroup in row-major
  // [token][channel] order; afterwards every thread owns a fixed group of channels (its
  // per-channel constants are loaded once), finishes the arithmetic and writes 16 bytes per
  // row, so that rows of the output tile leave as full cache lines.
  if (!PARTIALS) {
    typedef float f2 __attribute__((ext_vector_type(2)));
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    constexpr int TP = BN + 4;                              // tile pitch in floats (16-byte pad: rows spread over banks)
    constexpr int CW = YF32 ? 4 : 8;                        // outputs per 16-byte store
    constexpr int CPR = BN / CW;                            // chunks per tile row
    constexpr int RPP = 256 / CPR;                          // tile rows per pass
    constexpr int NPASS = BM / RPP;
    static_assert(256 % CPR == 0 && BM % RPP == 0, "output tiling");
    float* tile = reinterpret_cast<float*>(smem);
    // per-channel and per-row terms of this thread's share, from the copies the prologue left in
    // LDS: the output stage issues no load, so it never waits behind the main loop's last ones
    const int cc = tid % CPR, rr = tid / CPR;
    const int n = n0 + cc * CW;
    float sw[CW], ct[CW], zw[CW], rt[NPASS];
#pragma unroll
    for (int e4 = 0; e4 < CW / 4; ++e4) {
      const float4 s4 = *reinterpret_cast<const float4*>(c_sw + cc * CW + e4 * 4);
      const float4 c4 = *reinterpret_cast<const float4*>(c_ct + cc * CW + e4 * 4);
      const float4 z4 = *reinterpret_cast<const float4*>(c_zw + cc * CW + e4 * 4);
      sw[e4 * 4 + 0] = s4.x; sw[e4 * 4 + 1] = s4.y; sw[e4 * 4 + 2] = s4.z; sw[e4 * 4 + 3] = s4.w;
      ct[e4 * 4 + 0] = c4.x; ct[e4 * 4 + 1] = c4.y; ct[e4 * 4 + 2] = c4.z; ct[e4 * 4 + 3] = c4.w;
      zw[e4 * 4 + 0] = z4.x; zw[e4 * 4 + 1] = z4.y; zw[e4 * 4 + 2] = z4.z; zw[e4 * 4 + 3] = z4.w;
    }
#pragma unroll
    for (int pass = 0; pass < NPASS; ++pass) rt[pass] = c_rt[pass * RPP + rr];
    // quantizing output stage: this thread's eight columns are one unit (8 codes) of the next
    // site's layout and lie in one cluster; its constants, and which of the eight are padding
    constexpr int QB = QOUT ? OUT : 8;                      // bits of the codes written
    constexpr int kQMin = -(1 << (QB - 1));
    constexpr float kUMax = static_cast<float>((1 << QB) - 1);
    float q_inv_s = 0.0f, q_zbf = 0.0f, q_floor = 0.0f;
    double q_s = 0.0;
    int32_t q_fix = 0;
    uint32_t q_keep[2] = {0xffffffffu, 0xffffffffu}, q_fill[2] = {0u, 0u};
    if (QOUT) {
      int ci = 0;
      for (int i = 1; i < qo.g; ++i) ci += (n >= qo.pad_off[i]) ? 1 : 0;
      q_inv_s = qo.inv_s[ci];
      q_zbf = static_cast<float>(qo.zb[ci]);
      q_s = static_cast<double>(qo.s[ci]);
      q_floor = qo.relu ? 0.0f : -__builtin_huge_valf();
      int n_real = qo.pad_off[ci] + qo.n[ci] - n;           // real channels among the eight
      n_real = n_real < 0 ? 0 : (n_real > 8 ? 8 : n_real);
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (e >= n_real) {                                  // pad position: code 0 (biased byte = -qmin)
          q_keep[e / 4] &= ~(0xffu << (8 * (e & 3)));
          q_fill[e / 4] |= static_cast<uint32_t>(-kQMin) << (8 * (e & 3));
        }
      q_fix = 8 * kQMin - n_real * qo.z[ci];                // sum of biased bytes -> sum of (q - z) over real codes
    }
    __syncthreads();                                        // every wave is done with the pipeline buffers
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
      for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int tl = (wm * WM + i) * 32 + (lane & 31);
          const int nl = (wn * WN + j) * 32 + q * 8 + (lane >> 5) * 4;
          *reinterpret_cast<float4*>(tile + tl * TP + nl) =
              make_float4(facc[i][j][q * 4 + 0], facc[i][j][q * 4 + 1], facc[i][j][q * 4 + 2], facc[i][j][q * 4 + 3]);
        }
    __syncthreads();
    double q_part[NPASS];                                   // quantizing stage: this thread's share of each row's de-quantized sum
    const bool vec_ok = (a.N % 8) == 0 && n + CW <= a.N;
    unsigned char* ybase = static_cast<unsigned char*>(a.y);
#pragma unroll
    for (int pass = 0; pass < NPASS; ++pass) {
      const int row = pass * RPP + rr;
      const int64_t t = m0 + row;
      float v[CW];
#pragma unroll
      for (int e4 = 0; e4 < CW / 4; ++e4) {
        const float4 f = *reinterpret_cast<const float4*>(tile + row * TP + cc * CW + e4 * 4);
        v[e4 * 4 + 0] = f.x; v[e4 * 4 + 1] = f.y; v[e4 * 4 + 2] = f.z; v[e4 * 4 + 3] = f.w;
      }
#pragma unroll
      for (int e = 0; e < CW; ++e) v[e] = CWISE ? (v[e] - ct[e]) : sw[e] * ((v[e] - ct[e]) - zw[e] * rt[pass]);
      if (QOUT) {
        // The value the next site quantizes is the bf16 the plain output stage would have
        // stored; from there on the arithmetic of the quantize-only kernel (Eq. 1): ReLU,
        // multiply by 1/s, round half to even, add the zero point, clamp.
        uint32_t D[2] = {0u, 0u};
#pragma unroll
        for (int e = 0; e < CW / 2; ++e) {
          const f2 pr = {v[2 * e], v[2 * e + 1]};
          const b2 cv = __builtin_convertvector(pr, b2);
          const uint32_t w2 = *reinterpret_cast<const uint32_t*>(&cv);
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const int c = 2 * e + h;
            float y = __uint_as_float(h ? (w2 & 0xffff0000u) : (w2 << 16));
            y = fmaxf(y, q_floor);
            const float r = __fmul_rn(y, q_inv_s);
            float b = __fadd_rn(rintf(r), q_zbf);
            if (QB < 8) b = fminf(b, kUMax);                // the conversion saturates at 0 and 255
            D[c / 4] = __builtin_amdgcn_cvt_pk_u8_f32(b, c & 3, D[c / 4]);
          }
        }
        D[0] = (D[0] & q_keep[0]) | q_fill[0];
        D[1] = (D[1] & q_keep[1]) | q_fill[1];
        const uint32_t usum = __builtin_amdgcn_sad_u8(D[1], 0u, __builtin_amdgcn_sad_u8(D[0], 0u, 0u));
        const bool live = t < a.M && n < a.N;
        double part = live ? q_s * static_cast<double>(static_cast<int32_t>(usum) + q_fix) : 0.0;
        if (QB == 3) {
          // 32 codes in 12 bytes (x0, x1, x2), the four threads of a lane quad hold codes 8k..8k+7:
          // k = 0, 1, 2 own bits 7..2 of x_k; the thread with k = 3 (codes 24..31) supplies the low
          // two bits of x0 and x1 (upper two bits of its codes) and bits 0, 1 of x2 (their low bits)
          const int k = cc & 3;
          const uint32_t main3 = ((D[0] << 5) | (D[1] << 2)) ^ 0x90909090u;
          const uint32_t p0 = ((D[0] >> 1) & 0x03030303u) ^ 0x02020202u;
          const uint32_t p1 = ((D[1] >> 1) & 0x03030303u) ^ 0x02020202u;
          const uint32_t p2 = (D[0] & 0x01010101u) | ((D[1] & 0x01010101u) << 1);
          const uint32_t b0 = static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(p0), 0xFF, 0xF, 0xF, true));
          const uint32_t b1 = static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(p1), 0xFF, 0xF, 0xF, true));
          const uint32_t b2 = static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(p2), 0xFF, 0xF, 0xF, true));
          const uint32_t word = main3 | (k == 0 ? b0 : (k == 1 ? b1 : b2));
          if (live && k < 3)
            *reinterpret_cast<uint32_t*>(qo.codes + t * qo.row_bytes + (n >> 5) * 12 + k * 4) = word;
        } else if (live) {
          if (QB == 8) {
            uint2 o;
            o.x = D[0] ^ 0x80808080u;
            o.y = D[1] ^ 0x80808080u;
            *reinterpret_cast<uint2*>(qo.codes + t * qo.row_bytes + n) = o;
          } else {
            *reinterpret_cast<uint32_t*>(qo.codes + t * qo.row_bytes + (n >> 1)) = ((D[0] << 4) | D[1]) ^ 0x88888888u;
          }
        }
        q_part[pass] = part;
      } else if (t < a.M) {
        if (YF32) {
          if (vec_ok) {
            *reinterpret_cast<float4*>(ybase + (t * a.N + n) * 4) = make_float4(v[0], v[1], v[2], v[3]);
          } else {
#pragma unroll
            for (int e = 0; e < CW; ++e)
              if (n + e < a.N) reinterpret_cast<float*>(ybase)[t * a.N + n + e] = v[e];
          }
        } else {
          uint32_t w[CW / 2];
#pragma unroll
          for (int e = 0; e < CW / 2; ++e) {
            const f2 pr = {v[2 * e], v[2 * e + 1]};
            const b2 cv = __builtin_convertvector(pr, b2);   // round to nearest even
            w[e] = *reinterpret_cast<const uint32_t*>(&cv);
          }
          if (vec_ok) {
            *reinterpret_cast<uint4*>(ybase + (t * a.N + n) * 2) = make_uint4(w[0], w[1 % (CW / 2)], w[2 % (CW / 2)], w[3 % (CW / 2)]);
          } else {
#pragma unroll
            for (int e = 0; e < CW; ++e)
              if (n + e < a.N) reinterpret_cast<uint16_t*>(ybase)[t * a.N + n + e] = static_cast<uint16_t>(w[e / 2] >> (16 * (e & 1)));
          }
        }
      }
    }
    if (QOUT) {
      // Row sums of this column tile: each row's NPASS-th share sits in the CPR lanes that hold
      // the row.  Halving exchange: at each of the first log2(NPASS) steps a lane hands half of
      // its values to its partner and keeps the sums of the other half, so that it ends with
      // one value; plain exchanges over the remaining lane bits finish the sum.  The total of
      // pass p lands in the lanes whose upper log2(NPASS) bits of cc spell p.
      static_assert((NPASS & (NPASS - 1)) == 0 && NPASS <= CPR, "row-sum exchange");
      int have = NPASS, m = CPR / 2;
#pragma unroll
      for (; have > 1; have >>= 1, m >>= 1) {
        const bool upper = (cc & m) != 0;
#pragma unroll
        for (int k = 0; k < NPASS / 2; ++k) {
          if (k < have / 2) {
            const double send = upper ? q_part[k] : q_part[k + have / 2];
            const double keep = upper ? q_part[k + have / 2] : q_part[k];
            q_part[k] = keep + __shfl_xor(send, m, kWave);
          }
        }
      }
      double total = q_part[0];
#pragma unroll
      for (; m >= 1; m >>= 1) total += __shfl_xor(total, m, kWave);
      constexpr int LPP = CPR / NPASS;                      // lanes per pass
      const int64_t t = m0 + (cc / LPP) * RPP + rr;
      if ((cc % LPP) == 0 && t < a.M) qo.rt_part[static_cast<int64_t>(tn) * a.M + t] = total;
    }
  }
}

// Sum over the column tiles, in tile order, of the row sums the quantizing output stage left.
__global__ void __launch_bounds__(64) rowterm_reduce_kernel(const double* part, int tiles_n, int64_t M, float* rowterm) {
  const int64_t t = static_cast<int64_t>(blockIdx.x) * 64 + threadIdx.x;
  if (t >= M) return;
  // sixteen independent loads in flight, added in tile order (a thread per row has little else to hide latency with)
  double acc = 0.0;
  int j = 0;
  for (; j + 16 <= tiles_n; j += 16) {
    double v[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = part[static_cast<int64_t>(j + k) * M + t];
#pragma unroll
    for (int k = 0; k < 16; ++k) acc += v[k];
  }
  for (; j < tiles_n; ++j) acc += part[static_cast<int64_t>(j) * M + t];
  rowterm[t] = static_cast<float>(acc);
}

// ---------------------------------------------------------------------------------------------
template <int BITS, int WGM, int WGN, int WM, int WN, bool PARTIALS, int OUT, bool CWISE>
static int32_t launch_cfg(const GemmArgs& a, const GemmTab& tab, const GemmQuantOut& qo, float* q_rowterm, hipStream_t st) {
  constexpr int BM = WGM * WM * 32, BN = WGN * WN * 32;
  constexpr size_t pipe = 2 * kStepSlices * (2 * BM * 16 + kSlicePad);
  constexpr size_t stage = PARTIALS ? 0 : static_cast<size_t>(BM) * (BN + 4) * 4;   // fp32 output tile of the workgroup
  constexpr size_t terms = PARTIALS ? 0 : static_cast<size_t>(3 * BN + BM) * 4;     // output-stage vectors of the tile
  // per-cluster column scales: in the gap between the pipeline buffers and the vectors when it holds them
  constexpr size_t front = pipe > stage ? pipe : stage;
  constexpr size_t cw_bytes = (CWISE && !PARTIALS) ? static_cast<size_t>(32) * BN * 4 : 0;
  constexpr size_t shmem = front + terms + ((front - pipe >= cw_bytes) ? 0 : cw_bytes);
  auto kern = cluster_gemm_kernel<BITS, WGM, WGN, WM, WN, PARTIALS, OUT, CWISE>;
  static LdsGrant lds_granted;
  if (int32_t st_lds = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), shmem, &lds_granted, st)) return st_lds;
  GemmArgs b = a;
  b.tiles_n = (a.N + BN - 1) / BN;
  b.tiles_m = static_cast<int32_t>((a.M + BM - 1) / BM);
  // tile order inside an XCD's range: blocks of 32 (16) row tiles x 4 column tiles (measured best of the
  // shapes from 4 x 16 to 128 x 2 on the 8192 x 49152 x 12288 product, 1 % over 16 x 4, 5 % over 4 x 16)
  b.grp_m = (b.tiles_m % 32 == 0) ? 32 : ((b.tiles_m % 16 == 0) ? 16 : 0);
  b.grp_n = 4;
  const dim3 grid(static_cast<unsigned>(b.tiles_n) * static_cast<unsigned>(b.tiles_m));
  hipLaunchKernelGGL(kern, grid, dim3(256), shmem, st, b, tab, qo);
  RPTQ_HIP(hipGetLastError());
  if (OUT >= 2) {
    hipLaunchKernelGGL(rowterm_reduce_kernel, dim3(static_cast<unsigned>((a.M + 63) / 64)), dim3(64), 0, st,
                       qo.rt_part, b.tiles_n, a.M, q_rowterm);
    RPTQ_HIP(hipGetLastError());
  }
  return RPTQ_OK;
}

template <int BITS, bool PARTIALS, int OUT, bool CWISE = false>
static int32_t launch_shape(const GemmArgs& a, const GemmTab& tab, const GemmQuantOut& qo, float* q_rowterm, hipStream_t st) {
  if (a.M <= 32) return launch_cfg<BITS, 1, 4, 1, 1, PARTIALS, OUT, CWISE>(a, tab, qo, q_rowterm, st);
  // 64 x 256 tile; every wave covers all 64 tokens and 64 output channels: each expanded
  // weight fragment feeds two MFMAs and no two waves expand the same weights
  return launch_cfg<BITS, 1, 4, 2, 2, PARTIALS, OUT, CWISE>(a, tab, qo, q_rowterm, st);
}

// out_mode: -1 partial sums, kOutBf16, kOutF32, or the next site's code bits (3, 4, 8)
template <int BITS>
static int32_t launch_bits(const GemmArgs& a, const GemmTab& tab, int out_mode, const GemmQuantOut& qo, float* q_rowterm,
                           hipStream_t st) {
  if (a.scale_tab != nullptr || a.g2 != 0) {               // one weight pair per (output, cluster)
    switch (out_mode) {
      case -1: return launch_shape<BITS, true, kOutF32, true>(a, tab, qo, q_rowterm, st);
      case kOutF32: return launch_shape<BITS, false, kOutF32, true>(a, tab, qo, q_rowterm, st);
      case kOutBf16: return launch_shape<BITS, false, kOutBf16, true>(a, tab, qo, q_rowterm, st);
    }
    return RPTQ_ERR_BITS;
  }
  switch (out_mode) {
    case -1: return launch_shape<BITS, true, kOutF32>(a, tab, qo, q_rowterm, st);
    case kOutF32: return launch_shape<BITS, false, kOutF32>(a, tab, qo, q_rowterm, st);
    case kOutBf16: return launch_shape<BITS, false, kOutBf16>(a, tab, qo, q_rowterm, st);
    case 3: return launch_shape<BITS, false, 3>(a, tab, qo, q_rowterm, st);
    case 4: return launch_shape<BITS, false, 4>(a, tab, qo, q_rowterm, st);
    case 8: return launch_shape<BITS, false, 8>(a, tab, qo, q_rowterm, st);
  }
  return RPTQ_ERR_BITS;
}

// ---- scratch for callers that cannot allocate ----------------------------------------------
// The quantizing output stage leaves per-column-tile row sums for its second kernel.  Callers
// that can neither allocate that workspace nor keep one around use this array instead: one
// copy per device, held until the process ends, shared by every call on that device.
static __device__ __align__(256) unsigned char scratch[RPTQ_STATIC_SCRATCH_BYTES];

// Device address of the current device's copy of the array (looked up once per device).  The
// array's name is only a host-side handle: kernels are given this address.
int32_t gemm_static_scratch(void** ptr) {
  static void* addr[kMaxDevices] = {};
  int dev = 0;
  if (int32_t s = current_device(&dev)) return s;
  if (dev < 0 || dev >= kMaxDevices) return RPTQ_ERR_SHAPE;
  std::lock_guard<std::mutex> lock(state_mutex());
  if (addr[dev] == nullptr) {
    void* p = nullptr;
    RPTQ_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return hip_fail(hipErrorInvalidSymbol);
    addr[dev] = p;
  }
  *ptr = addr[dev];
  return RPTQ_OK;
}

// Smallest column tile any launch shape uses: bounds the number of column tiles.
constexpr int kMinTileN = 128;

size_t gemm_quant_workspace_bytes(int64_t M, int32_t N) {
  return static_cast<size_t>((N + kMinTileN - 1) / kMinTileN) * static_cast<size_t>(M) * sizeof(double);
}

int32_t launch_gemm(const void* codes, int64_t M, int32_t bits, const void* Wq, int32_t N,
                    const ClusterGeom& geom, const float* sX, const float* sW, const int32_t* zW,
                    const float* colterm, const float* rowterm, void* y, int32_t y_dtype,
                    const int32_t* zX, const int32_t* xsum, const int32_t* wsum, int32_t* yq,
                    const GemmQuantOut* quant_out, float* q_rowterm, const GemmCw* cw, hipStream_t st) {
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
  const int shift = (bits == 8 ? 0 : (bits == 4 ? 4 : 5)) + 4;
  a.scale_tab = cw ? cw->scale_tab : nullptr;
  a.cross_tab = cw ? cw->cross_tab : nullptr;
  a.rtc = cw ? cw->rtc : nullptr;
  a.n_padded = (N + RPTQ_N_ALIGN - 1) / RPTQ_N_ALIGN * RPTQ_N_ALIGN;
  a.g2 = cw ? (geom.g <= 32 ? 32 : 64) : 0;
  a.cw_prescale = 1.0f / static_cast<float>(1 << shift);
  GemmTab tab;
  tab.g = geom.g;
  for (int i = 0; i < RPTQ_MAX_CLUSTERS; ++i) {
    const bool in = i < geom.g;
    tab.slice_end[i] = in ? geom.pad_off[i + 1] / kGroup : -1;
    const double s_here = (in && sX) ? static_cast<double>(sX[i]) : 0.0;
    tab.scale[i] = static_cast<float>(s_here / static_cast<double>(1 << shift));
    tab.zx[i] = (in && zX) ? zX[i] : 0;
    tab.n[i] = in ? geom.off[i + 1] - geom.off[i] : 0;
  }
  GemmQuantOut qo = {};
  int out_mode = (y_dtype == RPTQ_DTYPE_F32) ? kOutF32 : kOutBf16;
  if (yq != nullptr) out_mode = -1;
  if (quant_out != nullptr) {
    qo = *quant_out;
    out_mode = qo.row_bytes * 8 / N;                        // bits of the codes written
  }
  if (bits == 3) return launch_bits<3>(a, tab, out_mode, qo, q_rowterm, st);
  if (bits == 4) return launch_bits<4>(a, tab, out_mode, qo, q_rowterm, st);
  return launch_bits<8>(a, tab, out_mode, qo, q_rowterm, st);
}

}  // namespace rptq
