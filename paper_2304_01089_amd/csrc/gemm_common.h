// Types shared by the cluster GEMM kernels (App. A.4, second method).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "rptq_internal.h"

namespace rptq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

struct GemmArgs {
  const uint8_t* codes;      // packed activation codes, row-major
  int64_t M;
  int32_t row_bytes;         // K_p * bits / 8
  const uint8_t* Wq;         // packed weights, fragment-major
  int32_t N;
  int32_t slices;            // K_p / 32
  int32_t used_slices;       // slices up to the end of the last cluster
  int32_t tiles_m, tiles_n;  // output tiles along M and N
  int32_t grp_m, grp_n;      // tile order: blocks of grp_m row tiles x grp_n column tiles
  const float* sW;
  const int32_t* zW;
  const float* colterm;
  const float* rowterm;
  void* y;
  // weights with one parameter pair per (output, cluster) (App. A.4 as printed)
  const float* scale_tab;    // [g, n_padded]: sX_i * sW[o,i]
  const float* cross_tab;    // [n_padded, g2]: -sW[o,i] * zW[o,i], MFMA operand order
  const float* rtc;          // [M, g2]: de-quantized row sum of every cluster, MFMA operand order
  int32_t n_padded;
  int32_t g2;
  float cw_prescale;         // 2^-shift: the operand bytes are code << shift
  // verification mode
  const int32_t* xsum;
  const int32_t* wsum;
  int32_t* yq;
};

struct GemmTab {
  int32_t g;
  int32_t slice_end[RPTQ_MAX_CLUSTERS];   // first slice after cluster i
  float scale[RPTQ_MAX_CLUSTERS];         // sX_i / 2^shift (the operand bytes are code << shift)
  int32_t zx[RPTQ_MAX_CLUSTERS];
  int32_t n[RPTQ_MAX_CLUSTERS];           // channels in cluster i
};

// Output stage that quantizes for the next site instead of storing Y (Sec. 4.2: the rows of
// this layer's weights were reordered offline, so column n of the product is padded position
// n of the next site's cluster-order layout).  Passed by value; unused by the other kernels.
struct GemmQuantOut {
  uint8_t* codes;                          // packed codes of the next site, [M, N * bits / 8]
  double* rt_part;                         // [tiles_n, M]: per column tile, the de-quantized row sum
  int32_t row_bytes;                       // N * bits / 8
  int32_t relu;
  int32_t g;
  int32_t pad_off[RPTQ_MAX_CLUSTERS + 1];  // padded start of the next site's clusters
  int32_t n[RPTQ_MAX_CLUSTERS];            // channels in each
  float inv_s[RPTQ_MAX_CLUSTERS];
  float s[RPTQ_MAX_CLUSTERS];
  int32_t z[RPTQ_MAX_CLUSTERS];
  int32_t zb[RPTQ_MAX_CLUSTERS];           // z - qmin
};

constexpr int kStepSlices = 8;            // slices per K step (256 codes): one barrier per step
constexpr int kSlicePad = 16;             // bytes added to a slice's LDS stride.  The staging stores of 8 consecutive
                                          // lanes go to the 8 slices of one row: with a stride of 2^n + 16 bytes they
                                          // fall into distinct 16-byte bank groups (a stride of 2^n + 64 put them into
                                          // two groups: 2-4 % slower on every shape)

template <int BITS>
struct ActFmt {
  static constexpr int kGroupBytes = BITS * 4;             // bytes of 32 packed codes
  static constexpr int kShift = (BITS == 8) ? 0 : (BITS == 4 ? 4 : 5);
};

}  // namespace rptq
