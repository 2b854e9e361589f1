// Types shared by the cluster GEMM kernels (App. A.4, second method).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

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
  int32_t tiles_m, tiles_n;  // output tiles along M and N
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
  float scale[RPTQ_MAX_CLUSTERS];         // (sX_i - sX_{i+1}) / 2^shift
  int32_t zx[RPTQ_MAX_CLUSTERS];
  int32_t n[RPTQ_MAX_CLUSTERS];           // channels in cluster i
};

constexpr int kStepSlices = 8;            // slices per K step (256 codes): one barrier per step
constexpr int kSlicePad = 64;             // bytes added to a slice's LDS stride: 16 banks, so the four
                                          // slices a 16-lane write group touches fall in distinct banks

template <int BITS>
struct ActFmt {
  static constexpr int kGroupBytes = BITS * 4;             // bytes of 32 packed codes
  static constexpr int kShift = (BITS == 8) ? 0 : (BITS == 4 ? 4 : 5);
};

}  // namespace rptq
