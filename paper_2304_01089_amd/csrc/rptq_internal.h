// Internal declarations shared by the translation units of librptq.
#pragma once
#include <stddef.h>
#include <stdint.h>
#include <hip/hip_runtime.h>

#include <mutex>

#include "rptq.h"

namespace rptq {

constexpr int kGroup = 32;                 // codes per packed group; cluster padding unit
constexpr int kWBlockCols = 128;           // columns of one packed weight block (32 rows x 128 columns = 2 KiB)
constexpr int32_t kZLimit = 1 << 21;       // largest |zero point| the fp32 clamp bounds carry exactly

// Cluster geometry passed to kernels by value (g <= RPTQ_MAX_CLUSTERS).
struct ClusterGeom {
  int32_t g;
  int32_t k;                               // unpadded channel count
  int32_t k_padded;                        // K_p
  int32_t off[RPTQ_MAX_CLUSTERS + 1];      // unpadded cluster offsets
  int32_t pad_off[RPTQ_MAX_CLUSTERS + 1];  // padded start of each cluster; pad_off[g] = end of last cluster
};

// Per-cluster quantizer constants for the LN+quant kernels.
struct QuantTab {
  float inv_s[RPTQ_MAX_CLUSTERS];
  float lo[RPTQ_MAX_CLUSTERS];             // float(qmin - z): clamp bounds applied before rounding
  float hi[RPTQ_MAX_CLUSTERS];             // float(qmax - z)
  int32_t zb[RPTQ_MAX_CLUSTERS];           // z - qmin: turns round(r) into the biased code
  float s[RPTQ_MAX_CLUSTERS];
  int32_t z[RPTQ_MAX_CLUSTERS];
};

struct GemmQuantOut;                       // gemm_common.h

// Tables of a linear layer whose weights carry one (s, z) per (output, cluster) (App. A.4 as printed).
struct GemmCw {
  const float* scale_tab;                  // [g, N_p]
  const float* cross_tab;                  // [N_p, g2]; NULL in verification mode
  const float* rtc;                        // [M, g2]; NULL in verification mode
};

// Key/value cache: what the kernels need to know about one position of the per-head cluster
// order (the cache layout is dense, so every position carries its cluster's constants).
struct KvPos {
  int32_t src;                             // original channel held at this position
  float inv_s;
  float s;
  int32_t z;
};

// Validation helpers (host.cpp).  All return an rptq_status.
int32_t check_clusters(const int32_t* cluster_off, int32_t g, ClusterGeom* geom);
int32_t check_bits(int32_t bits);
bool aligned16(const void* p);

// Records a failed HIP call for rptq_last_hip_error() and returns RPTQ_ERR_HIP.
int32_t hip_fail(hipError_t e);
#define RPTQ_HIP(expr)                                   \
  do {                                                   \
    hipError_t e_ = (expr);                              \
    if (e_ != hipSuccess) return ::rptq::hip_fail(e_);   \
  } while (0)

// ---- what the library remembers between calls (host.cpp) ---------------------------------
// One-time driver answers are kept per device (index of the current device at the call) in
// small tables guarded by one mutex; a device index beyond kMaxDevices is simply not cached.
constexpr int kMaxDevices = 64;
std::mutex& state_mutex();
// Index of the current device (hipGetDevice); RPTQ_ERR_HIP on failure.
int32_t current_device(int* dev);
// RPTQ_ERR_CAPTURE when `st` is recording a graph: a driver query may not run then.
int32_t require_not_capturing(hipStream_t st);
// Compute units of the current device (cached).
int32_t device_compute_units(hipStream_t st, int* cus);

// Raises a kernel's dynamic-LDS limit when a launch needs more than the default 64 KiB.  The
// driver call is made once per device and size (granted[] belongs to one kernel: a static
// array of kMaxDevices zeros in its launcher), so that repeated launches, and launches under
// stream capture, make no driver call at all.
struct LdsGrant {
  int bytes[kMaxDevices] = {};
};
int32_t ensure_dynamic_lds(const void* kern, size_t bytes, LdsGrant* granted, hipStream_t st);

// Workgroups of one launch shape resident per compute unit (occupancy query), cached per
// device for the last shape asked: a serving loop asks for the same shape again and again.
struct OccupancyMemo {
  int threads[kMaxDevices] = {};
  size_t shmem[kMaxDevices] = {};
  int per_cu[kMaxDevices] = {};
};
int32_t resident_workgroups(const void* kern, int threads, size_t shmem, OccupancyMemo* memo, hipStream_t st,
                            int* per_cu);

// Host clustering (host.cpp), exposed through rptq_cluster_channels.
int32_t cluster_channels(const float* ch_min, const float* ch_max, int32_t d, int32_t g, int32_t bits,
                         uint64_t seed, int32_t max_iter, int32_t* assign, int32_t* perm,
                         int32_t* cluster_off, float* s, float* inv_s, int32_t* z, int32_t* g_eff);

// Kernel launchers (one per .hip file).  Arguments are already validated.
int32_t launch_channel_minmax(const void* const* x_batches, const int64_t* rows, int32_t n_batches, int32_t d,
                              const float* gamma, const float* beta, float eps, int32_t relu,
                              float* ch_min_dev, float* ch_max_dev, uint32_t* keys, hipStream_t st);
// perm_pad_host: [k_padded] built by the caller; perm_out_host: [N] or NULL (uploaded through zW).
// Synchronizes `st` and returns RPTQ_ERR_RANGE when the weight kernel met a non-finite weight
// or a scale that is not a normal fp32 number.
int32_t launch_fold(const float* gamma, const float* beta, const int32_t* perm_pad_host, const ClusterGeom& geom,
                    const float* sX, const int32_t* zX, const void* W, int32_t w_dtype, int32_t N,
                    const int32_t* perm_out_host, int32_t* perm_pad, float* gamma_pad, float* beta_pad,
                    void* Wq_packed, float* sW, int32_t* zW, int32_t* wsum, float* colterm, hipStream_t st);
int32_t launch_ln_quant(const void* x, int64_t M, int32_t d, const float* gamma_pad, const float* beta_pad,
                        float eps, int32_t relu, const int32_t* perm_pad, const ClusterGeom& geom,
                        const QuantTab& qt, int32_t bits, void* codes, int32_t* xsum, float* rowterm,
                        hipStream_t st);
int32_t launch_gemm(const void* codes, int64_t M, int32_t bits, const void* Wq, int32_t N,
                    const ClusterGeom& geom, const float* sX, const float* sW, const int32_t* zW,
                    const float* colterm, const float* rowterm, void* y, int32_t y_dtype,
                    const int32_t* zX, const int32_t* xsum, const int32_t* wsum, int32_t* yq,
                    const GemmQuantOut* quant_out, float* q_rowterm, const GemmCw* cw, hipStream_t st);
int32_t launch_fold_cw(const int32_t* perm_pad_host, const ClusterGeom& geom, const float* sX, const int32_t* zX,
                       const void* W, int32_t w_dtype, int32_t N, const int32_t* perm_out_host, int32_t* perm_pad,
                       void* Wq_packed, float* sW, int32_t* zW, int32_t* wsum, float* scale_tab, float* cross_tab,
                       float* colterm, hipStream_t st);
int32_t launch_cluster_rowsums(const void* codes, int64_t M, const ClusterGeom& geom, int32_t bits, const float* sX,
                               const int32_t* zX, float* rtc, hipStream_t st);
size_t gemm_quant_workspace_bytes(int64_t M, int32_t N);
// Device address of the library's static scratch array on the current device (gemm.hip).
int32_t gemm_static_scratch(void** ptr);
size_t ln_scatter_workspace_bytes(int64_t M, int32_t d, int32_t k_padded);
int32_t launch_ln_scatter(const void* x, int64_t M, int32_t d, const float* gamma, const float* beta, float eps,
                          int32_t relu, const int32_t* perm_pad, const ClusterGeom& geom, const QuantTab& qt, int32_t bits,
                          void* codes, void* workspace, hipStream_t st);
int32_t launch_unpack_codes(const void* codes, int64_t rows, const ClusterGeom& geom, int32_t bits, int8_t* out,
                            hipStream_t st);
int32_t launch_unpack_weights(const void* Wq, int32_t N, const ClusterGeom& geom, int8_t* out, hipStream_t st);
// method1.hip: the first method of App. A.4 (de-quantize to bf16, floating-point product)
int32_t launch_dequant_codes(const void* codes, int64_t M, const ClusterGeom& geom, int32_t bits, const float* sX,
                             const int32_t* zX, void* out, hipStream_t st);
int32_t launch_dequant_weights(const void* Wq, int32_t N, const ClusterGeom& geom, const float* sW, const int32_t* zW,
                               void* out, hipStream_t st);
int32_t launch_gemm_bf16(const void* xh, const void* wh, int64_t M, int32_t N, int32_t K, void* y, int32_t y_f32,
                         hipStream_t st);
int32_t launch_kv_quant(const void* x, int64_t T, int32_t d, const KvPos* pos, int32_t bits, void* codes, hipStream_t st);
int32_t launch_kv_dequant(const void* codes, int64_t T, int32_t d, const KvPos* pos, int32_t bits, void* out, hipStream_t st);
// Per-head clustering (host.cpp), exposed through rptq_cluster_heads.
int32_t cluster_heads(const float* const* ch_min, const float* const* ch_max, int32_t n_tensors, int32_t d,
                      int32_t n_heads, int32_t g, int32_t bits, uint64_t seed, int32_t max_iter, int32_t* assign,
                      int32_t* perm, int32_t* cluster_off, float* s, float* inv_s, int32_t* z, int32_t* g_eff);

}  // namespace rptq
