// extern "C" entry points of librptq: host-side validation, then the kernel launchers.
#include <cmath>
#include <cstring>
#include <vector>

#include "rptq_internal.h"
#include "gemm_common.h"

using namespace rptq;

namespace {

int32_t make_quant_tab(const ClusterGeom& geom, const float* s, const float* inv_s, const int32_t* z, int bits,
                       QuantTab* qt) {
  const int qmin = -(1 << (bits - 1)), qmax = (1 << (bits - 1)) - 1;
  for (int i = 0; i < RPTQ_MAX_CLUSTERS; ++i) {
    const bool in = i < geom.g;
    if (in) {
      if (!(std::isfinite(inv_s[i]) && inv_s[i] > 0.0f)) return RPTQ_ERR_RANGE;
      if (z[i] > kZLimit || z[i] < -kZLimit) return RPTQ_ERR_RANGE;
      if (s && !(std::isfinite(s[i]) && s[i] > 0.0f)) return RPTQ_ERR_RANGE;
    }
    qt->inv_s[i] = in ? inv_s[i] : 1.0f;
    qt->z[i] = in ? z[i] : 0;
    qt->lo[i] = static_cast<float>(qmin - qt->z[i]);
    qt->hi[i] = static_cast<float>(qmax - qt->z[i]);
    qt->zb[i] = qt->z[i] - qmin;
    qt->s[i] = (in && s) ? s[i] : 0.0f;
  }
  return RPTQ_OK;
}

int32_t check_permutation(const int32_t* perm, int32_t n) {
  std::vector<uint8_t> seen(static_cast<size_t>(n), 0);
  for (int32_t i = 0; i < n; ++i) {
    const int32_t p = perm[i];
    if (p < 0 || p >= n || seen[p]) return RPTQ_ERR_PERM;
    seen[p] = 1;
  }
  return RPTQ_OK;
}

}  // namespace

extern "C" {

int32_t rptq_channel_minmax(const void* const* x_batches, const int64_t* rows, int32_t n_batches, int32_t d,
                            const float* gamma, const float* beta, float eps, int32_t relu,
                            float* ch_min_dev, float* ch_max_dev, void* workspace, size_t workspace_bytes,
                            void* stream) {
  if (!x_batches || !rows || !ch_min_dev || !ch_max_dev || !workspace) return RPTQ_ERR_NULL;
  if ((gamma == nullptr) != (beta == nullptr)) return RPTQ_ERR_NULL;
  if (n_batches < 1 || d < 8 || d > RPTQ_MAX_CHANNELS || d % 8 != 0) return RPTQ_ERR_SHAPE;
  if (!(eps >= 0.0f) || !std::isfinite(eps)) return RPTQ_ERR_RANGE;
  int64_t total = 0;
  for (int b = 0; b < n_batches; ++b) {
    if (rows[b] < 0) return RPTQ_ERR_SHAPE;
    if (rows[b] > 0 && !x_batches[b]) return RPTQ_ERR_NULL;
    if (!aligned16(x_batches[b])) return RPTQ_ERR_ALIGN;
    total += rows[b];
  }
  if (total < 1) return RPTQ_ERR_SHAPE;
  if (workspace_bytes < static_cast<size_t>(d) * 2 * sizeof(uint32_t)) return RPTQ_ERR_WORKSPACE;
  if (!aligned16(workspace) || !aligned16(gamma) || !aligned16(beta)) return RPTQ_ERR_ALIGN;
  return launch_channel_minmax(x_batches, rows, n_batches, d, gamma, beta, eps, relu, ch_min_dev, ch_max_dev,
                               static_cast<uint32_t*>(workspace), static_cast<hipStream_t>(stream));
}

int32_t rptq_calibrate(const void* const* x_batches, const int64_t* rows, int32_t n_batches, int32_t d,
                       const float* gamma, const float* beta, float eps, int32_t relu,
                       int32_t g, int32_t bits, uint64_t seed, int32_t max_iter,
                       float* ch_min, float* ch_max, int32_t* assign, int32_t* perm,
                       int32_t* cluster_off, float* s, float* inv_s, int32_t* z, int32_t* g_eff,
                       void* workspace, size_t workspace_bytes, void* stream) {
  if (!ch_min || !ch_max || !assign || !perm || !cluster_off || !s || !inv_s || !z || !g_eff) return RPTQ_ERR_NULL;
  if (d < 1 || g < 1 || g > d || g > RPTQ_MAX_CLUSTERS || max_iter < 1) return RPTQ_ERR_SHAPE;
  if (int32_t st = check_bits(bits)) return st;
  if (workspace_bytes < rptq_calibrate_workspace_bytes(d) || rptq_calibrate_workspace_bytes(d) == 0)
    return workspace ? RPTQ_ERR_WORKSPACE : RPTQ_ERR_NULL;
  float* dev_min = reinterpret_cast<float*>(static_cast<uint32_t*>(workspace) + 2 * static_cast<size_t>(d));
  float* dev_max = dev_min + d;
  if (int32_t st = rptq_channel_minmax(x_batches, rows, n_batches, d, gamma, beta, eps, relu, dev_min, dev_max,
                                       workspace, workspace_bytes, stream))
    return st;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  RPTQ_HIP(hipMemcpyAsync(ch_min, dev_min, sizeof(float) * d, hipMemcpyDeviceToHost, hs));
  RPTQ_HIP(hipMemcpyAsync(ch_max, dev_max, sizeof(float) * d, hipMemcpyDeviceToHost, hs));
  RPTQ_HIP(hipStreamSynchronize(hs));
  return cluster_channels(ch_min, ch_max, d, g, bits, seed, max_iter, assign, perm, cluster_off, s, inv_s, z, g_eff);
}

int32_t rptq_fold_reorder(const float* gamma, const float* beta, int32_t d,
                          const int32_t* perm_in,
                          const int32_t* cluster_off, int32_t g, const float* sX, const int32_t* zX,
                          const void* W, int32_t w_dtype, int32_t w_rows, int32_t N, int32_t K,
                          const int32_t* perm_out,
                          int32_t* perm_pad, float* gamma_pad, float* beta_pad,
                          void* Wq_packed, float* sW, int32_t* zW, int32_t* wsum, float* colterm,
                          void* stream) {
  if (!perm_in || !perm_pad) return RPTQ_ERR_NULL;
  if ((gamma == nullptr) != (beta == nullptr)) return RPTQ_ERR_NULL;
  if (gamma && (!gamma_pad || !beta_pad)) return RPTQ_ERR_NULL;
  if (W && (!Wq_packed || !sW || !zW || !wsum || !colterm || !sX || !zX)) return RPTQ_ERR_NULL;
  ClusterGeom geom;
  if (int32_t st = check_clusters(cluster_off, g, &geom)) return st;
  if (d < 1 || geom.k != d) return RPTQ_ERR_SHAPE;
  if (W) {
    if (K != d || N < 1 || w_rows < 1) return RPTQ_ERR_SHAPE;
    if (!perm_out && N > w_rows) return RPTQ_ERR_SHAPE;
    if (w_dtype != RPTQ_DTYPE_BF16 && w_dtype != RPTQ_DTYPE_F32) return RPTQ_ERR_SHAPE;
    for (int i = 0; i < g; ++i) {
      if (!(std::isfinite(sX[i]) && sX[i] > 0.0f)) return RPTQ_ERR_RANGE;
      if (zX[i] > kZLimit || zX[i] < -kZLimit) return RPTQ_ERR_RANGE;
    }
    if (perm_out)                                    // every source row exists, or the entry is a pad row
      for (int32_t o = 0; o < N; ++o)
        if (perm_out[o] < -1 || perm_out[o] >= w_rows) return RPTQ_ERR_PERM;
  }
  if (int32_t st = check_permutation(perm_in, d)) return st;
  if (!aligned16(perm_pad) || !aligned16(gamma) || !aligned16(beta) || !aligned16(gamma_pad) ||
      !aligned16(beta_pad) || !aligned16(W) || !aligned16(Wq_packed) || !aligned16(sW) || !aligned16(zW) ||
      !aligned16(wsum) || !aligned16(colterm))
    return RPTQ_ERR_ALIGN;
  // source channel of every padded position (-1 = pad), from the validated index
  std::vector<int32_t> pad(static_cast<size_t>(geom.k_padded), -1);
  for (int i = 0; i < g; ++i)
    for (int32_t j = geom.off[i]; j < geom.off[i + 1]; ++j) pad[geom.pad_off[i] + (j - geom.off[i])] = perm_in[j];
  return launch_fold(gamma, beta, pad.data(), geom, sX, zX, W, w_dtype, N, perm_out, perm_pad, gamma_pad, beta_pad,
                     Wq_packed, sW, zW, wsum, colterm, static_cast<hipStream_t>(stream));
}

int32_t rptq_ln_quant(const void* x, int64_t M, int32_t d,
                      const float* gamma_pad, const float* beta_pad, float eps, int32_t relu,
                      const int32_t* perm_pad, const int32_t* cluster_off, int32_t g,
                      const float* s, const float* inv_s, const int32_t* z, int32_t bits,
                      void* codes_packed, int32_t* xsum, float* rowterm, void* stream) {
  if (!x || !perm_pad || !inv_s || !z || !codes_packed) return RPTQ_ERR_NULL;
  if ((gamma_pad == nullptr) != (beta_pad == nullptr)) return RPTQ_ERR_NULL;
  if (rowterm && !s) return RPTQ_ERR_NULL;
  if (int32_t st = check_bits(bits)) return st;
  ClusterGeom geom;
  if (int32_t st = check_clusters(cluster_off, g, &geom)) return st;
  if (M < 0 || d < 8 || d % 8 != 0 || geom.k != d) return RPTQ_ERR_SHAPE;
  if (!(eps >= 0.0f) || !std::isfinite(eps)) return RPTQ_ERR_RANGE;
  QuantTab qt;
  if (int32_t st = make_quant_tab(geom, s, inv_s, z, bits, &qt)) return st;
  if (!aligned16(x) || !aligned16(gamma_pad) || !aligned16(beta_pad) || !aligned16(perm_pad) ||
      !aligned16(codes_packed) || !aligned16(xsum) || !aligned16(rowterm))
    return RPTQ_ERR_ALIGN;
  return launch_ln_quant(x, M, d, gamma_pad, beta_pad, eps, relu, perm_pad, geom, qt, bits, codes_packed, xsum,
                         rowterm, static_cast<hipStream_t>(stream));
}

size_t rptq_ln_quant_scatter_workspace_bytes(int64_t M, int32_t d, int32_t k_padded) {
  if (M < 0 || d < 8 || d > RPTQ_MAX_CHANNELS || k_padded < 1 || k_padded % RPTQ_K_ALIGN != 0) return 0;
  return ln_scatter_workspace_bytes(M, d, k_padded);
}

int32_t rptq_ln_quant_scatter(const void* x, int64_t M, int32_t d, const float* gamma, const float* beta, float eps,
                              int32_t relu, const int32_t* perm_pad, const int32_t* cluster_off, int32_t g,
                              const float* inv_s, const int32_t* z, int32_t bits, void* codes_packed,
                              void* workspace, size_t workspace_bytes, void* stream) {
  if (!x || !perm_pad || !inv_s || !z || !codes_packed || !workspace) return RPTQ_ERR_NULL;
  if ((gamma == nullptr) != (beta == nullptr)) return RPTQ_ERR_NULL;
  if (int32_t st = check_bits(bits)) return st;
  ClusterGeom geom;
  if (int32_t st = check_clusters(cluster_off, g, &geom)) return st;
  if (M < 0 || d < 8 || d % 8 != 0 || geom.k != d) return RPTQ_ERR_SHAPE;
  if (!(eps >= 0.0f) || !std::isfinite(eps)) return RPTQ_ERR_RANGE;
  QuantTab qt;
  if (int32_t st = make_quant_tab(geom, nullptr, inv_s, z, bits, &qt)) return st;
  if (workspace_bytes < ln_scatter_workspace_bytes(M, d, geom.k_padded)) return RPTQ_ERR_WORKSPACE;
  if (!aligned16(x) || !aligned16(gamma) || !aligned16(beta) || !aligned16(perm_pad) || !aligned16(codes_packed) ||
      (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
    return RPTQ_ERR_ALIGN;
  return launch_ln_scatter(x, M, d, gamma, beta, eps, relu, perm_pad, geom, qt, bits, codes_packed, workspace,
                           static_cast<hipStream_t>(stream));
}

int32_t rptq_cluster_gemm(const void* codes_packed, int64_t M, int32_t bits,
                          const void* Wq_packed, int32_t N, const int32_t* cluster_off, int32_t g,
                          const float* sX, const float* sW, const int32_t* zW,
                          const float* colterm, const float* rowterm,
                          void* y, int32_t y_dtype, void* stream) {
  if (!codes_packed || !Wq_packed || !sX || !sW || !zW || !colterm || !rowterm || !y) return RPTQ_ERR_NULL;
  if (int32_t st = check_bits(bits)) return st;
  ClusterGeom geom;
  if (int32_t st = check_clusters(cluster_off, g, &geom)) return st;
  if (M < 0 || N < 1) return RPTQ_ERR_SHAPE;
  if (y_dtype != RPTQ_DTYPE_BF16 && y_dtype != RPTQ_DTYPE_F32) return RPTQ_ERR_SHAPE;
  for (int i = 0; i < g; ++i)
    if (!(std::isfinite(sX[i]) && sX[i] > 0.0f)) return RPTQ_ERR_RANGE;
  if (!aligned16(codes_packed) || !aligned16(Wq_packed) || !aligned16(sW) || !aligned16(zW) || !aligned16(colterm) ||
      !aligned16(rowterm) || !aligned16(y))
    return RPTQ_ERR_ALIGN;
  return launch_gemm(codes_packed, M, bits, Wq_packed, N, geom, sX, sW, zW, colterm, rowterm, y, y_dtype, nullptr,
                     nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, static_cast<hipStream_t>(stream));
}

size_t rptq_cluster_gemm_quant_workspace_bytes(int64_t M, int32_t N) {
  if (M < 0 || N < 1) return 0;
  return gemm_quant_workspace_bytes(M, N);
}

static int32_t gemm_quant_impl(const void* codes_packed, int64_t M, int32_t bits,
                                const void* Wq_packed, int32_t N, const int32_t* cluster_off, int32_t g,
                                const float* sX, const float* sW, const int32_t* zW,
                                const float* colterm, const float* rowterm, int32_t relu,
                                const int32_t* next_cluster_off, int32_t next_g, const float* next_s,
                                const float* next_inv_s, const int32_t* next_z, int32_t next_bits,
                                void* next_codes, float* next_rowterm,
                                void* workspace, size_t workspace_bytes, bool static_scratch, void* stream) {
  if (!codes_packed || !Wq_packed || !sX || !sW || !zW || !colterm || !rowterm) return RPTQ_ERR_NULL;
  if (!next_s || !next_inv_s || !next_z || !next_codes || !next_rowterm) return RPTQ_ERR_NULL;
  if (!static_scratch && !workspace) return RPTQ_ERR_NULL;
  if (int32_t st = check_bits(bits)) return st;
  if (int32_t st = check_bits(next_bits)) return st;
  ClusterGeom geom, next;
  if (int32_t st = check_clusters(cluster_off, g, &geom)) return st;
  if (int32_t st = check_clusters(next_cluster_off, next_g, &next)) return st;
  // the product's columns are the padded positions of the next site's layout
  if (M < 0 || N < 1 || N != next.k_padded) return RPTQ_ERR_SHAPE;
  for (int i = 0; i < g; ++i)
    if (!(std::isfinite(sX[i]) && sX[i] > 0.0f)) return RPTQ_ERR_RANGE;
  QuantTab qt;
  if (int32_t st = make_quant_tab(next, next_s, next_inv_s, next_z, next_bits, &qt)) return st;
  if (workspace_bytes < gemm_quant_workspace_bytes(M, N)) return RPTQ_ERR_WORKSPACE;
  if (static_scratch) {                            // validation is complete: now the device's own array
    if (int32_t st = gemm_static_scratch(&workspace)) return st;
  }
  if (!aligned16(codes_packed) || !aligned16(Wq_packed) || !aligned16(sW) || !aligned16(zW) || !aligned16(colterm) ||
      !aligned16(rowterm) || !aligned16(next_codes) || !aligned16(next_rowterm) || !aligned16(workspace))
    return RPTQ_ERR_ALIGN;
  GemmQuantOut qo = {};
  qo.codes = static_cast<uint8_t*>(next_codes);
  qo.rt_part = static_cast<double*>(workspace);
  qo.row_bytes = N * next_bits / 8;
  qo.relu = relu;
  qo.g = next.g;
  for (int i = 0; i <= RPTQ_MAX_CLUSTERS; ++i) qo.pad_off[i] = next.pad_off[i <= next.g ? i : next.g];
  for (int i = 0; i < RPTQ_MAX_CLUSTERS; ++i) {
    qo.n[i] = i < next.g ? next.off[i + 1] - next.off[i] : 0;
    qo.inv_s[i] = qt.inv_s[i];
    qo.s[i] = qt.s[i];
    qo.z[i] = qt.z[i];
    qo.zb[i] = qt.zb[i];
  }
  return launch_gemm(codes_packed, M, bits, Wq_packed, N, geom, sX, sW, zW, colterm, rowterm, nullptr,
                     RPTQ_DTYPE_BF16, nullptr, nullptr, nullptr, nullptr, &qo, next_rowterm, nullptr,
                     static_cast<hipStream_t>(stream));
}

int32_t rptq_cluster_gemm_quant(const void* codes_packed, int64_t M, int32_t bits,
                                const void* Wq_packed, int32_t N, const int32_t* cluster_off, int32_t g,
                                const float* sX, const float* sW, const int32_t* zW,
                                const float* colterm, const float* rowterm, int32_t relu,
                                const int32_t* next_cluster_off, int32_t next_g, const float* next_s,
                                const float* next_inv_s, const int32_t* next_z, int32_t next_bits,
                                void* next_codes, float* next_rowterm,
                                void* workspace, size_t workspace_bytes, void* stream) {
  return gemm_quant_impl(codes_packed, M, bits, Wq_packed, N, cluster_off, g, sX, sW, zW, colterm, rowterm, relu,
                         next_cluster_off, next_g, next_s, next_inv_s, next_z, next_bits, next_codes, next_rowterm,
                         workspace, workspace_bytes, false, stream);
}

int32_t rptq_cluster_gemm_quant_static(const void* codes_packed, int64_t M, int32_t bits,
                                       const void* Wq_packed, int32_t N, const int32_t* cluster_off, int32_t g,
                                       const float* sX, const float* sW, const int32_t* zW,
                                       const float* colterm, const float* rowterm, int32_t relu,
                                       const int32_t* next_cluster_off, int32_t next_g, const float* next_s,
                                       const float* next_inv_s, const int32_t* next_z, int32_t next_bits,
                                       void* next_codes, float* next_rowterm, void* stream) {
  return gemm_quant_impl(codes_packed, M, bits, Wq_packed, N, cluster_off, g, sX, sW, zW, colterm, rowterm, relu,
                         next_cluster_off, next_g, next_s, next_inv_s, next_z, next_bits, next_codes, next_rowterm,
                         nullptr, RPTQ_STATIC_SCRATCH_BYTES, true, stream);
}

size_t rptq_kv_table_bytes(int32_t d) {
  if (d < 1 || d > RPTQ_MAX_CHANNELS) return 0;
  return static_cast<size_t>(d) * sizeof(KvPos);
}

int32_t rptq_kv_tables(const int32_t* perm, const int32_t* cluster_off, const float* s, const float* inv_s,
                       const int32_t* z, int32_t d, int32_t n_heads, int32_t g, void* table, void* stream) {
  if (!perm || !cluster_off || !s || !inv_s || !z || !table) return RPTQ_ERR_NULL;
  if (d < kGroup || d > RPTQ_MAX_CHANNELS || d % kGroup != 0 || n_heads < 1 || d % n_heads != 0) return RPTQ_ERR_SHAPE;
  const int32_t dh = d / n_heads;
  if (1024 % dh != 0 || g < 1 || g > dh || g > RPTQ_MAX_CLUSTERS) return RPTQ_ERR_SHAPE;
  if (int32_t st = check_permutation(perm, d)) return st;
  std::vector<KvPos> tab(static_cast<size_t>(d));
  for (int32_t h = 0; h < n_heads; ++h) {
    const int32_t* off = cluster_off + static_cast<size_t>(h) * (g + 1);
    if (off[0] != 0 || off[g] != dh) return RPTQ_ERR_PERM;
    for (int32_t i = 0; i < g; ++i) {
      if (off[i + 1] < off[i]) return RPTQ_ERR_PERM;
      if (off[i + 1] == off[i]) continue;
      const size_t k = static_cast<size_t>(h) * g + i;
      if (!(std::isfinite(s[k]) && s[k] > 0.0f) || !(std::isfinite(inv_s[k]) && inv_s[k] > 0.0f)) return RPTQ_ERR_RANGE;
      if (z[k] > kZLimit || z[k] < -kZLimit) return RPTQ_ERR_RANGE;
      for (int32_t j = off[i]; j < off[i + 1]; ++j) {
        const int32_t c = perm[h * dh + j];
        if (c / dh != h) return RPTQ_ERR_PERM;               // a channel may not leave its head
        tab[h * dh + j] = KvPos{c, inv_s[k], s[k], z[k]};
      }
    }
  }
  if (!aligned16(table)) return RPTQ_ERR_ALIGN;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  RPTQ_HIP(hipMemcpyAsync(table, tab.data(), tab.size() * sizeof(KvPos), hipMemcpyHostToDevice, hs));
  RPTQ_HIP(hipStreamSynchronize(hs));
  return RPTQ_OK;
}

static int32_t check_kv(const void* a, const void* table, const void* b, int64_t T, int32_t d, int32_t bits) {
  if (!a || !table || !b) return RPTQ_ERR_NULL;
  if (int32_t st = check_bits(bits)) return st;
  if (T < 0 || d < kGroup || d > RPTQ_MAX_CHANNELS || d % kGroup != 0) return RPTQ_ERR_SHAPE;
  if (!aligned16(a) || !aligned16(table) || !aligned16(b)) return RPTQ_ERR_ALIGN;
  return RPTQ_OK;
}

int32_t rptq_kv_quant(const void* x, int64_t T, int32_t d, const void* table, int32_t bits, void* codes, void* stream) {
  if (int32_t st = check_kv(x, table, codes, T, d, bits)) return st;
  return launch_kv_quant(x, T, d, static_cast<const KvPos*>(table), bits, codes, static_cast<hipStream_t>(stream));
}

int32_t rptq_kv_dequant(const void* codes, int64_t T, int32_t d, const void* table, int32_t bits, void* out,
                        void* stream) {
  if (int32_t st = check_kv(codes, table, out, T, d, bits)) return st;
  return launch_kv_dequant(codes, T, d, static_cast<const KvPos*>(table), bits, out, static_cast<hipStream_t>(stream));
}

int32_t rptq_cluster_gemm_partials(const void* codes_packed, int64_t M, int32_t bits,
                                   const void* Wq_packed, int32_t N, const int32_t* cluster_off, int32_t g,
                                   const int32_t* zX, const int32_t* zW, const int32_t* xsum,
                                   const int32_t* wsum, int32_t* yq, void* stream) {
  if (!codes_packed || !Wq_packed || !zX || !zW || !xsum || !wsum || !yq) return RPTQ_ERR_NULL;
  if (int32_t st = check_bits(bits)) return st;
  ClusterGeom geom;
  if (int32_t st = check_clusters(cluster_off, g, &geom)) return st;
  if (M < 0 || N < 1) return RPTQ_ERR_SHAPE;
  for (int i = 0; i < g; ++i)
    if (zX[i] > kZLimit || zX[i] < -kZLimit) return RPTQ_ERR_RANGE;
  if (!aligned16(codes_packed) || !aligned16(Wq_packed) || !aligned16(zW) || !aligned16(xsum) || !aligned16(wsum) ||
      !aligned16(yq))
    return RPTQ_ERR_ALIGN;
  return launch_gemm(codes_packed, M, bits, Wq_packed, N, geom, nullptr, nullptr, zW, nullptr, nullptr, nullptr,
                     RPTQ_DTYPE_F32, zX, xsum, wsum, yq, nullptr, nullptr, nullptr, static_cast<hipStream_t>(stream));
}

// ---- weights with one parameter pair per (output channel, input cluster): App. A.4 as printed ----
constexpr int32_t kCwMaxClusters = 32;       // the per-column scale table of a tile lives in LDS

static size_t n_padded_of(int32_t N) { return (static_cast<size_t>(N) + RPTQ_N_ALIGN - 1) / RPTQ_N_ALIGN * RPTQ_N_ALIGN; }

size_t rptq_cw_scale_bytes(int32_t N, int32_t g) {
  if (N < 1 || g < 1 || g > kCwMaxClusters) return 0;
  return n_padded_of(N) * static_cast<size_t>(g) * sizeof(float);
}

size_t rptq_cw_cross_bytes(int32_t N, int32_t g) {
  if (N < 1 || g < 1 || g > kCwMaxClusters) return 0;
  return n_padded_of(N) * 32 * sizeof(float);
}

size_t rptq_cw_rowsum_bytes(int64_t M, int32_t g) {
  if (M < 0 || g < 1 || g > kCwMaxClusters) return 0;
  return static_cast<size_t>(M) * 32 * sizeof(float);
}

int32_t rptq_fold_reorder_cw(const int32_t* perm_in, const int32_t* cluster_off, int32_t g, const float* sX,
                             const int32_t* zX, const void* W, int32_t w_dtype, int32_t w_rows, int32_t N, int32_t K,
                             const int32_t* perm_out, int32_t* perm_pad, void* Wq_packed, float* sW, int32_t* zW,
                             int32_t* wsum, float* scale_tab, float* cross_tab, float* colterm, void* stream) {
  if (!perm_in || !perm_pad || !W || !Wq_packed || !sW || !zW || !wsum || !scale_tab || !cross_tab || !colterm || !sX || !zX)
    return RPTQ_ERR_NULL;
  ClusterGeom geom;
  if (int32_t st = check_clusters(cluster_off, g, &geom)) return st;
  if (g > kCwMaxClusters) return RPTQ_ERR_SHAPE;
  if (K < 1 || geom.k != K || N < 1 || w_rows < 1) return RPTQ_ERR_SHAPE;
  if (!perm_out && N > w_rows) return RPTQ_ERR_SHAPE;
  if (w_dtype != RPTQ_DTYPE_BF16 && w_dtype != RPTQ_DTYPE_F32) return RPTQ_ERR_SHAPE;
  for (int i = 0; i < g; ++i) {
    if (!(std::isfinite(sX[i]) && sX[i] > 0.0f)) return RPTQ_ERR_RANGE;
    if (zX[i] > kZLimit || zX[i] < -kZLimit) return RPTQ_ERR_RANGE;
  }
  if (perm_out)
    for (int32_t o = 0; o < N; ++o)
      if (perm_out[o] < -1 || perm_out[o] >= w_rows) return RPTQ_ERR_PERM;
  if (int32_t st = check_permutation(perm_in, K)) return st;
  if (!aligned16(perm_pad) || !aligned16(W) || !aligned16(Wq_packed) || !aligned16(sW) || !aligned16(zW) ||
      !aligned16(wsum) || !aligned16(scale_tab) || !aligned16(cross_tab) || !aligned16(colterm))
    return RPTQ_ERR_ALIGN;
  std::vector<int32_t> pad(static_cast<size_t>(geom.k_padded), -1);
  for (int i = 0; i < g; ++i)
    for (int32_t j = geom.off[i]; j < geom.off[i + 1]; ++j) pad[geom.pad_off[i] + (j - geom.off[i])] = perm_in[j];
  return launch_fold_cw(pad.data(), geom, sX, zX, W, w_dtype, N, perm_out, perm_pad, Wq_packed, sW, zW, wsum, scale_tab,
                        cross_tab, colterm, static_cast<hipStream_t>(stream));
}

int32_t rptq_cluster_rowsums(const void* codes_packed, int64_t M, int32_t bits, const int32_t* cluster_off, int32_t g,
                             const float* sX, const int32_t* zX, float* rowsums, void* stream) {
  if (!codes_packed || !sX || !zX || !rowsums) return RPTQ_ERR_NULL;
  if (int32_t st = check_bits(bits)) return st;
  ClusterGeom geom;
  if (int32_t st = check_clusters(cluster_off, g, &geom)) return st;
  if (M < 0 || g > kCwMaxClusters) return RPTQ_ERR_SHAPE;
  for (int i = 0; i < g; ++i) {
    if (!(std::isfinite(sX[i]) && sX[i] > 0.0f)) return RPTQ_ERR_RANGE;
    if (zX[i] > kZLimit || zX[i] < -kZLimit) return RPTQ_ERR_RANGE;
  }
  if (!aligned16(codes_packed) || !aligned16(rowsums)) return RPTQ_ERR_ALIGN;
  return launch_cluster_rowsums(codes_packed, M, geom, bits, sX, zX, rowsums, static_cast<hipStream_t>(stream));
}

int32_t rptq_cluster_gemm_cw(const void* codes_packed, int64_t M, int32_t bits, const void* Wq_packed, int32_t N,
                             const int32_t* cluster_off, int32_t g, const float* scale_tab, const float* cross_tab,
                             const float* colterm, const float* rowsums, void* y, int32_t y_dtype, void* stream) {
  if (!codes_packed || !Wq_packed || !scale_tab || !cross_tab || !colterm || !rowsums || !y) return RPTQ_ERR_NULL;
  if (int32_t st = check_bits(bits)) return st;
  ClusterGeom geom;
  if (int32_t st = check_clusters(cluster_off, g, &geom)) return st;
  if (M < 0 || N < 1 || g > kCwMaxClusters) return RPTQ_ERR_SHAPE;
  if (y_dtype != RPTQ_DTYPE_BF16 && y_dtype != RPTQ_DTYPE_F32) return RPTQ_ERR_SHAPE;
  if (!aligned16(codes_packed) || !aligned16(Wq_packed) || !aligned16(scale_tab) || !aligned16(cross_tab) ||
      !aligned16(colterm) || !aligned16(rowsums) || !aligned16(y))
    return RPTQ_ERR_ALIGN;
  const GemmCw cw = {scale_tab, cross_tab, rowsums};
  // (the per-row scale, zero point and row term of the per-row scheme are not used: their slots read the column term)
  return launch_gemm(codes_packed, M, bits, Wq_packed, N, geom, nullptr, colterm, reinterpret_cast<const int32_t*>(colterm),
                     colterm, rowsums, y, y_dtype, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, &cw,
                     static_cast<hipStream_t>(stream));
}

int32_t rptq_cluster_gemm_partials_cw(const void* codes_packed, int64_t M, int32_t bits, const void* Wq_packed,
                                      int32_t N, const int32_t* cluster_off, int32_t g, const int32_t* zX,
                                      const int32_t* zW, const int32_t* xsum, const int32_t* wsum, int32_t* yq,
                                      void* stream) {
  if (!codes_packed || !Wq_packed || !zX || !zW || !xsum || !wsum || !yq) return RPTQ_ERR_NULL;
  if (int32_t st = check_bits(bits)) return st;
  ClusterGeom geom;
  if (int32_t st = check_clusters(cluster_off, g, &geom)) return st;
  if (M < 0 || N < 1 || g > kCwMaxClusters) return RPTQ_ERR_SHAPE;
  for (int i = 0; i < g; ++i)
    if (zX[i] > kZLimit || zX[i] < -kZLimit) return RPTQ_ERR_RANGE;
  if (!aligned16(codes_packed) || !aligned16(Wq_packed) || !aligned16(zW) || !aligned16(xsum) || !aligned16(wsum) ||
      !aligned16(yq))
    return RPTQ_ERR_ALIGN;
  const GemmCw cw = {nullptr, nullptr, nullptr};
  return launch_gemm(codes_packed, M, bits, Wq_packed, N, geom, nullptr, nullptr, zW, nullptr, nullptr, nullptr,
                     RPTQ_DTYPE_F32, zX, xsum, wsum, yq, nullptr, nullptr, &cw, static_cast<hipStream_t>(stream));
}

int32_t rptq_unpack_codes(const void* codes_packed, int64_t rows, const int32_t* cluster_off, int32_t g,
                          int32_t bits, int8_t* out, void* stream) {
  if (!codes_packed || !out) return RPTQ_ERR_NULL;
  if (int32_t st = check_bits(bits)) return st;
  ClusterGeom geom;
  if (int32_t st = check_clusters(cluster_off, g, &geom)) return st;
  if (rows < 0) return RPTQ_ERR_SHAPE;
  return launch_unpack_codes(codes_packed, rows, geom, bits, out, static_cast<hipStream_t>(stream));
}

int32_t rptq_unpack_weights(const void* Wq_packed, int32_t N, const int32_t* cluster_off, int32_t g,
                            int8_t* out, void* stream) {
  if (!Wq_packed || !out) return RPTQ_ERR_NULL;
  ClusterGeom geom;
  if (int32_t st = check_clusters(cluster_off, g, &geom)) return st;
  if (N < 1) return RPTQ_ERR_SHAPE;
  return launch_unpack_weights(Wq_packed, N, geom, out, static_cast<hipStream_t>(stream));
}

// ---- first method of App. A.4 (comparison variant) ------------------------------------------------
int32_t rptq_dequant_codes(const void* codes_packed, int64_t M, int32_t bits, const int32_t* cluster_off, int32_t g,
                           const float* sX, const int32_t* zX, void* x_hat, void* stream) {
  if (!codes_packed || !sX || !zX || !x_hat) return RPTQ_ERR_NULL;
  if (int32_t st = check_bits(bits)) return st;
  ClusterGeom geom;
  if (int32_t st = check_clusters(cluster_off, g, &geom)) return st;
  if (M < 0) return RPTQ_ERR_SHAPE;
  for (int i = 0; i < g; ++i) {
    if (!(std::isfinite(sX[i]) && sX[i] > 0.0f)) return RPTQ_ERR_RANGE;
    if (zX[i] > kZLimit || zX[i] < -kZLimit) return RPTQ_ERR_RANGE;
  }
  if (!aligned16(codes_packed) || !aligned16(x_hat)) return RPTQ_ERR_ALIGN;
  return launch_dequant_codes(codes_packed, M, geom, bits, sX, zX, x_hat, static_cast<hipStream_t>(stream));
}

int32_t rptq_dequant_weights(const void* Wq_packed, int32_t N, const int32_t* cluster_off, int32_t g, const float* sW,
                             const int32_t* zW, void* w_hat, void* stream) {
  if (!Wq_packed || !sW || !zW || !w_hat) return RPTQ_ERR_NULL;
  ClusterGeom geom;
  if (int32_t st = check_clusters(cluster_off, g, &geom)) return st;
  if (N < 1) return RPTQ_ERR_SHAPE;
  if (!aligned16(Wq_packed) || !aligned16(sW) || !aligned16(zW) || !aligned16(w_hat)) return RPTQ_ERR_ALIGN;
  return launch_dequant_weights(Wq_packed, N, geom, sW, zW, w_hat, static_cast<hipStream_t>(stream));
}

int32_t rptq_gemm_bf16(const void* x_hat, const void* w_hat, int64_t M, int32_t N, int32_t K, void* y, int32_t y_dtype,
                       void* stream) {
  if (!x_hat || !w_hat || !y) return RPTQ_ERR_NULL;
  if (M < 0 || N < 4 || (N % 4) != 0 || K < 64 || (K % 64) != 0 || K > RPTQ_MAX_K_PADDED) return RPTQ_ERR_SHAPE;
  if (y_dtype != RPTQ_DTYPE_BF16 && y_dtype != RPTQ_DTYPE_F32) return RPTQ_ERR_SHAPE;
  if (!aligned16(x_hat) || !aligned16(w_hat) || !aligned16(y)) return RPTQ_ERR_ALIGN;
  return launch_gemm_bf16(x_hat, w_hat, M, N, K, y, y_dtype == RPTQ_DTYPE_F32, static_cast<hipStream_t>(stream));
}

}  // extern "C"
