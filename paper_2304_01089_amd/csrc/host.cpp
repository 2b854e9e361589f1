// Host-side pieces of librptq: argument checks, size queries, status strings, and the
// clustering step of calibration (K-Means over per-channel (min,max) points, reorder
// index, Min-Max parameters per cluster: Sec. 4.1 and Eq. 2 of the paper).
//
// Built with -ffp-contract=off: the K-Means rule is defined on separately rounded
// float64 operations in a fixed order so that its result is reproducible.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <vector>

#include "rptq_internal.h"

namespace rptq {

static std::atomic<int32_t> g_last_hip_error{0};

int32_t hip_fail(hipError_t e) {
  g_last_hip_error.store(static_cast<int32_t>(e));
  return RPTQ_ERR_HIP;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---- per-device memo of one-time driver answers ---------------------------------------------
std::mutex& state_mutex() {
  static std::mutex m;
  return m;
}

int32_t current_device(int* dev) {
  RPTQ_HIP(hipGetDevice(dev));
  return RPTQ_OK;
}

int32_t require_not_capturing(hipStream_t st) {
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  RPTQ_HIP(hipStreamIsCapturing(st, &cs));
  return cs == hipStreamCaptureStatusNone ? RPTQ_OK : RPTQ_ERR_CAPTURE;
}

int32_t device_compute_units(hipStream_t st, int* cus) {
  static int cached[kMaxDevices] = {};
  int dev = 0;
  if (int32_t s = current_device(&dev)) return s;
  const bool tracked = dev >= 0 && dev < kMaxDevices;
  std::lock_guard<std::mutex> lock(state_mutex());
  if (tracked && cached[dev] > 0) {
    *cus = cached[dev];
    return RPTQ_OK;
  }
  if (int32_t s = require_not_capturing(st)) return s;
  int n = 0;
  RPTQ_HIP(hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev));
  if (n < 1) n = 1;
  if (tracked) cached[dev] = n;
  *cus = n;
  return RPTQ_OK;
}

int32_t ensure_dynamic_lds(const void* kern, size_t bytes, LdsGrant* granted, hipStream_t st) {
  if (bytes <= 64 * 1024) return RPTQ_OK;
  int dev = 0;
  if (int32_t s = current_device(&dev)) return s;
  const bool tracked = dev >= 0 && dev < kMaxDevices;
  std::lock_guard<std::mutex> lock(state_mutex());
  if (tracked && granted->bytes[dev] >= static_cast<int>(bytes)) return RPTQ_OK;
  if (int32_t s = require_not_capturing(st)) return s;
  RPTQ_HIP(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes)));
  if (tracked) granted->bytes[dev] = static_cast<int>(bytes);
  return RPTQ_OK;
}

int32_t resident_workgroups(const void* kern, int threads, size_t shmem, OccupancyMemo* memo, hipStream_t st,
                            int* per_cu) {
  int dev = 0;
  if (int32_t s = current_device(&dev)) return s;
  const bool tracked = dev >= 0 && dev < kMaxDevices;
  std::lock_guard<std::mutex> lock(state_mutex());
  if (tracked && memo->per_cu[dev] > 0 && memo->threads[dev] == threads && memo->shmem[dev] == shmem) {
    *per_cu = memo->per_cu[dev];
    return RPTQ_OK;
  }
  if (int32_t s = require_not_capturing(st)) return s;
  int n = 0;
  RPTQ_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kern, threads, shmem));
  if (n < 1) n = 1;
  if (tracked) {
    memo->threads[dev] = threads;
    memo->shmem[dev] = shmem;
    memo->per_cu[dev] = n;
  }
  *per_cu = n;
  return RPTQ_OK;
}

int32_t check_bits(int32_t bits) { return (bits == 3 || bits == 4 || bits == 8) ? RPTQ_OK : RPTQ_ERR_BITS; }

int32_t check_clusters(const int32_t* cluster_off, int32_t g, ClusterGeom* geom) {
  if (!cluster_off) return RPTQ_ERR_NULL;
  if (g < 1 || g > RPTQ_MAX_CLUSTERS) return RPTQ_ERR_SHAPE;
  if (cluster_off[0] != 0) return RPTQ_ERR_PERM;
  int64_t padded = 0;
  for (int i = 0; i < g; ++i) {
    if (cluster_off[i + 1] <= cluster_off[i]) return RPTQ_ERR_PERM;
    if (cluster_off[i + 1] > RPTQ_MAX_CHANNELS) return RPTQ_ERR_SHAPE;
    if (geom) {
      geom->off[i] = cluster_off[i];
      geom->pad_off[i] = static_cast<int32_t>(padded);
    }
    int32_t n = cluster_off[i + 1] - cluster_off[i];
    padded += (n + kGroup - 1) / kGroup * kGroup;
  }
  const int64_t k_padded = (padded + RPTQ_K_ALIGN - 1) / RPTQ_K_ALIGN * RPTQ_K_ALIGN;
  // int32 headroom of the product kernels: |running sum| <= 2^14 * K_p must stay below 2^30
  static_assert(static_cast<int64_t>(RPTQ_MAX_K_PADDED) * (1 << 14) <= (int64_t{1} << 30), "accumulator headroom");
  if (k_padded > RPTQ_MAX_K_PADDED) return RPTQ_ERR_SHAPE;
  if (geom) {
    geom->g = g;
    geom->k = cluster_off[g];
    geom->off[g] = cluster_off[g];
    geom->pad_off[g] = static_cast<int32_t>(padded);
    geom->k_padded = static_cast<int32_t>(k_padded);
    for (int i = g + 1; i <= RPTQ_MAX_CLUSTERS; ++i) {
      geom->off[i] = geom->off[g];
      geom->pad_off[i] = geom->pad_off[g];
    }
  }
  return RPTQ_OK;
}

// ---------------------------------------------------------------------------
// Eq. 2 for one group sharing (s, z); float64, round half to even.
// ---------------------------------------------------------------------------
static int32_t minmax_params(float xmin, float xmax, int bits, float* s, float* inv_s, int32_t* z) {
  const double lo = xmin, hi = xmax;
  if (!(std::isfinite(lo) && std::isfinite(hi)) || hi < lo) return RPTQ_ERR_RANGE;
  double s64, zz;
  if (hi == lo) {
    s64 = 1.0;
    zz = -std::nearbyint(lo);
  } else {
    s64 = (hi - lo) / static_cast<double>(1 << bits);
    zz = -std::nearbyint((hi + lo) / (2.0 * s64));
  }
  if (!(std::fabs(zz) <= static_cast<double>(kZLimit))) return RPTQ_ERR_RANGE;
  const float s32 = static_cast<float>(s64);
  if (!(s32 > 0.0f) || !std::isfinite(s32) || !std::isnormal(s32)) return RPTQ_ERR_RANGE;
  *s = s32;
  *inv_s = static_cast<float>(1.0 / static_cast<double>(s32));
  *z = static_cast<int32_t>(zz);
  return RPTQ_OK;
}

// ---------------------------------------------------------------------------
// SplitMix64 (Steele, Lea, Flood 2014): the counter-based generator behind the seeding.
// ---------------------------------------------------------------------------
struct SplitMix64 {
  uint64_t state;
  explicit SplitMix64(uint64_t seed) : state(seed) {}
  uint64_t next() {
    state += 0x9E3779B97F4A7C15ull;
    uint64_t v = state;
    v = (v ^ (v >> 30)) * 0xBF58476D1CE4E5B9ull;
    v = (v ^ (v >> 27)) * 0x94D049BB133111EBull;
    return v ^ (v >> 31);
  }
  double uniform() { return static_cast<double>(next() >> 11) * (1.0 / 9007199254740992.0); }
};

static inline double sqdist(double px, double py, double cx, double cy) {
  const double dx = px - cx;
  const double dy = py - cy;
  const double a = dx * dx;
  const double b = dy * dy;
  return a + b;
}

static void assign_points(const std::vector<double>& px, const std::vector<double>& py,
                          const std::vector<double>& cx, const std::vector<double>& cy,
                          std::vector<int32_t>& out) {
  const size_t C = px.size(), gk = cx.size();
  for (size_t i = 0; i < C; ++i) {
    double best = sqdist(px[i], py[i], cx[0], cy[0]);
    int32_t bk = 0;
    for (size_t k = 1; k < gk; ++k) {
      const double dd = sqdist(px[i], py[i], cx[k], cy[k]);
      if (dd < best) {          // strict: ties stay with the lowest cluster id
        best = dd;
        bk = static_cast<int32_t>(k);
      }
    }
    out[i] = bk;
  }
}

int32_t cluster_channels(const float* ch_min, const float* ch_max, int32_t d, int32_t g, int32_t bits,
                         uint64_t seed, int32_t max_iter, int32_t* assign, int32_t* perm,
                         int32_t* cluster_off, float* s, float* inv_s, int32_t* z, int32_t* g_eff) {
  if (!ch_min || !ch_max || !assign || !perm || !cluster_off || !s || !inv_s || !z || !g_eff) return RPTQ_ERR_NULL;
  if (d < 1 || d > RPTQ_MAX_CHANNELS || g < 1 || g > d || g > RPTQ_MAX_CLUSTERS || max_iter < 1) return RPTQ_ERR_SHAPE;
  if (int32_t st = check_bits(bits)) return st;
  const size_t C = static_cast<size_t>(d);
  std::vector<double> px(C), py(C);
  for (size_t i = 0; i < C; ++i) {
    if (!std::isfinite(ch_min[i]) || !std::isfinite(ch_max[i]) || ch_max[i] < ch_min[i]) return RPTQ_ERR_RANGE;
    px[i] = ch_min[i];
    py[i] = ch_max[i];
  }

  // ---- D^2-weighted seeding ------------------------------------------------
  SplitMix64 rng(seed);
  std::vector<double> cx, cy, d2(C), cum(C);
  {
    size_t first = static_cast<size_t>(rng.uniform() * static_cast<double>(C));
    first = std::min(first, C - 1);
    cx.push_back(px[first]);
    cy.push_back(py[first]);
    for (size_t i = 0; i < C; ++i) d2[i] = sqdist(px[i], py[i], cx[0], cy[0]);
  }
  while (static_cast<int32_t>(cx.size()) < g) {
    double acc = 0.0;
    for (size_t i = 0; i < C; ++i) {
      acc = acc + d2[i];
      cum[i] = acc;
    }
    const double total = cum[C - 1];
    if (!(total > 0.0)) break;
    const double target = rng.uniform() * total;
    size_t nxt = std::upper_bound(cum.begin(), cum.end(), target) - cum.begin();   // first cum > target
    nxt = std::min(nxt, C - 1);
    cx.push_back(px[nxt]);
    cy.push_back(py[nxt]);
    for (size_t i = 0; i < C; ++i) d2[i] = std::min(d2[i], sqdist(px[i], py[i], cx.back(), cy.back()));
  }
  const size_t gk = cx.size();

  // ---- Lloyd iterations -----------------------------------------------------
  std::vector<int32_t> labels(C, -1), fresh(C);
  std::vector<int64_t> cnt(gk);
  std::vector<double> sx(gk), sy(gk), own(C);
  for (int it = 0; it < max_iter; ++it) {
    assign_points(px, py, cx, cy, fresh);
    if (fresh == labels) break;
    labels = fresh;
    std::fill(cnt.begin(), cnt.end(), 0);
    std::fill(sx.begin(), sx.end(), 0.0);
    std::fill(sy.begin(), sy.end(), 0.0);
    for (size_t i = 0; i < C; ++i) {          // ascending channel index
      const int32_t l = labels[i];
      cnt[l] += 1;
      sx[l] = sx[l] + px[i];
      sy[l] = sy[l] + py[i];
    }
    bool any_empty = false;
    for (size_t k = 0; k < gk; ++k) {
      if (cnt[k] > 0) {
        cx[k] = sx[k] / static_cast<double>(cnt[k]);
        cy[k] = sy[k] / static_cast<double>(cnt[k]);
      } else {
        any_empty = true;
      }
    }
    if (any_empty) {
      for (size_t i = 0; i < C; ++i) own[i] = sqdist(px[i], py[i], cx[labels[i]], cy[labels[i]]);
      for (size_t k = 0; k < gk; ++k) {
        if (cnt[k] > 0) continue;
        size_t far = 0;
        for (size_t i = 1; i < C; ++i)
          if (own[i] > own[far]) far = i;     // strict: lowest index on ties
        cx[k] = px[far];
        cy[k] = py[far];
        own[far] = -1.0;
      }
      std::fill(labels.begin(), labels.end(), -1);   // forces another pass
    }
  }
  if (std::find(labels.begin(), labels.end(), -1) != labels.end()) assign_points(px, py, cx, cy, labels);

  // ---- canonical labels (first occurrence), reorder index --------------------
  std::vector<int32_t> relabel(gk, -1);
  int32_t ge = 0;
  for (size_t i = 0; i < C; ++i) {
    int32_t& r = relabel[labels[i]];
    if (r < 0) r = ge++;
    assign[i] = r;
  }
  std::vector<int32_t> count(ge, 0);
  for (size_t i = 0; i < C; ++i) count[assign[i]] += 1;
  cluster_off[0] = 0;
  for (int32_t k = 0; k < ge; ++k) cluster_off[k + 1] = cluster_off[k] + count[k];
  std::vector<int32_t> cursor(cluster_off, cluster_off + ge);
  for (size_t i = 0; i < C; ++i) perm[cursor[assign[i]]++] = static_cast<int32_t>(i);   // ascending inside a cluster

  // ---- one Eq. 2 parameter pair per cluster -----------------------------------
  for (int32_t k = 0; k < ge; ++k) {
    float lo = ch_min[perm[cluster_off[k]]], hi = ch_max[perm[cluster_off[k]]];
    for (int32_t j = cluster_off[k]; j < cluster_off[k + 1]; ++j) {
      lo = std::min(lo, ch_min[perm[j]]);
      hi = std::max(hi, ch_max[perm[j]]);
    }
    if (int32_t st = minmax_params(lo + 0.0f, hi + 0.0f, bits, &s[k], &inv_s[k], &z[k])) return st;
  }
  *g_eff = ge;
  return RPTQ_OK;
}

// ---------------------------------------------------------------------------
// The same K-Means rule on points of any dimension (row-major pts[C][D]): used for the
// four-number points (Qmax, Qmin, Kmax, Kmin) that give queries and keys one shared reorder
// index (Sec. 4.2).  Squared distances add their terms in dimension order.
// ---------------------------------------------------------------------------
static inline double sqdist_nd(const double* p, const double* c, int D) {
  double acc = 0.0;
  for (int j = 0; j < D; ++j) {
    const double dj = p[j] - c[j];
    const double sq = dj * dj;
    acc = (j == 0) ? sq : acc + sq;
  }
  return acc;
}

static void kmeans_nd(const std::vector<double>& pts, size_t C, int D, int32_t g, uint64_t seed, int32_t max_iter,
                      std::vector<int32_t>& labels, size_t* g_used) {
  SplitMix64 rng(seed);
  std::vector<double> cen;                      // [gk][D]
  std::vector<double> d2(C), cum(C);
  {
    size_t first = static_cast<size_t>(rng.uniform() * static_cast<double>(C));
    first = std::min(first, C - 1);
    cen.insert(cen.end(), pts.begin() + first * D, pts.begin() + (first + 1) * D);
    for (size_t i = 0; i < C; ++i) d2[i] = sqdist_nd(&pts[i * D], &cen[0], D);
  }
  while (static_cast<int32_t>(cen.size() / D) < g) {
    double acc = 0.0;
    for (size_t i = 0; i < C; ++i) {
      acc = acc + d2[i];
      cum[i] = acc;
    }
    const double total = cum[C - 1];
    if (!(total > 0.0)) break;
    const double target = rng.uniform() * total;
    size_t nxt = std::upper_bound(cum.begin(), cum.end(), target) - cum.begin();
    nxt = std::min(nxt, C - 1);
    const size_t k = cen.size() / D;
    cen.insert(cen.end(), pts.begin() + nxt * D, pts.begin() + (nxt + 1) * D);
    for (size_t i = 0; i < C; ++i) d2[i] = std::min(d2[i], sqdist_nd(&pts[i * D], &cen[k * D], D));
  }
  const size_t gk = cen.size() / D;
  auto assign_all = [&](std::vector<int32_t>& out) {
    for (size_t i = 0; i < C; ++i) {
      double best = sqdist_nd(&pts[i * D], &cen[0], D);
      int32_t bk = 0;
      for (size_t k = 1; k < gk; ++k) {
        const double dd = sqdist_nd(&pts[i * D], &cen[k * D], D);
        if (dd < best) {
          best = dd;
          bk = static_cast<int32_t>(k);
        }
      }
      out[i] = bk;
    }
  };
  labels.assign(C, -1);
  std::vector<int32_t> fresh(C);
  std::vector<int64_t> cnt(gk);
  std::vector<double> sum(gk * D), own(C);
  for (int it = 0; it < max_iter; ++it) {
    assign_all(fresh);
    if (fresh == labels) break;
    labels = fresh;
    std::fill(cnt.begin(), cnt.end(), 0);
    std::fill(sum.begin(), sum.end(), 0.0);
    for (size_t i = 0; i < C; ++i) {            // ascending point index
      const int32_t l = labels[i];
      cnt[l] += 1;
      for (int j = 0; j < D; ++j) sum[l * D + j] = sum[l * D + j] + pts[i * D + j];
    }
    bool any_empty = false;
    for (size_t k = 0; k < gk; ++k) {
      if (cnt[k] > 0) {
        for (int j = 0; j < D; ++j) cen[k * D + j] = sum[k * D + j] / static_cast<double>(cnt[k]);
      } else {
        any_empty = true;
      }
    }
    if (any_empty) {
      for (size_t i = 0; i < C; ++i) own[i] = sqdist_nd(&pts[i * D], &cen[labels[i] * D], D);
      for (size_t k = 0; k < gk; ++k) {
        if (cnt[k] > 0) continue;
        size_t far = 0;
        for (size_t i = 1; i < C; ++i)
          if (own[i] > own[far]) far = i;
        for (int j = 0; j < D; ++j) cen[k * D + j] = pts[far * D + j];
        own[far] = -1.0;
      }
      std::fill(labels.begin(), labels.end(), -1);
    }
  }
  if (std::find(labels.begin(), labels.end(), -1) != labels.end()) assign_all(labels);
  *g_used = gk;
}

int32_t cluster_heads(const float* const* ch_min, const float* const* ch_max, int32_t n_tensors, int32_t d,
                      int32_t n_heads, int32_t g, int32_t bits, uint64_t seed, int32_t max_iter, int32_t* assign,
                      int32_t* perm, int32_t* cluster_off, float* s, float* inv_s, int32_t* z, int32_t* g_eff) {
  if (!ch_min || !ch_max || !assign || !perm || !cluster_off || !s || !inv_s || !z || !g_eff) return RPTQ_ERR_NULL;
  if (n_tensors != 1 && n_tensors != 2) return RPTQ_ERR_SHAPE;
  for (int t = 0; t < n_tensors; ++t)
    if (!ch_min[t] || !ch_max[t]) return RPTQ_ERR_NULL;
  if (d < 1 || d > RPTQ_MAX_CHANNELS || n_heads < 1 || d % n_heads != 0 || max_iter < 1) return RPTQ_ERR_SHAPE;
  const int32_t dh = d / n_heads;
  if (g < 1 || g > dh || g > RPTQ_MAX_CLUSTERS) return RPTQ_ERR_SHAPE;
  if (int32_t st = check_bits(bits)) return st;
  for (int t = 0; t < n_tensors; ++t)
    for (int32_t c = 0; c < d; ++c)
      if (!std::isfinite(ch_min[t][c]) || !std::isfinite(ch_max[t][c]) || ch_max[t][c] < ch_min[t][c]) return RPTQ_ERR_RANGE;
  const int D = 2 * n_tensors;
  std::vector<double> pts(static_cast<size_t>(dh) * D);
  std::vector<int32_t> labels;
  for (int32_t h = 0; h < n_heads; ++h) {
    const int32_t c0 = h * dh;
    for (int32_t c = 0; c < dh; ++c) {
      if (n_tensors == 1) {                    // (min, max), as for any single tensor (Sec. 4.1)
        pts[c * D + 0] = ch_min[0][c0 + c];
        pts[c * D + 1] = ch_max[0][c0 + c];
      } else {                                 // (Qmax, Qmin, Kmax, Kmin), as Sec. 4.2 lists them
        pts[c * D + 0] = ch_max[0][c0 + c];
        pts[c * D + 1] = ch_min[0][c0 + c];
        pts[c * D + 2] = ch_max[1][c0 + c];
        pts[c * D + 3] = ch_min[1][c0 + c];
      }
    }
    size_t gk = 0;
    kmeans_nd(pts, static_cast<size_t>(dh), D, g, seed + static_cast<uint64_t>(h), max_iter, labels, &gk);
    // canonical labels by first occurrence, members in ascending channel order
    std::vector<int32_t> relabel(gk, -1), count;
    int32_t ge = 0;
    for (int32_t c = 0; c < dh; ++c) {
      int32_t& r = relabel[labels[c]];
      if (r < 0) r = ge++;
      assign[c0 + c] = r;
    }
    count.assign(ge, 0);
    for (int32_t c = 0; c < dh; ++c) count[assign[c0 + c]] += 1;
    int32_t* off = cluster_off + static_cast<size_t>(h) * (g + 1);
    off[0] = 0;
    for (int32_t k = 0; k < ge; ++k) off[k + 1] = off[k] + count[k];
    for (int32_t k = ge; k < g; ++k) off[k + 1] = off[ge];
    std::vector<int32_t> cursor(off, off + ge);
    for (int32_t c = 0; c < dh; ++c) perm[c0 + cursor[assign[c0 + c]]++] = c0 + c;
    g_eff[h] = ge;
    for (int t = 0; t < n_tensors; ++t) {
      const size_t tb = (static_cast<size_t>(t) * n_heads + h) * g;
      for (int32_t k = 0; k < g; ++k) {
        s[tb + k] = 1.0f;
        inv_s[tb + k] = 1.0f;
        z[tb + k] = 0;
      }
      for (int32_t k = 0; k < ge; ++k) {
        float lo = ch_min[t][perm[c0 + off[k]]], hi = ch_max[t][perm[c0 + off[k]]];
        for (int32_t j = off[k]; j < off[k + 1]; ++j) {
          lo = std::min(lo, ch_min[t][perm[c0 + j]]);
          hi = std::max(hi, ch_max[t][perm[c0 + j]]);
        }
        if (int32_t st = minmax_params(lo + 0.0f, hi + 0.0f, bits, &s[tb + k], &inv_s[tb + k], &z[tb + k])) return st;
      }
    }
  }
  return RPTQ_OK;
}

}  // namespace rptq

using namespace rptq;

extern "C" {

int32_t rptq_padded_k(const int32_t* cluster_off, int32_t g, int32_t* k_padded) {
  if (!k_padded) return RPTQ_ERR_NULL;
  ClusterGeom geom;
  if (int32_t st = check_clusters(cluster_off, g, &geom)) return st;
  *k_padded = geom.k_padded;
  return RPTQ_OK;
}

size_t rptq_codes_bytes(int64_t M, int32_t k_padded, int32_t bits) {
  if (M < 0 || k_padded < 1 || k_padded % RPTQ_K_ALIGN != 0 || check_bits(bits) != RPTQ_OK) return 0;
  return static_cast<size_t>(M) * static_cast<size_t>(k_padded) * static_cast<size_t>(bits) / 8;
}

size_t rptq_weight_bytes(int32_t N, int32_t k_padded) {
  if (N < 1 || k_padded < 1 || k_padded % RPTQ_K_ALIGN != 0) return 0;
  const size_t n_p = (static_cast<size_t>(N) + RPTQ_N_ALIGN - 1) / RPTQ_N_ALIGN * RPTQ_N_ALIGN;
  return n_p * static_cast<size_t>(k_padded) / 2;
}

size_t rptq_calibrate_workspace_bytes(int32_t d) {
  if (d < 1 || d > RPTQ_MAX_CHANNELS) return 0;
  return static_cast<size_t>(d) * 4 * sizeof(uint32_t);   // keys (min,max) + fp32 results (min,max)
}

int32_t rptq_cluster_channels(const float* ch_min, const float* ch_max, int32_t d, int32_t g, int32_t bits,
                              uint64_t seed, int32_t max_iter, int32_t* assign, int32_t* perm,
                              int32_t* cluster_off, float* s, float* inv_s, int32_t* z, int32_t* g_eff) {
  return cluster_channels(ch_min, ch_max, d, g, bits, seed, max_iter, assign, perm, cluster_off, s, inv_s, z, g_eff);
}

int32_t rptq_cluster_heads(const float* const* ch_min, const float* const* ch_max, int32_t n_tensors, int32_t d,
                           int32_t n_heads, int32_t g, int32_t bits, uint64_t seed, int32_t max_iter,
                           int32_t* assign, int32_t* perm, int32_t* cluster_off, float* s, float* inv_s, int32_t* z,
                           int32_t* g_eff) {
  return cluster_heads(ch_min, ch_max, n_tensors, d, n_heads, g, bits, seed, max_iter, assign, perm, cluster_off, s,
                       inv_s, z, g_eff);
}

int32_t rptq_device_info(int32_t* compute_units, int32_t* clock_khz, int32_t* memory_clock_khz,
                         int32_t* memory_bus_bits) {
  int dev = 0;
  RPTQ_HIP(hipGetDevice(&dev));
  int v = 0;
  if (compute_units) {
    RPTQ_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev));
    *compute_units = v;
  }
  if (clock_khz) {
    RPTQ_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeClockRate, dev));
    *clock_khz = v;
  }
  if (memory_clock_khz) {
    RPTQ_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeMemoryClockRate, dev));
    *memory_clock_khz = v;
  }
  if (memory_bus_bits) {
    RPTQ_HIP(hipDeviceGetAttribute(&v, hipDeviceAttributeMemoryBusWidth, dev));
    *memory_bus_bits = v;
  }
  return RPTQ_OK;
}

const char* rptq_strerror(int32_t status) {
  switch (status) {
    case RPTQ_OK: return "ok";
    case RPTQ_ERR_NULL: return "a required pointer is NULL";
    case RPTQ_ERR_SHAPE: return "a size is out of range or inconsistent";
    case RPTQ_ERR_BITS: return "activation bits must be 3, 4 or 8";
    case RPTQ_ERR_ALIGN: return "device pointer not 16-byte aligned";
    case RPTQ_ERR_PERM: return "not a permutation, or cluster offsets not strictly increasing from 0";
    case RPTQ_ERR_RANGE: return "zero point or scale outside the exactly representable range";
    case RPTQ_ERR_WORKSPACE: return "workspace too small (or the call needs more than the static scratch array holds)";
    case RPTQ_ERR_HIP: return "a HIP call failed (see rptq_last_hip_error)";
    case RPTQ_ERR_CAPTURE: return "first launch of this shape on this device must happen outside stream capture";
    default: return "unknown status";
  }
}

int32_t rptq_last_hip_error(void) { return g_last_hip_error.load(); }

const char* rptq_version(void) { return "rptq-gfx950 0.1"; }

}  // extern "C"
