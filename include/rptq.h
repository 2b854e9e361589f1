/*
 * rptq.h - C ABI of the MI355X (gfx950) implementation of the RPTQ inference hot path
 * (reorder-based post-training quantization, arXiv 2304.01089).
 *
 * The path: a LayerNorm whose output leaves the kernel already in cluster order
 * (Sec. 4.2, "Avoid explicit reordering"), asymmetric round-to-nearest activation
 * quantization with one (scale, zero point) per channel cluster (Eq. 1, Eq. 2,
 * Sec. 4.1), and the integer-domain cluster-wise product of App. A.4 against 4-bit
 * per-output-channel weights whose input columns were permuted offline (Sec. 4.2).
 *
 * Conventions
 *  - Every function returns an rptq_status (0 = RPTQ_OK, negative = error).  Arguments
 *    are validated on the host before any HIP call; a failed validation launches nothing.
 *  - The caller owns all memory.  "device" pointers are HIP device memory, 16-byte
 *    aligned; "host" pointers are ordinary host memory.  What the library keeps between
 *    calls, per device and behind a lock (calls may come from several host threads and
 *    for several devices): the answers of its one-time driver queries (compute-unit
 *    count, workgroups resident per compute unit and raised dynamic-LDS limit of each
 *    launch shape) and a status word the offline kernels report bad input through.
 *    Nothing a result depends on.
 *  - The first launch of a shape on a device makes those driver queries and must
 *    therefore happen outside stream capture (RPTQ_ERR_CAPTURE otherwise); every later
 *    launch of the online entry points (rptq_ln_quant, rptq_cluster_gemm, rptq_cluster_gemm_quant) makes no
 *    driver call besides the kernel launches, allocates nothing and never synchronizes.
 *  - `stream` is a hipStream_t passed as void*.  Calls are asynchronous on that stream
 *    unless the description says the call synchronizes.
 *  - Cluster tables (cluster_off, scales, zero points) are small host arrays with
 *    1 <= g <= RPTQ_MAX_CLUSTERS; they travel to the kernels by value.
 *  - bf16 is the upper half of an IEEE fp32.
 *
 * Padded cluster-order layout ("K_p")
 *    Cluster i with n_i = cluster_off[i+1]-cluster_off[i] channels occupies
 *    pad32(n_i) consecutive positions; the total is rounded up to a multiple of
 *    RPTQ_K_ALIGN (256).  Pad positions hold activation code 0 and weight code 0 and
 *    never contribute.  rptq_padded_k() returns K_p.
 *
 * Packed activation codes: row-major, one row = K_p/32 groups of 32 codes.
 *    8 bit : 32 bytes, code j in byte j (two's complement).
 *    4 bit : 16 bytes = 4 dwords; byte b of dword u = (c[8u+b] << 4) | (c[8u+4+b] & 15).
 *    3 bit : 12 bytes = dwords x0,x1,x2 with f = c & 7:
 *            x0.byte b = f[b]<<5    | f[4+b]<<2  | f[24+b]>>1
 *            x1.byte b = f[8+b]<<5  | f[12+b]<<2 | f[28+b]>>1
 *            x2.byte b = f[16+b]<<5 | f[20+b]<<2 | (f[28+b]&1)<<1 | (f[24+b]&1)
 *    (each field sits where one shift and one mask turn it into a sign-carrying int8
 *    lane of an MFMA operand: 3-bit codes are stored packed and computed as 8-bit,
 *    as App. A.4 says such values must be cast to a supported width).
 *
 * Packed weights: N_p = N rounded up to 256 rows, in blocks of 32 rows x 128 columns of K_p;
 *    block (rb, kb) starts at byte ((rb * K_p/128) + kb) * 2048 and holds two halves of 1 KiB
 *    (K slices 0,1 and 2,3 of the block), each of 64 slots of 16 bytes; slot h*32 + r (h = 0,1)
 *    carries row rb*32+r; bytes 8e..8e+7 of the slot (e = 0,1) are columns
 *    kb*128 + (2*half + e)*32 + h*16 .. +15 as two 4-bit dwords in the 4-bit code format above.
 *    (One MFMA lane's operand bytes for two consecutive K slices are 16 contiguous bytes, a
 *    wave's are 1 KiB contiguous - eight whole cache lines per load: weights stream from HBM
 *    straight into operand registers.)
 */
#ifndef RPTQ_H
#define RPTQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RPTQ_MAX_CLUSTERS 64
#define RPTQ_K_ALIGN 256
#define RPTQ_N_ALIGN 256
#define RPTQ_MAX_CHANNELS 32768
/* Integer headroom of the product kernels: an int8 MFMA operand byte is code << 5, << 4 or
 * << 0 (|.| <= 128) for activations and code << 4 (|.| <= 128) for weights, and an int32
 * accumulator holds the sum over one cluster, which may be all of K_p, so
 * |sum| <= 2^14 * K_p.  K_p <= RPTQ_MAX_K_PADDED keeps that below 2^30; every entry point
 * refuses a cluster table whose K_p is larger (RPTQ_ERR_SHAPE). */
#define RPTQ_MAX_K_PADDED 65536

typedef enum {
  RPTQ_OK = 0,
  RPTQ_ERR_NULL = -1,      /* a required pointer is NULL */
  RPTQ_ERR_SHAPE = -2,     /* a size is out of range or inconsistent */
  RPTQ_ERR_BITS = -3,      /* activation bits not in {3,4,8} */
  RPTQ_ERR_ALIGN = -4,     /* a device pointer is not 16-byte aligned */
  RPTQ_ERR_PERM = -5,      /* perm is not a permutation / cluster_off not increasing */
  RPTQ_ERR_RANGE = -6,     /* a zero point or scale is outside what the kernels carry exactly */
  RPTQ_ERR_WORKSPACE = -7, /* workspace too small */
  RPTQ_ERR_HIP = -8,       /* a HIP call failed; see rptq_last_hip_error() */
  RPTQ_ERR_CAPTURE = -9    /* first launch of this shape on this device while the stream is capturing */
} rptq_status;

enum { RPTQ_DTYPE_BF16 = 0, RPTQ_DTYPE_F32 = 1 };

/* ---- sizes (host only, no HIP call) ------------------------------------------- */

/* K_p of the padded cluster-order layout.  cluster_off: host [g+1], strictly increasing from 0. */
int32_t rptq_padded_k(const int32_t* cluster_off, int32_t g, int32_t* k_padded);
/* Bytes of a packed activation-code buffer of M rows (0 on bad arguments). */
size_t rptq_codes_bytes(int64_t M, int32_t k_padded, int32_t bits);
/* Bytes of a packed weight buffer for N output channels (0 on bad arguments). */
size_t rptq_weight_bytes(int32_t N, int32_t k_padded);
/* Device workspace rptq_calibrate needs for d channels. */
size_t rptq_calibrate_workspace_bytes(int32_t d);

/* ---- calibration: Sec. 4.1 ------------------------------------------------------
 * Per-channel minimum and maximum of the site's activation over all calibration rows
 * (first displayed equation of Sec. 4.1), K-Means over the points (min_c, max_c) into g
 * clusters, the reorder index S = [S^1..S^g], and one Min-Max (Eq. 2) parameter pair per
 * cluster.  The activation is LayerNorm(x) when gamma/beta are given (biased variance,
 * statistics in fp64, elementwise chain in fp32), else x, with max(.,0) applied when
 * relu != 0.
 *
 * K-Means rule (the paper names the algorithm only): Euclidean distance on raw fp32
 * (min,max) points held as fp64; D^2-weighted seeding driven by SplitMix64(seed); Lloyd
 * iterations until the assignment repeats or max_iter; ties to the lowest cluster id;
 * an empty cluster is re-seeded with the point farthest from its own centre; clusters
 * are renumbered by first occurrence and members keep ascending channel order.
 *
 *  x_batches  host array [n_batches] of device bf16 [rows[b], d] row-major
 *  gamma,beta device fp32 [d], both NULL for a non-LayerNorm site
 *  ch_min/max host fp32 [d] out;  assign host int32 [d] out (cluster of each channel)
 *  perm       host int32 [d] out: reordered column j is original channel perm[j]
 *  cluster_off host int32 [g+1] out; s, inv_s host fp32 [g] out; z host int32 [g] out
 *  g_eff      host out: clusters actually produced (<= g when points coincide); entries
 *             beyond g_eff are not written
 *  workspace  device, rptq_calibrate_workspace_bytes(d)
 * Synchronizes the stream before returning.  RPTQ_ERR_RANGE if a zero point exceeds 2^21.
 */
int32_t rptq_calibrate(const void* const* x_batches, const int64_t* rows, int32_t n_batches, int32_t d,
                       const float* gamma, const float* beta, float eps, int32_t relu,
                       int32_t g, int32_t bits, uint64_t seed, int32_t max_iter,
                       float* ch_min, float* ch_max, int32_t* assign, int32_t* perm,
                       int32_t* cluster_off, float* s, float* inv_s, int32_t* z, int32_t* g_eff,
                       void* workspace, size_t workspace_bytes, void* stream);

/* ---- offline folding: Sec. 4.2 --------------------------------------------------
 * Folds the reorder index into LayerNorm's parameters and into the weights of the linear
 * layer that reads the site: gamma/beta are gathered into the padded cluster-order
 * layout, W's columns are permuted by perm_in (and its rows by perm_out, the reorder
 * index of the layer's *output*, when given), every output row is quantized to 4 bits
 * with its own Eq. 2 parameters over the whole row, and the codes are packed.  Also
 * emits what the integer form of App. A.4 needs per output channel: the per-cluster code
 * sums wsum[o,i] = sum_{c in cluster i} wq[o,c] and colterm[o] = sum_i sX_i zX_i wsum[o,i].
 *
 *  gamma,beta device fp32 [d] (NULL,NULL: skip the LayerNorm part)
 *  perm_in    host int32 [K] (K == d): the site's reorder index; must be a permutation of
 *             0..K-1 (RPTQ_ERR_PERM).  The library builds perm_pad from it on the host and
 *             uploads it; no device copy of the index is read.
 *  cluster_off,sX,zX  host [g+1],[g],[g]: the site's calibration result
 *  W          device [w_rows,K] row-major, w_dtype RPTQ_DTYPE_BF16 or RPTQ_DTYPE_F32; NULL: only
 *             the LayerNorm part / perm_pad
 *  w_rows     rows of W.  Without perm_out, N <= w_rows is required.
 *  perm_out   host int32 [N] or NULL; output row o' is original row perm_out[o'], which must lie
 *             in 0..w_rows-1, or be -1 (RPTQ_ERR_PERM otherwise); -1 makes o' a pad row (weights
 *             0, sW = 1, zW = 0, so Y[:,o'] = 0).  Passing the *next* site's perm_pad with N = its
 *             K_p lays the product's columns out as that site's padded cluster-order positions
 *             (what rptq_cluster_gemm_quant needs).
 *  perm_pad   device int32 [K_p] out: source channel of each padded position, -1 = pad
 *  gamma_pad,beta_pad device fp32 [K_p] out (untouched when gamma == NULL)
 *  Wq_packed  device out, rptq_weight_bytes(N, K_p)
 *  sW device fp32 [N], zW device int32 [N], wsum device int32 [N,g], colterm device fp32 [N]
 * Offline call: synchronizes the stream before returning (so that it can report what the
 * kernels found), cannot be captured.  RPTQ_ERR_RANGE when a weight is not finite or a row's
 * range gives a scale that is not a normal fp32 number; the outputs are then unspecified.
 */
int32_t rptq_fold_reorder(const float* gamma, const float* beta, int32_t d,
                          const int32_t* perm_in,
                          const int32_t* cluster_off, int32_t g, const float* sX, const int32_t* zX,
                          const void* W, int32_t w_dtype, int32_t w_rows, int32_t N, int32_t K,
                          const int32_t* perm_out,
                          int32_t* perm_pad, float* gamma_pad, float* beta_pad,
                          void* Wq_packed, float* sW, int32_t* zW, int32_t* wsum, float* colterm,
                          void* stream);

/* ---- online stage 1+2: LayerNorm in cluster order + per-cluster quantization -----
 * For every row t and padded position j with source channel c = perm_pad[j] in cluster i:
 *     y = ((x[t,c] - mu_t) * rstd_t) * gamma_pad[j] + beta_pad[j]      (Sec. 4.2)
 *     q = clamp(round(y * inv_s_i) + z_i, -2^(bits-1), 2^(bits-1)-1)  (Eq. 1; App. A.4)
 * mu_t, rstd_t over the whole row (biased variance) in fp64, rounded once to fp32; the
 * five elementwise operations are separately rounded fp32; round is half-to-even.
 * gamma_pad == NULL: no LayerNorm, y = x[t,c] (or max(x,0) when relu != 0), the
 * quantize-only form used after a linear layer whose rows were permuted offline.
 *
 *  x          device bf16 [M,d] row-major, original channel order
 *  perm_pad   device int32 [K_p] from rptq_fold_reorder
 *  cluster_off,s,inv_s,z  host [g+1],[g],[g],[g]
 *  codes_packed device out, rptq_codes_bytes(M, K_p, bits)
 *  xsum       device int32 [M,g] out or NULL: per-cluster code sums
 *  rowterm    device fp32 [M] out or NULL: sum_i s_i (xsum[t,i] - n_i z_i), the row sum of
 *             the de-quantized activation, which the product's zero-point term needs
 * Inputs must be finite: a NaN or infinity in x gives unspecified codes for its row (no
 * fault, no error).
 * Shapes the kernel does not cover return RPTQ_ERR_SHAPE before anything is launched: a
 * workgroup holds at most 960 unit threads of at most 2 (LayerNorm; 1 at 3 bits) or 4 (2)
 * units of 8 (16) codes, i.e. K_p <= 15360 with LayerNorm and K_p <= 30720 without, and two
 * bf16 copies of a row plus the partial sums must fit the 160 KiB of LDS.
 */
int32_t rptq_ln_quant(const void* x, int64_t M, int32_t d,
                      const float* gamma_pad, const float* beta_pad, float eps, int32_t relu,
                      const int32_t* perm_pad, const int32_t* cluster_off, int32_t g,
                      const float* s, const float* inv_s, const int32_t* z, int32_t bits,
                      void* codes_packed, int32_t* xsum, float* rowterm, void* stream);

/* ---- the same stage with the reorder as an offset of the write address ----------------
 * Sec. 4.2 ("Avoid explicit reordering") as the paper words it: LayerNorm runs in the
 * original channel order with gamma and beta untouched, and every result is written to the
 * address its reorder index gives it.  The smallest unit of a scattered write is a byte, so
 * the codes leave as one int8 each into an [M, K_p] buffer in the workspace and a second
 * kernel packs them.  Kept as the measured alternative to rptq_ln_quant (which gathers through
 * LDS and stores packed codes once); the packed codes are bit-identical.  No rowterm / xsum.
 *  gamma,beta device fp32 [d] in the ORIGINAL channel order (both NULL: no LayerNorm)
 *  workspace  device, 256-byte aligned, rptq_ln_quant_scatter_workspace_bytes(M, d, K_p)
 *  other arguments as rptq_ln_quant
 */
size_t rptq_ln_quant_scatter_workspace_bytes(int64_t M, int32_t d, int32_t k_padded);
int32_t rptq_ln_quant_scatter(const void* x, int64_t M, int32_t d, const float* gamma, const float* beta, float eps,
                              int32_t relu, const int32_t* perm_pad, const int32_t* cluster_off, int32_t g,
                              const float* inv_s, const int32_t* z, int32_t bits, void* codes_packed,
                              void* workspace, size_t workspace_bytes, void* stream);

/* ---- the first method of App. A.4 as a measured alternative ------------------------------
 * "De-quantize, concatenate, multiply in floating point": both operands are turned back into
 * x_hat = s (x_q - z) (the line under Eq. 1) - the integer difference exact in fp32, one fp32
 * product, one rounding to bf16 (ties to even) - in the padded cluster-order layout with zeros
 * at pad positions, and multiplied on the bf16 matrix cores with fp32 accumulation:
 *   Y[t,o] = sum_j x_hat[t,j] w_hat[o,j].
 * Kept beside rptq_cluster_gemm (the second method) to measure what the integer form saves.
 *  rptq_dequant_codes:    codes_packed device (M rows, bits in {3,4,8}); cluster_off,sX,zX host
 *                         [g+1],[g],[g]; x_hat device out bf16 [M, K_p]
 *  rptq_dequant_weights:  Wq_packed device (N, K_p) as written by rptq_fold_reorder; sW device
 *                         fp32 [N], zW device int32 [N]; w_hat device out bf16 [N, K_p]
 *  rptq_gemm_bf16:        x_hat, w_hat device bf16 [M,K], [N,K] row-major, K a multiple of 64
 *                         (K_p is), N a multiple of 4; y device out [M,N] row-major, y_dtype
 *                         RPTQ_DTYPE_BF16 or RPTQ_DTYPE_F32
 * All three are asynchronous on `stream`, allocate nothing, 16-byte aligned device pointers;
 * RPTQ_ERR_SHAPE / _RANGE / _ALIGN / _NULL as for the other entry points.
 */
int32_t rptq_dequant_codes(const void* codes_packed, int64_t M, int32_t bits, const int32_t* cluster_off, int32_t g,
                           const float* sX, const int32_t* zX, void* x_hat, void* stream);
int32_t rptq_dequant_weights(const void* Wq_packed, int32_t N, const int32_t* cluster_off, int32_t g, const float* sW,
                             const int32_t* zW, void* w_hat, void* stream);
int32_t rptq_gemm_bf16(const void* x_hat, const void* w_hat, int64_t M, int32_t N, int32_t K, void* y, int32_t y_dtype,
                       void* stream);

/* ---- online stage 3: cluster-wise integer product (App. A.4, second method) ------
 * Per cluster i the int32 product P_i[t,o] = sum_{c in i} xq[t,c] wq[o,c] runs on int8
 * MFMA; with the zero-point terms of App. A.4 the result is
 *   Y[t,o] = sW_o * ( sum_i sX_i P_i[t,o] - colterm[o] - zW_o * rowterm[t] )
 * which equals sum_i sX_i sW_o Yq_i with
 *   Yq_i = P_i - zX_i wsum[o,i] - zW_o xsum[t,i] + n_i zX_i zW_o.
 * Rows up to 32 take the weight-streaming kernel, larger M the LDS-tiled one.
 *
 *  codes_packed device, M rows, `bits` in {3,4,8};  Wq_packed device (N, K_p)
 *  cluster_off,sX host [g+1],[g];  sW,colterm device fp32 [N]; zW device int32 [N]
 *  rowterm    device fp32 [M]
 *  y          device out [M,N] row-major, y_dtype RPTQ_DTYPE_BF16 or RPTQ_DTYPE_F32
 */
int32_t rptq_cluster_gemm(const void* codes_packed, int64_t M, int32_t bits,
                          const void* Wq_packed, int32_t N, const int32_t* cluster_off, int32_t g,
                          const float* sX, const float* sW, const int32_t* zW,
                          const float* colterm, const float* rowterm,
                          void* y, int32_t y_dtype, void* stream);

/* ---- stage 3 with the next site's quantizer as its output stage (Sec. 4.2; Eq. 1) ------
 * For a linear layer whose output feeds another quantized site (fc1 -> ReLU -> fc2): the
 * layer's rows were reordered offline into the next site's padded cluster order (perm_out
 * of rptq_fold_reorder = that site's perm_pad, N = its K_p), so the product leaves the
 * matrix cores already in that order and is quantized in place of being stored:
 *     h = bf16(Y[t,n])  (the value rptq_cluster_gemm would have stored; round to nearest even)
 *     q = clamp(round(max(h,0) * inv_s_i) + z_i, ...)   i = next site's cluster of position n
 * exactly as rptq_ln_quant without LayerNorm does on a stored bf16 Y; pad positions get
 * code 0.  The bf16 tensor between the two layers is never written or read.
 *
 *  first twelve arguments: as rptq_cluster_gemm; N must equal the next site's K_p
 *  relu       != 0: max(h,0) before quantizing
 *  next_*     host: the next site's cluster_off [next_g+1], s, inv_s, z [next_g]; next_bits in {3,4,8}
 *  next_codes device out, rptq_codes_bytes(M, N, next_bits)
 *  next_rowterm device fp32 [M] out: as rptq_ln_quant's rowterm, for the next product
 *  workspace  device, rptq_cluster_gemm_quant_workspace_bytes(M, N) (RPTQ_ERR_WORKSPACE if
 *             smaller); holds per-column-tile row sums between the two kernels of this call
 */
size_t rptq_cluster_gemm_quant_workspace_bytes(int64_t M, int32_t N);
int32_t rptq_cluster_gemm_quant(const void* codes_packed, int64_t M, int32_t bits,
                                const void* Wq_packed, int32_t N, const int32_t* cluster_off, int32_t g,
                                const float* sX, const float* sW, const int32_t* zW,
                                const float* colterm, const float* rowterm, int32_t relu,
                                const int32_t* next_cluster_off, int32_t next_g, const float* next_s,
                                const float* next_inv_s, const int32_t* next_z, int32_t next_bits,
                                void* next_codes, float* next_rowterm,
                                void* workspace, size_t workspace_bytes, void* stream);

/* ---- the same call for callers that cannot allocate ------------------------------------
 * For code under HIP graph capture, tight serving loops and harnesses that forbid hipMalloc:
 * rptq_cluster_gemm_quant without the workspace argument.  The per-column-tile row sums go
 * to a scratch array of RPTQ_STATIC_SCRATCH_BYTES that lives in the library's device image
 * (one copy per device, held until the process ends); the call itself allocates nothing.
 * RPTQ_ERR_WORKSPACE when rptq_cluster_gemm_quant_workspace_bytes(M, N) exceeds that size
 * (nothing is launched).  Every call on a device uses that device's one array: calls that
 * overlap in time on one device (two streams, two threads) race on it and must be serialized
 * by the caller; nothing has to be cleared between calls, every entry that is read was
 * written by the same call.  As with every launch shape, the first call on a device looks
 * things up in the driver (here also the array's address) and belongs outside stream capture.
 * Arguments, results and errors otherwise exactly as rptq_cluster_gemm_quant. */
#define RPTQ_STATIC_SCRATCH_BYTES (8u << 20)
int32_t rptq_cluster_gemm_quant_static(const void* codes_packed, int64_t M, int32_t bits,
                                       const void* Wq_packed, int32_t N, const int32_t* cluster_off, int32_t g,
                                       const float* sX, const float* sW, const int32_t* zW,
                                       const float* colterm, const float* rowterm, int32_t relu,
                                       const int32_t* next_cluster_off, int32_t next_g, const float* next_s,
                                       const float* next_inv_s, const int32_t* next_z, int32_t next_bits,
                                       void* next_codes, float* next_rowterm, void* stream);

/* ---- weights with one parameter pair per (output channel, input cluster) ---------------
 * App. A.4 as printed: the reordered weight matrix is divided along its input channels into
 * the activation's clusters and every block W~_{o,i} has its own Eq. 2 pair
 * (s^W_{o,i}, z^W_{o,i}); the second method then gives
 *   Y[t,o] = sum_i sX_i sW[o,i] ( P_i[t,o] - zX_i wsum[o,i] - zW[o,i] xsum[t,i] + n_i zX_i zW[o,i] ).
 * The kernels evaluate it as
 *   Y = sum_i (sX_i sW[o,i]) P_i  -  colterm[o]  -  sum_i (sW[o,i] zW[o,i]) * rowsums[t,i]
 * with colterm[o] = sum_i sX_i sW[o,i] zX_i wsum[o,i] and rowsums[t,i] = sX_i (xsum[t,i] - n_i zX_i),
 * the last sum being a rank-g update of the fp32 tile on the matrix cores.  At most 32 clusters.
 *
 * rptq_fold_reorder_cw: rptq_fold_reorder's weight part with the per-block parameters.
 *   perm_in, cluster_off, sX, zX, W, w_dtype, w_rows, N, K, perm_out, perm_pad, Wq_packed: as there
 *   sW device fp32 [N,g], zW device int32 [N,g], wsum device int32 [N,g] out
 *   scale_tab device fp32 out, rptq_cw_scale_bytes(N, g): [g, N_p], sX_i sW[o,i] (N_p = N rounded up to 256)
 *   cross_tab device fp32 out, rptq_cw_cross_bytes(N, g): [N_p, 32], -sW[o,i] zW[o,i] at column
 *             (i & 1) * 16 + i / 2 (the operand order of the fp32 MFMA of depth 2)
 *   colterm   device fp32 [N] out
 * rptq_cluster_rowsums: rowsums of a batch of packed activation codes (an online step, between
 *   rptq_ln_quant and the product):  rowsums device fp32 out, rptq_cw_rowsum_bytes(M, g): [M, 32],
 *   same column order as cross_tab.  cluster_off, sX, zX host.
 * rptq_cluster_gemm_cw: the product.  rptq_cluster_gemm_partials_cw: the literal integers
 *   Yq_i [g,M,N] with zW device int32 [N,g] (a weight block that lies far from zero relative to
 *   its width has a zero point of up to 2^28, which is carried exactly everywhere; the int32
 *   Yq_i are then stored modulo 2^32).
 */
size_t rptq_cw_scale_bytes(int32_t N, int32_t g);
size_t rptq_cw_cross_bytes(int32_t N, int32_t g);
size_t rptq_cw_rowsum_bytes(int64_t M, int32_t g);
int32_t rptq_fold_reorder_cw(const int32_t* perm_in, const int32_t* cluster_off, int32_t g, const float* sX,
                             const int32_t* zX, const void* W, int32_t w_dtype, int32_t w_rows, int32_t N, int32_t K,
                             const int32_t* perm_out, int32_t* perm_pad, void* Wq_packed, float* sW, int32_t* zW,
                             int32_t* wsum, float* scale_tab, float* cross_tab, float* colterm, void* stream);
int32_t rptq_cluster_rowsums(const void* codes_packed, int64_t M, int32_t bits, const int32_t* cluster_off, int32_t g,
                             const float* sX, const int32_t* zX, float* rowsums, void* stream);
int32_t rptq_cluster_gemm_cw(const void* codes_packed, int64_t M, int32_t bits, const void* Wq_packed, int32_t N,
                             const int32_t* cluster_off, int32_t g, const float* scale_tab, const float* cross_tab,
                             const float* colterm, const float* rowsums, void* y, int32_t y_dtype, void* stream);
int32_t rptq_cluster_gemm_partials_cw(const void* codes_packed, int64_t M, int32_t bits, const void* Wq_packed,
                                      int32_t N, const int32_t* cluster_off, int32_t g, const int32_t* zX,
                                      const int32_t* zW, const int32_t* xsum, const int32_t* wsum, int32_t* yq,
                                      void* stream);

/* ---- attention sites: shared query/key index, key/value cache codes ---------------------
 * Sec. 4.2 (last paragraph): queries and keys are multiplied over their channels, so they
 * must share one reorder index; it comes from K-Means over the points
 * (Qmax_c, Qmin_c, Kmax_c, Kmin_c).  Sec. 5.1: one index per attention head; the settings
 * W4A4KV, W4A3KV and W3A3KV quantize only the key and value caches.
 *
 * rptq_cluster_heads (host only): one clustering per head over the head's d / n_heads
 * channels, with the K-Means rule of rptq_calibrate on points of two numbers (min, max) for
 * one tensor, or of four numbers in the order above for two tensors (queries first); head h
 * is seeded with seed + h.  Channels never leave their head.
 *   ch_min,ch_max  host arrays of n_tensors (1 or 2) pointers to host fp32 [d]
 *   assign host int32 [d] out: cluster of each channel inside its head
 *   perm   host int32 [d] out: reordered position j holds original channel perm[j]
 *   cluster_off host int32 [n_heads, g+1] out: offsets inside the head; clusters that did not
 *          form (coinciding points) repeat the last offset;  g_eff host int32 [n_heads] out
 *   s, inv_s host fp32 [n_tensors, n_heads, g], z host int32 [n_tensors, n_heads, g] out: every
 *          tensor's own Eq. 2 pair per cluster (1, 1, 0 where the cluster did not form)
 *
 * rptq_kv_tables: turns one tensor's part of that result into the device table the two cache
 * kernels read (one 16-byte entry per position: source channel, 1/s, s, z).  Validates on the
 * host that perm is a permutation that keeps every channel in its head, that the offsets of
 * every head run from 0 to d / n_heads without decreasing, and the parameters' ranges.
 * d % 32 == 0, and d / n_heads must divide 1024 (a wave handles 1024 consecutive channels).
 * Offline: synchronizes the stream.
 *   s, inv_s, z    host [n_heads, g]: one tensor's slice of rptq_cluster_heads' output
 *   table  device out, rptq_kv_table_bytes(d)
 *
 * rptq_kv_quant: cache codes of a key or value tensor.  For row t and position j with
 * source channel c and cluster parameters (s, z):  q = clamp(round(x[t,c] / s) + z, ...)
 * (Eq. 1, evaluated as in rptq_ln_quant: fp32 product with the stored reciprocal, round half
 * to even).  The layout is dense: d codes per row in the 32-code group formats above
 * (d * bits / 8 bytes per row, no cluster padding).
 *   x device bf16 [T, d] row-major, original channel order;  codes device out [T, d*bits/8]
 *
 * rptq_kv_dequant: reads the cache back, x_hat = s (x_q - z) (the line under Eq. 1): the
 * exact integer difference times the fp32 scale, rounded once to fp32 and then to bf16
 * (ties to even), in the head's cluster order (the order its consumers - the products with
 * queries reordered by the same index - work in).
 *   out device bf16 [T, d]
 */
int32_t rptq_cluster_heads(const float* const* ch_min, const float* const* ch_max, int32_t n_tensors, int32_t d,
                           int32_t n_heads, int32_t g, int32_t bits, uint64_t seed, int32_t max_iter,
                           int32_t* assign, int32_t* perm, int32_t* cluster_off, float* s, float* inv_s, int32_t* z,
                           int32_t* g_eff);
size_t rptq_kv_table_bytes(int32_t d);
int32_t rptq_kv_tables(const int32_t* perm, const int32_t* cluster_off, const float* s, const float* inv_s,
                       const int32_t* z, int32_t d, int32_t n_heads, int32_t g, void* table, void* stream);
int32_t rptq_kv_quant(const void* x, int64_t T, int32_t d, const void* table, int32_t bits, void* codes, void* stream);
int32_t rptq_kv_dequant(const void* codes, int64_t T, int32_t d, const void* table, int32_t bits, void* out,
                        void* stream);

/* ---- helpers for verification (not on the timed path) ---------------------------- */

/* The literal per-cluster integers Yq_i of App. A.4 from the same MFMA main loop:
 * yq device int32 [g,M,N].  zX host [g]; zW, xsum, wsum device. */
int32_t rptq_cluster_gemm_partials(const void* codes_packed, int64_t M, int32_t bits,
                                   const void* Wq_packed, int32_t N, const int32_t* cluster_off, int32_t g,
                                   const int32_t* zX, const int32_t* zW, const int32_t* xsum,
                                   const int32_t* wsum, int32_t* yq, void* stream);
/* Packed activation codes -> int8 [rows,K] in cluster order with padding removed. */
int32_t rptq_unpack_codes(const void* codes_packed, int64_t rows, const int32_t* cluster_off, int32_t g,
                          int32_t bits, int8_t* out, void* stream);
/* Packed weights -> int8 [N,K] in cluster order with padding removed. */
int32_t rptq_unpack_weights(const void* Wq_packed, int32_t N, const int32_t* cluster_off, int32_t g,
                            int8_t* out, void* stream);
/* Per-channel min/max part of rptq_calibrate alone (device results, fp32 [d] each);
 * asynchronous.  workspace as for rptq_calibrate. */
int32_t rptq_channel_minmax(const void* const* x_batches, const int64_t* rows, int32_t n_batches, int32_t d,
                            const float* gamma, const float* beta, float eps, int32_t relu,
                            float* ch_min_dev, float* ch_max_dev, void* workspace, size_t workspace_bytes,
                            void* stream);
/* Host-only part of rptq_calibrate: K-Means, reorder index, parameters from given min/max. */
int32_t rptq_cluster_channels(const float* ch_min, const float* ch_max, int32_t d, int32_t g, int32_t bits,
                              uint64_t seed, int32_t max_iter, int32_t* assign, int32_t* perm,
                              int32_t* cluster_off, float* s, float* inv_s, int32_t* z, int32_t* g_eff);

/* What the current device reports about itself, for roofline denominators: compute units,
 * engine clock and memory clock in kHz, memory bus width in bits (each may be NULL). */
int32_t rptq_device_info(int32_t* compute_units, int32_t* clock_khz, int32_t* memory_clock_khz,
                         int32_t* memory_bus_bits);

const char* rptq_strerror(int32_t status);
int32_t rptq_last_hip_error(void);
const char* rptq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RPTQ_H */
