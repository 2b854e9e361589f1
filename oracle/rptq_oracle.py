"""CPU oracle for the RPTQ inference hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, numpy implementation of what the hot path computes, written
from the paper (arXiv 2304.01089): calibration min/max, K-Means over the
per-channel (min, max) points, the reorder index, Min-Max parameters per
cluster, LayerNorm followed by per-cluster quantization, per-output-channel
weight quantization, and the two forms of the cluster-wise matrix product.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this module.  It shares no code with the HIP library and never calls it.

Arithmetic is float64 and exact integers, except where the method's own
working precision is part of the result (the fp32 LayerNorm chain that decides
the integer codes); those places say so.

Parity status of each function (what pins it, in tests/test_oracle_*.py):

* quantize / minmax_params ........ printed 4-bit range, Eq. 1-2 worked
  examples, dequantization error bound                        -> pinned
* layernorm_f32 ................... torch fp64 layer_norm, constant rows,
  zero-mean/unit-variance property                            -> pinned
* calibrate_minmax ................ numpy min/max, brute force -> pinned
* kmeans .......................... brute-force optimal partition on tiny
  inputs, 1-D interval DP optimum, Lloyd invariants, pure-Python re-run of
  the sequential sums.  The seeding rule is this build's choice (the paper
  names none): partition *quality* beyond those cases is  parity unpinned.
* reorder_index / cluster_params .. permutation properties, g=1 and g=C
  special cases                                               -> pinned
* ln_quant ........................ explicit permute-then-quantize, g=1
  per-tensor and g=C per-channel reductions                   -> pinned
* quantize_weights ................ Eq. 1-2 per row, permutation invariance
                                                              -> pinned
* cluster_gemm_int ................ triple-loop brute force on tiny shapes;
  equality with cluster_gemm_dequant (App. A.4, method 1 == method 2)
                                                              -> pinned
* kmeans_points ................... equals kmeans bit for bit in two
  dimensions; brute-force optimal partition of tiny 4-D inputs; pure-Python
  re-run; Lloyd invariants (partition quality beyond that: parity unpinned,
  as for kmeans)                                              -> pinned
* quantize_weights_per_cluster .... Eq. 1-2 written out per (row, cluster);
  one cluster reduces to quantize_weights                     -> pinned
* cluster_gemm_int_pc / cluster_gemm_dequant_pc (App. A.4 with its own
  per-(output, cluster) weight parameters) ... triple loop; method 1 ==
  method 2; reduces to cluster_gemm_int when every cluster of a row carries
  the row's pair                                              -> pinned
* round_to_bf16 / dequantize_bf16 / cluster_gemm_dequant_bf16 (App. A.4,
  method 1 on bf16 operands) ... exact rational rounding on samples and ties;
  identical to cluster_gemm_dequant when every de-quantized value is a bf16
  number; otherwise within the rounding bound of two bf16 operands -> pinned
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

F32 = np.float32
F64 = np.float64

Z_LIMIT = 1 << 21          # |zero point| accepted by the path (fp32-exact offsets)


# ---------------------------------------------------------------------------
# Eq. 1 and Eq. 2
# ---------------------------------------------------------------------------
def code_range(k: int) -> Tuple[int, int]:
    """Signed k-bit range of Eq. 1: [-2^(k-1), 2^(k-1)-1]."""
    return -(1 << (k - 1)), (1 << (k - 1)) - 1


def minmax_params(xmin, xmax, k: int):
    """Min-Max rule, Eq. 2: s = (Xmax-Xmin)/2^k, z = -round((Xmax+Xmin)/(2s)).

    Inputs are the fp32 extrema of the group that shares (s, z); the rule is
    evaluated in float64 and round is round-half-to-even.  Returns
    (s32, inv_s32, z): the scale rounded to fp32, the fp32 reciprocal the
    quantizer multiplies by, and the integer zero point.  A group with
    Xmax == Xmin (Eq. 2 would divide by zero) gets s = 1, z = -round(Xmin).
    """
    lo = np.asarray(xmin, dtype=F32).astype(F64)
    hi = np.asarray(xmax, dtype=F32).astype(F64)
    degenerate = hi == lo
    span = np.where(degenerate, 1.0, hi - lo)
    s64 = np.where(degenerate, 1.0, span / float(1 << k))
    z = np.where(degenerate, -np.rint(lo), -np.rint((hi + lo) / (2.0 * s64)))
    z = z + 0.0                                   # -0.0 -> +0.0
    s32 = s64.astype(F32)
    inv_s32 = (1.0 / s32.astype(F64)).astype(F32)
    return s32, inv_s32, z.astype(np.int64)


def quantize(x, inv_s, z, k: int):
    """Q_k of Eq. 1 on fp32 values: clamp(round(x/s) + z, -2^(k-1), 2^(k-1)-1).

    x/s is evaluated as the fp32 product x * inv_s (inv_s the stored fp32
    reciprocal of s); round is round-half-to-even; the order round, add z,
    clamp is the printed one.  Broadcasts inv_s and z against x.
    """
    lo, hi = code_range(k)
    r = np.asarray(x, dtype=F32) * np.asarray(inv_s, dtype=F32)      # one fp32 rounding
    q = np.rint(r.astype(F64)) + np.asarray(z, dtype=F64)
    return np.clip(q, lo, hi).astype(np.int32)


def dequantize(q, s, z):
    """x_hat = s (x_q - z), the line under Eq. 1, in float64."""
    return np.asarray(s, dtype=F64) * (np.asarray(q, dtype=F64) - np.asarray(z, dtype=F64))


# ---------------------------------------------------------------------------
# LayerNorm in the path's working precision
# ---------------------------------------------------------------------------
FRAGILE_REL = 2.0 ** -44


def _fp32_midpoint_distance(v64: np.ndarray) -> np.ndarray:
    """Distance from each float64 value to the nearest fp32 rounding boundary."""
    v32 = v64.astype(F32)
    up = np.nextafter(v32, F32(np.inf)).astype(F64)
    dn = np.nextafter(v32, F32(-np.inf)).astype(F64)
    c = v32.astype(F64)
    return np.minimum(np.abs(v64 - 0.5 * (c + up)), np.abs(v64 - 0.5 * (c + dn)))


def layernorm_f32(x, gamma, beta, eps: float):
    """LayerNorm over the last axis with biased variance (standard definition;
    the paper's section on avoiding explicit reordering takes it as given).

    Row statistics are evaluated in float64 from the bf16-exact inputs
    (two-pass) and rounded once to fp32; the per-element chain is five
    separately rounded fp32 operations, t = x - mu; u = t * rstd;
    v = u * gamma; y = v + beta (the fifth, y * inv_s, belongs to quantize).

    Returns (y fp32 [M,d], fragile bool [M]).  A row is fragile when its
    float64 mean or rstd lies so close to an fp32 rounding boundary that a
    different summation order (mean) or an algebraically equal variance
    formula (rstd) could round it the other way.
    """
    x = np.asarray(x, dtype=F32)
    d = x.shape[-1]
    xd = x.astype(F64)
    mu = xd.sum(axis=-1) / d
    dev = xd - mu[..., None]
    var = (dev * dev).sum(axis=-1) / d
    rstd = 1.0 / np.sqrt(var + float(eps))
    mean_abs = np.abs(xd).sum(axis=-1) / d
    # bf16 inputs are multiples of their smallest element's ulp q; while sum|x| < 2^52 q every
    # partial sum in any order is exact in float64, so the mean cannot depend on the order.
    mag = np.where(xd != 0.0, np.abs(xd), np.inf)
    q = np.exp2(np.floor(np.log2(mag.min(axis=-1))) - 7.0)
    order_free = ~np.isfinite(q) | (mean_abs * d < 2.0 ** 52 * q)
    ratio = 1.0 + mu * mu / np.maximum(var, 1e-300)
    fragile = (~order_free & (_fp32_midpoint_distance(mu) < FRAGILE_REL * np.maximum(mean_abs, 1e-300))) | (
        _fp32_midpoint_distance(rstd) < FRAGILE_REL * rstd * np.minimum(ratio, 1e30))
    mu32 = mu.astype(F32)[..., None]
    rstd32 = rstd.astype(F32)[..., None]
    t = x - mu32
    u = t * rstd32
    v = u * np.asarray(gamma, dtype=F32)
    y = v + np.asarray(beta, dtype=F32)
    return y, fragile


def site_activation(x, gamma=None, beta=None, eps: float = 1e-5, relu: bool = False):
    """The tensor a quantization site sees: LN(x) at a LayerNorm site, else x
    or max(x, 0).  Returns (a fp32, fragile rows)."""
    if gamma is not None:
        y, fragile = layernorm_f32(x, gamma, beta, eps)
    else:
        y = np.asarray(x, dtype=F32)
        fragile = np.zeros(y.shape[:-1], dtype=bool)
    if relu:
        y = np.maximum(y, F32(0.0))
    return y, fragile


# ---------------------------------------------------------------------------
# Calibration: per-channel min / max (Sec. 4.1, first displayed equation)
# ---------------------------------------------------------------------------
def calibrate_minmax(batches: Sequence[np.ndarray], gamma=None, beta=None,
                     eps: float = 1e-5, relu: bool = False):
    """X_min[c], X_max[c] over every calibration row of the site's activation."""
    cmin = None
    cmax = None
    for xb in batches:
        a, _ = site_activation(xb, gamma, beta, eps, relu)
        a = a.reshape(-1, a.shape[-1])
        bmin = a.min(axis=0)
        bmax = a.max(axis=0)
        cmin = bmin if cmin is None else np.minimum(cmin, bmin)
        cmax = bmax if cmax is None else np.maximum(cmax, bmax)
    return (cmin + F32(0.0)).astype(F32), (cmax + F32(0.0)).astype(F32)   # -0.0 -> +0.0


# ---------------------------------------------------------------------------
# K-Means over the points (X_min_c, X_max_c)  (Sec. 4.1)
# ---------------------------------------------------------------------------
class SplitMix64:
    """Counter-based 64-bit generator (Steele, Lea, Flood 2014): state += golden
    gamma; output = mix(state).  uniform() is the top 53 bits as [0,1)."""
    MASK = (1 << 64) - 1

    def __init__(self, seed: int):
        self.state = seed & self.MASK

    def next_u64(self) -> int:
        self.state = (self.state + 0x9E3779B97F4A7C15) & self.MASK
        zz = self.state
        zz = ((zz ^ (zz >> 30)) * 0xBF58476D1CE4E5B9) & self.MASK
        zz = ((zz ^ (zz >> 27)) * 0x94D049BB133111EB) & self.MASK
        return zz ^ (zz >> 31)

    def uniform(self) -> float:
        return (self.next_u64() >> 11) * (1.0 / 9007199254740992.0)


def _sqdist(px, py, cx, cy):
    dx = px - cx
    dy = py - cy
    return dx * dx + dy * dy          # three separately rounded float64 operations


def kmeans(ch_min, ch_max, g: int, seed: int = 0, max_iter: int = 100):
    """Lloyd's K-Means on the C points (X_min_c, X_max_c), Euclidean, raw units.

    The paper asks for K-Means and fixes nothing else, so the rule here is this
    build's reading: D^2-weighted seeding (k-means++) driven by SplitMix64(seed),
    then assign / update until the assignment repeats or max_iter passes.
    Everything is float64; per-cluster sums run over members in ascending
    channel index; ties go to the lowest cluster id; an empty cluster is
    re-seeded with the point farthest from its own centre (lowest index on
    ties).  Returns (labels[C] in raw cluster ids, centres[g_used, 2], n_iter).
    """
    px = np.asarray(ch_min, dtype=F32).astype(F64)
    py = np.asarray(ch_max, dtype=F32).astype(F64)
    C = px.shape[0]
    if not (1 <= g <= C):
        raise ValueError("g must be in [1, C]")
    rng = SplitMix64(seed)

    # --- seeding ---------------------------------------------------------
    first = min(int(rng.uniform() * C), C - 1)
    cx = [px[first]]
    cy = [py[first]]
    d2 = _sqdist(px, py, cx[0], cy[0])
    while len(cx) < g:
        cum = np.cumsum(d2)                       # sequential prefix sums
        total = cum[-1]
        if not total > 0.0:                       # fewer distinct points than g
            break
        target = rng.uniform() * total
        nxt = min(int(np.searchsorted(cum, target, side="right")), C - 1)
        cx.append(px[nxt])
        cy.append(py[nxt])
        d2 = np.minimum(d2, _sqdist(px, py, cx[-1], cy[-1]))
    gk = len(cx)
    cx = np.array(cx, dtype=F64)
    cy = np.array(cy, dtype=F64)

    # --- Lloyd iterations --------------------------------------------------
    labels = np.full(C, -1, dtype=np.int64)
    n_iter = 0
    for n_iter in range(1, max_iter + 1):
        dist = _sqdist(px[:, None], py[:, None], cx[None, :], cy[None, :])   # [C, gk]
        new_labels = np.argmin(dist, axis=1)      # first minimum = lowest cluster id
        if np.array_equal(new_labels, labels):
            break
        labels = new_labels
        cnt = np.bincount(labels, minlength=gk)
        sx = np.bincount(labels, weights=px, minlength=gk)   # ascending-index sums
        sy = np.bincount(labels, weights=py, minlength=gk)
        nz = cnt > 0
        cx = np.where(nz, sx / np.maximum(cnt, 1), cx)
        cy = np.where(nz, sy / np.maximum(cnt, 1), cy)
        if not nz.all():
            own = _sqdist(px, py, cx[labels], cy[labels])
            for kk in np.nonzero(~nz)[0]:
                far = int(np.argmax(own))         # first maximum = lowest index
                cx[kk] = px[far]
                cy[kk] = py[far]
                own[far] = -1.0
            labels = np.full(C, -1, dtype=np.int64)          # force another pass
    if (labels < 0).any():                        # max_iter ended on a re-seed pass
        dist = _sqdist(px[:, None], py[:, None], cx[None, :], cy[None, :])
        labels = np.argmin(dist, axis=1)
    return labels.astype(np.int64), np.stack([cx, cy], axis=1), n_iter


def _sqdist_nd(P, cen):
    """Squared Euclidean distance of every point [C, D] to one centre [D]:
    the squares are added in dimension order (separately rounded float64)."""
    acc = None
    for j in range(P.shape[-1]):
        dj = P[..., j] - cen[..., j]
        sq = dj * dj
        acc = sq if acc is None else acc + sq
    return acc


def kmeans_points(points, g: int, seed: int = 0, max_iter: int = 100):
    """The rule of `kmeans` on points of any dimension (used for the points
    (Qmax, Qmin, Kmax, Kmin) that give queries and keys one shared reorder
    index, Sec. 4.2): D^2-weighted seeding from SplitMix64(seed), Lloyd
    iterations until the assignment repeats, ties to the lowest cluster id,
    member sums in ascending point index, empty clusters re-seeded with the
    point farthest from its own centre.  Squared distances add their terms in
    dimension order.  Returns (labels[C], centres[g_used, D], n_iter)."""
    P = np.asarray(points, dtype=F32).astype(F64)
    C, D = P.shape
    if not (1 <= g <= C):
        raise ValueError("g must be in [1, C]")
    rng = SplitMix64(seed)
    first = min(int(rng.uniform() * C), C - 1)
    cen = [P[first].copy()]
    d2 = _sqdist_nd(P, cen[0])
    while len(cen) < g:
        cum = np.cumsum(d2)
        total = cum[-1]
        if not total > 0.0:
            break
        target = rng.uniform() * total
        nxt = min(int(np.searchsorted(cum, target, side="right")), C - 1)
        cen.append(P[nxt].copy())
        d2 = np.minimum(d2, _sqdist_nd(P, cen[-1]))
    gk = len(cen)
    cen = np.stack(cen, axis=0)
    labels = np.full(C, -1, dtype=np.int64)
    n_iter = 0
    for n_iter in range(1, max_iter + 1):
        dist = _sqdist_nd(P[:, None, :], cen[None, :, :])            # [C, gk]
        new_labels = np.argmin(dist, axis=1)
        if np.array_equal(new_labels, labels):
            break
        labels = new_labels
        cnt = np.bincount(labels, minlength=gk)
        nz = cnt > 0
        for j in range(D):
            sj = np.bincount(labels, weights=P[:, j], minlength=gk)
            cen[:, j] = np.where(nz, sj / np.maximum(cnt, 1), cen[:, j])
        if not nz.all():
            own = _sqdist_nd(P, cen[labels])
            for kk in np.nonzero(~nz)[0]:
                far = int(np.argmax(own))
                cen[kk] = P[far]
                own[far] = -1.0
            labels = np.full(C, -1, dtype=np.int64)
    if (labels < 0).any():
        dist = _sqdist_nd(P[:, None, :], cen[None, :, :])
        labels = np.argmin(dist, axis=1)
    return labels.astype(np.int64), cen, n_iter


def canonical_labels(labels):
    """Relabel clusters by first occurrence: the cluster holding channel 0 is 0,
    the next unseen cluster is 1, ...  Empty clusters disappear."""
    labels = np.asarray(labels)
    out = np.empty(labels.shape[0], dtype=np.int32)
    seen = {}
    for i, l in enumerate(labels.tolist()):
        if l not in seen:
            seen[l] = len(seen)
        out[i] = seen[l]
    return out, len(seen)


def reorder_index(assign, g_eff: int):
    """S = [S^1, ..., S^g] (Sec. 4.1): channels sorted by (cluster, original
    index).  Returns (perm[C] with x_reordered[:, j] = x[:, perm[j]],
    cluster_off[g_eff+1])."""
    assign = np.asarray(assign, dtype=np.int64)
    perm = np.argsort(assign, kind="stable").astype(np.int32)
    counts = np.bincount(assign, minlength=g_eff)
    off = np.zeros(g_eff + 1, dtype=np.int32)
    off[1:] = np.cumsum(counts)
    return perm, off


def cluster_params(ch_min, ch_max, perm, cluster_off, k: int):
    """One (s, z) per cluster (Sec. 4.1; Sec. 5.1 settings): the cluster's range
    is the min of its members' minima and the max of their maxima, then Eq. 2."""
    g = len(cluster_off) - 1
    lo = np.empty(g, dtype=F32)
    hi = np.empty(g, dtype=F32)
    for i in range(g):
        members = perm[cluster_off[i]:cluster_off[i + 1]]
        lo[i] = np.asarray(ch_min, dtype=F32)[members].min()
        hi[i] = np.asarray(ch_max, dtype=F32)[members].max()
    s, inv_s, z = minmax_params(lo, hi, k)
    return s, inv_s, z, lo, hi


@dataclass
class Calibration:
    ch_min: np.ndarray
    ch_max: np.ndarray
    assign: np.ndarray        # canonical cluster id per original channel
    perm: np.ndarray
    cluster_off: np.ndarray
    s: np.ndarray
    inv_s: np.ndarray
    z: np.ndarray
    g_eff: int


def calibrate(batches, gamma, beta, eps, relu, g, bits, seed=0, max_iter=100) -> Calibration:
    """Min/max, K-Means, reorder index and per-cluster parameters in one call."""
    ch_min, ch_max = calibrate_minmax(batches, gamma, beta, eps, relu)
    raw, _, _ = kmeans(ch_min, ch_max, g, seed, max_iter)
    assign, g_eff = canonical_labels(raw)
    perm, off = reorder_index(assign, g_eff)
    s, inv_s, z, _, _ = cluster_params(ch_min, ch_max, perm, off, bits)
    return Calibration(ch_min, ch_max, assign, perm, off, s, inv_s, z, g_eff)


# ---------------------------------------------------------------------------
# Reorder folded into LayerNorm and weights (Sec. 4.2)
# ---------------------------------------------------------------------------
def fold_layernorm(gamma, beta, perm):
    """gamma', beta' in cluster order: LN' emits channel perm[j] at position j."""
    return np.asarray(gamma, dtype=F32)[perm], np.asarray(beta, dtype=F32)[perm]


def ln_quant(x, gamma, beta, eps, relu, perm, cluster_off, inv_s, z, k: int):
    """Site activation in cluster order, quantized per cluster (App. A.4, first
    equation).  perm=None means x is already in cluster order.

    Returns (codes int32 [M,d] in cluster order, xsum int64 [M,g] per-cluster
    code sums, fragile rows)."""
    a, fragile = site_activation(x, gamma, beta, eps, relu)      # original channel order
    if perm is not None:
        a = a[:, perm]                                           # X~[:, j] = X[:, S_j]
    g = len(cluster_off) - 1
    sizes = np.diff(cluster_off)
    inv_col = np.repeat(np.asarray(inv_s, dtype=F32), sizes)
    z_col = np.repeat(np.asarray(z, dtype=np.int64), sizes)
    codes = quantize(a, inv_col[None, :], z_col[None, :], k)
    xsum = np.stack([codes[:, cluster_off[i]:cluster_off[i + 1]].sum(axis=1, dtype=np.int64)
                     for i in range(g)], axis=1)
    return codes, xsum, fragile


def quantize_weights(W, perm_in, perm_out=None, k: int = 4):
    """W~ = W[perm_out][:, perm_in] (Sec. 4.2), then Eq. 1-2 with one (s, z) per
    output channel over the whole row.  Returns (wq int32 [N,K], sW fp32 [N],
    inv_sW fp32 [N], zW int64 [N])."""
    W = np.asarray(W, dtype=F32)
    if perm_out is not None:
        W = W[perm_out]
    Wt = W[:, perm_in]
    s, inv_s, z = minmax_params(Wt.min(axis=1), Wt.max(axis=1), k)
    wq = quantize(Wt, inv_s[:, None], z[:, None], k)
    return wq, s, inv_s, z


def quantize_weights_per_cluster(W, perm_in, cluster_off, perm_out=None, k: int = 4):
    """The weight scheme of App. A.4 as printed: W~ = W[perm_out][:, perm_in] is
    divided along its input channels into the activation's clusters and every
    (output channel o, cluster i) block gets its own Eq. 2 pair
    (s^W_{o,i}, z^W_{o,i}) from the block's minimum and maximum, then Eq. 1.
    Returns (wq int32 [N,K], sW fp32 [N,g], inv_sW fp32 [N,g], zW int64 [N,g])."""
    W = np.asarray(W, dtype=F32)
    if perm_out is not None:
        W = W[perm_out]
    Wt = W[:, perm_in]
    g = len(cluster_off) - 1
    N = Wt.shape[0]
    wq = np.empty(Wt.shape, dtype=np.int32)
    sW = np.empty((N, g), dtype=F32)
    inv = np.empty((N, g), dtype=F32)
    zW = np.empty((N, g), dtype=np.int64)
    for i in range(g):
        a, b = int(cluster_off[i]), int(cluster_off[i + 1])
        blk = Wt[:, a:b]
        sW[:, i], inv[:, i], zW[:, i] = minmax_params(blk.min(axis=1), blk.max(axis=1), k)
        wq[:, a:b] = quantize(blk, inv[:, i][:, None], zW[:, i][:, None], k)
    return wq, sW, inv, zW


# ---------------------------------------------------------------------------
# Cluster-wise product (App. A.4)
# ---------------------------------------------------------------------------
def cluster_gemm_dequant(xq, wq, cluster_off, sX, zX, sW, zW):
    """Method 1: de-quantize both operands, concatenate, Y = X_hat W_hat^T (fp64)."""
    sizes = np.diff(cluster_off)
    sx_col = np.repeat(np.asarray(sX, dtype=F64), sizes)
    zx_col = np.repeat(np.asarray(zX, dtype=F64), sizes)
    xh = sx_col[None, :] * (np.asarray(xq, dtype=F64) - zx_col[None, :])
    wh = np.asarray(sW, dtype=F64)[:, None] * (np.asarray(wq, dtype=F64) - np.asarray(zW, dtype=F64)[:, None])
    return xh @ wh.T


def round_to_bf16(x32):
    """fp32 -> nearest bf16 (ties to even), returned as fp32."""
    u = np.ascontiguousarray(x32, dtype=F32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r & np.uint32(0xFFFF0000)).view(F32)


def dequantize_bf16(q, s, z):
    """x_hat = s (x_q - z) (the line under Eq. 1) held as bf16: the integer
    difference is exact in fp32, the product with the fp32 scale is rounded once
    to fp32 and once more to bf16 (ties to even).  Returns fp32 holding bf16 values."""
    n = (np.asarray(q, dtype=np.int64) - np.asarray(z, dtype=np.int64)).astype(F32)
    return round_to_bf16(np.asarray(s, dtype=F32) * n)


def cluster_gemm_dequant_bf16(xq, wq, cluster_off, sX, zX, sW, zW):
    """Method 1 of App. A.4 on 16-bit floating-point operands: both tensors are
    de-quantized to bf16 (dequantize_bf16) and multiplied, Y = X_hat W_hat^T.  The
    product itself is exact here (fp64 of bf16 values: every term has 16
    significant bits); the GPU accumulates it in fp32.
    Returns (X_hat fp32 [M,K], W_hat fp32 [N,K], Y float64 [M,N])."""
    sizes = np.diff(cluster_off)
    sx_col = np.repeat(np.asarray(sX, dtype=F32), sizes)
    zx_col = np.repeat(np.asarray(zX, dtype=np.int64), sizes)
    xh = dequantize_bf16(xq, sx_col[None, :], zx_col[None, :])
    wh = dequantize_bf16(wq, np.asarray(sW, dtype=F32)[:, None], np.asarray(zW, dtype=np.int64)[:, None])
    return xh, wh, xh.astype(F64) @ wh.astype(F64).T


def cluster_gemm_int(xq, wq, cluster_off, sX, zX, sW, zW):
    """Method 2: per cluster i, the integer
        Yq_i[t,o] = sum_c xq*wq - zX_i * sum_c wq[o,c] - zW_o * sum_c xq[t,c] + n_i zX_i zW_o
    (c over the cluster's n_i channels; the printed last term omits n_i, which
    the algebra of method 1 requires), then Y = sum_i sX_i sW_o Yq_i.

    The integer products run as float64 matrix products of integer-valued
    operands, exact while every partial sum stays below 2^53.
    Returns (P int64 [g,M,N] raw products, Yq int64 [g,M,N], Y float64 [M,N])."""
    xq = np.asarray(xq)
    wq = np.asarray(wq)
    g = len(cluster_off) - 1
    M, N = xq.shape[0], wq.shape[0]
    P = np.empty((g, M, N), dtype=np.int64)
    Yq = np.empty((g, M, N), dtype=np.int64)
    Y = np.zeros((M, N), dtype=F64)
    zW = np.asarray(zW, dtype=np.int64)
    for i in range(g):
        a, b = int(cluster_off[i]), int(cluster_off[i + 1])
        xi = xq[:, a:b].astype(F64)
        wi = wq[:, a:b].astype(F64)
        Pi = np.rint(xi @ wi.T).astype(np.int64)
        wsum = wq[:, a:b].sum(axis=1, dtype=np.int64)
        xsum = xq[:, a:b].sum(axis=1, dtype=np.int64)
        zx = int(zX[i])
        Yq[i] = Pi - zx * wsum[None, :] - zW[None, :] * xsum[:, None] + (b - a) * zx * zW[None, :]
        P[i] = Pi
        Y += float(sX[i]) * np.asarray(sW, dtype=F64)[None, :] * Yq[i].astype(F64)
    return P, Yq, Y


def cluster_gemm_dequant_pc(xq, wq, cluster_off, sX, zX, sW, zW):
    """Method 1 of App. A.4 with per-(output, cluster) weight parameters
    sW, zW [N, g]: de-quantize every cluster block of both operands, Y = X_hat W_hat^T."""
    sizes = np.diff(cluster_off)
    sx_col = np.repeat(np.asarray(sX, dtype=F64), sizes)
    zx_col = np.repeat(np.asarray(zX, dtype=F64), sizes)
    xh = sx_col[None, :] * (np.asarray(xq, dtype=F64) - zx_col[None, :])
    sw_col = np.repeat(np.asarray(sW, dtype=F64), sizes, axis=1)
    zw_col = np.repeat(np.asarray(zW, dtype=F64), sizes, axis=1)
    wh = sw_col * (np.asarray(wq, dtype=F64) - zw_col)
    return xh @ wh.T


def cluster_gemm_int_pc(xq, wq, cluster_off, sX, zX, sW, zW):
    """Method 2 of App. A.4 as printed, with the weight pair of every (output o,
    cluster i): the integer
        Yq_i[t,o] = sum_c xq*wq - zX_i sum_c wq[o,c] - zW[o,i] sum_c xq[t,c] + n_i zX_i zW[o,i]
    and Y = sum_i sX_i sW[o,i] Yq_i.  Returns (Yq int64 [g,M,N], Y float64 [M,N])."""
    xq = np.asarray(xq)
    wq = np.asarray(wq)
    g = len(cluster_off) - 1
    M, N = xq.shape[0], wq.shape[0]
    Yq = np.empty((g, M, N), dtype=np.int64)
    Y = np.zeros((M, N), dtype=F64)
    zW = np.asarray(zW, dtype=np.int64)
    sW = np.asarray(sW, dtype=F64)
    for i in range(g):
        a, b = int(cluster_off[i]), int(cluster_off[i + 1])
        Pi = np.rint(xq[:, a:b].astype(F64) @ wq[:, a:b].astype(F64).T).astype(np.int64)
        wsum = wq[:, a:b].sum(axis=1, dtype=np.int64)
        xsum = xq[:, a:b].sum(axis=1, dtype=np.int64)
        zx = int(zX[i])
        Yq[i] = Pi - zx * wsum[None, :] - zW[None, :, i] * xsum[:, None] + (b - a) * zx * zW[None, :, i]
        Y += float(sX[i]) * sW[None, :, i] * Yq[i].astype(F64)
    return Yq, Y
