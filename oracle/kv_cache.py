"""CPU oracle for the attention-site part of RPTQ.  TEST INFRASTRUCTURE ONLY.

What it covers (arXiv 2304.01089):

* one reorder index per attention head shared by queries and keys, from K-Means
  over the four-number points (Qmax, Qmin, Kmax, Kmin) of the head's channels
  (Sec. 4.2, last paragraph; per-head indices: Sec. 5.1), and the ordinary
  two-number points for a tensor clustered alone (the value cache);
* the key/value-cache codes of the W4A4KV / W4A3KV / W3A3KV settings (Sec. 5.1):
  per head, channels in cluster order, Eq. 1 with one Eq. 2 pair per cluster;
* reading the cache back: x_hat = s (x_q - z), the line under Eq. 1.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
module.  It shares no code with the HIP library and never calls it.

Parity status (tests/test_oracle_kv.py):

* cluster_heads ........ per head equal to kmeans_points / kmeans + the pinned
  reorder_index and cluster_params; Q K^T unchanged by the shared index  -> pinned
* kv_quant ............. per head equal to the pinned ln_quant without LayerNorm
                                                                        -> pinned
* kv_dequant ........... exact rational arithmetic on samples (fp32 product,
  bf16 round-half-even), error bound s/2 of the round trip              -> pinned
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence

import numpy as np

from . import rptq_oracle as o

F32 = np.float32
F64 = np.float64


@dataclass
class HeadClusters:
    n_heads: int
    d_head: int
    g: int
    assign: np.ndarray        # [D] cluster of each channel inside its head (canonical ids)
    perm: np.ndarray          # [D] reordered position j holds original channel perm[j]; heads stay in place
    cluster_off: np.ndarray   # [H, g+1] offsets inside the head; clusters that do not exist repeat the last offset
    g_eff: np.ndarray         # [H]
    s: np.ndarray             # [n_tensors, H, g] fp32 (1 where the cluster does not exist)
    inv_s: np.ndarray
    z: np.ndarray             # [n_tensors, H, g] int64


def cluster_heads(ch_min: Sequence[np.ndarray], ch_max: Sequence[np.ndarray], n_heads: int, g: int, bits: int,
                  seed: int = 0, max_iter: int = 100) -> HeadClusters:
    """One clustering per attention head (Sec. 5.1) over the head's channels.

    One tensor (ch_min/ch_max lists of length 1): the points are (min, max) as
    in Sec. 4.1.  Two tensors (queries, keys): the points are
    (Qmax, Qmin, Kmax, Kmin) and both tensors get the same reorder index
    (Sec. 4.2).  Head h uses seed + h.  Every tensor gets its own Eq. 2 pair per
    cluster from its own extrema over the cluster's channels."""
    nt = len(ch_min)
    assert nt in (1, 2) and len(ch_max) == nt
    D = np.asarray(ch_min[0]).shape[0]
    dh = D // n_heads
    assert dh * n_heads == D and 1 <= g <= dh
    assign = np.empty(D, dtype=np.int32)
    perm = np.empty(D, dtype=np.int32)
    off = np.zeros((n_heads, g + 1), dtype=np.int32)
    g_eff = np.zeros(n_heads, dtype=np.int32)
    s = np.ones((nt, n_heads, g), dtype=F32)
    inv_s = np.ones((nt, n_heads, g), dtype=F32)
    z = np.zeros((nt, n_heads, g), dtype=np.int64)
    for h in range(n_heads):
        sl = slice(h * dh, (h + 1) * dh)
        if nt == 1:
            raw, _, _ = o.kmeans(ch_min[0][sl], ch_max[0][sl], g, seed + h, max_iter)
        else:
            pts = np.stack([ch_max[0][sl], ch_min[0][sl], ch_max[1][sl], ch_min[1][sl]], axis=1)
            raw, _, _ = o.kmeans_points(pts, g, seed + h, max_iter)
        lab, ge = o.canonical_labels(raw)
        p, co = o.reorder_index(lab, ge)
        assign[sl] = lab
        perm[sl] = p + h * dh
        off[h, :ge + 1] = co
        off[h, ge + 1:] = co[-1]
        g_eff[h] = ge
        for t in range(nt):
            st, it, zt, _, _ = o.cluster_params(np.asarray(ch_min[t])[sl], np.asarray(ch_max[t])[sl], p, co, bits)
            s[t, h, :ge], inv_s[t, h, :ge], z[t, h, :ge] = st, it, zt
    return HeadClusters(n_heads, dh, g, assign, perm, off, g_eff, s, inv_s, z)


def position_tables(hc: HeadClusters, tensor: int = 0):
    """Per reordered position: (s, inv_s, z) of the cluster the position falls in."""
    D = hc.n_heads * hc.d_head
    s = np.empty(D, dtype=F32)
    inv = np.empty(D, dtype=F32)
    z = np.empty(D, dtype=np.int64)
    for h in range(hc.n_heads):
        for i in range(int(hc.g_eff[h])):
            a, b = h * hc.d_head + hc.cluster_off[h, i], h * hc.d_head + hc.cluster_off[h, i + 1]
            s[a:b], inv[a:b], z[a:b] = hc.s[tensor, h, i], hc.inv_s[tensor, h, i], hc.z[tensor, h, i]
    return s, inv, z


def kv_quant(x, hc: HeadClusters, tensor: int, k: int):
    """Cache codes of a key or value tensor x [T, D] (bf16-exact fp32, original
    channel order): position j holds Q_k(x[:, perm[j]]; s, z of j's cluster)
    (Eq. 1; App. A.4 first equation).  Returns int32 [T, D] in cluster order."""
    _, inv, z = position_tables(hc, tensor)
    a = np.asarray(x, dtype=F32)[:, hc.perm]
    return o.quantize(a, inv[None, :], z[None, :], k)


round_to_bf16 = o.round_to_bf16      # fp32 -> nearest bf16 (ties to even), returned as fp32


def kv_dequant(codes, hc: HeadClusters, tensor: int, original_order: bool = False):
    """x_hat = s (x_q - z) (the line under Eq. 1) as the cache reader delivers it:
    the product of the fp32 scale and the exact integer, rounded once to fp32
    and then to bf16 (ties to even).  Cluster order, or original channel order
    when asked.  Returns fp32 [T, D] holding bf16 values."""
    s, _, z = position_tables(hc, tensor)
    n = (np.asarray(codes, dtype=np.int64) - z[None, :]).astype(F32)      # exact: |n| < 2^24
    y = round_to_bf16(s[None, :] * n)                                     # one fp32 rounding, then bf16
    if original_order:
        out = np.empty_like(y)
        out[:, hc.perm] = y
        return out
    return y
