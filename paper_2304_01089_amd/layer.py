"""Buffer management around the C entry points: allocates the device tensors a site and
its linear layers need (torch is used for memory only) and calls the library."""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional

import numpy as np

from . import binding as B


@dataclass
class Calibration:
    """Host result of rptq_calibrate for one site, plus device copies the kernels read."""
    d: int
    bits: int
    ch_min: np.ndarray
    ch_max: np.ndarray
    assign: np.ndarray
    perm: np.ndarray
    cluster_off: np.ndarray
    s: np.ndarray
    inv_s: np.ndarray
    z: np.ndarray
    g_eff: int
    k_padded: int
    perm_pad: object = None          # device int32 [K_p]
    perm_pad_host: np.ndarray = None
    gamma_pad: object = None
    beta_pad: object = None


@dataclass
class FoldedLinear:
    N: int
    Wq: object
    sW: object
    zW: object
    wsum: object
    colterm: object


def calibrate_site(x_batches, gamma, beta, eps, relu, g, bits, seed=0, max_iter=100) -> Calibration:
    import torch
    res = B.rptq_calibrate(x_batches, gamma, beta, eps, relu, g, bits, seed, max_iter)
    d = x_batches[0].shape[1]
    cal = Calibration(d=d, bits=bits, k_padded=B.rptq_padded_k(res["cluster_off"]), **res)
    dev = x_batches[0].device
    cal.perm_pad = torch.empty(cal.k_padded, dtype=torch.int32, device=dev)
    if gamma is not None:
        cal.gamma_pad = torch.empty(cal.k_padded, dtype=torch.float32, device=dev)
        cal.beta_pad = torch.empty(cal.k_padded, dtype=torch.float32, device=dev)
    B.rptq_fold_reorder(gamma, beta, d, cal.perm, cal.cluster_off, None, None, None, 0, d, None,
                        cal.perm_pad, cal.gamma_pad, cal.beta_pad, None, None, None, None, None)
    cal.perm_pad_host = cal.perm_pad.cpu().numpy()
    return cal


def identity_site(cal: Calibration) -> Calibration:
    """The same site for an input that already arrives in its cluster order (the output of a
    linear layer whose rows were permuted offline by this site's reorder index): the gather
    is the identity; clusters, parameters and padding are unchanged.  No LayerNorm."""
    import copy
    import torch
    out = copy.copy(cal)
    ident = np.arange(cal.d, dtype=np.int32)
    out.perm = ident
    out.perm_pad = torch.empty_like(cal.perm_pad)
    out.gamma_pad = None
    out.beta_pad = None
    B.rptq_fold_reorder(None, None, cal.d, ident, cal.cluster_off, None, None, None, 0, cal.d, None,
                        out.perm_pad, None, None, None, None, None, None, None)
    out.perm_pad_host = out.perm_pad.cpu().numpy()
    return out


def fold_linear(cal: Calibration, W, perm_out=None, next_site: Optional[Calibration] = None) -> FoldedLinear:
    """perm_out: reorder index of the layer's output (rows of W), a host array.  next_site: lay the rows out
    as that site's padded cluster-order positions instead (pad rows are zero), which is what
    cluster_gemm_quant needs; the layer then has next_site.k_padded outputs."""
    import torch
    N, K = W.shape
    if next_site is not None:
        perm_out = next_site.perm_pad_host
        N = next_site.k_padded
    dev = W.device
    out = FoldedLinear(
        N=N,
        Wq=torch.empty(B.rptq_weight_bytes(N, cal.k_padded), dtype=torch.uint8, device=dev),
        sW=torch.empty(N, dtype=torch.float32, device=dev),
        zW=torch.empty(N, dtype=torch.int32, device=dev),
        wsum=torch.empty((N, cal.g_eff), dtype=torch.int32, device=dev),
        colterm=torch.empty(N, dtype=torch.float32, device=dev))
    B.rptq_fold_reorder(None, None, cal.d, cal.perm, cal.cluster_off, cal.s, cal.z, W, N, K, perm_out,
                        cal.perm_pad, None, None, out.Wq, out.sW, out.zW, out.wsum, out.colterm)
    return out


def ln_quant(cal: Calibration, x, eps=1e-5, relu=False, codes=None, xsum=None, rowterm=None, want_xsum=False):
    import torch
    M = x.shape[0]
    dev = x.device
    if codes is None:
        codes = torch.empty(B.rptq_codes_bytes(M, cal.k_padded, cal.bits), dtype=torch.uint8, device=dev)
    if rowterm is None:
        rowterm = torch.empty(M, dtype=torch.float32, device=dev)
    if xsum is None and want_xsum:
        xsum = torch.empty((M, cal.g_eff), dtype=torch.int32, device=dev)
    B.rptq_ln_quant(x, M, cal.d, cal.gamma_pad, cal.beta_pad, eps, relu, cal.perm_pad, cal.cluster_off,
                    cal.s, cal.inv_s, cal.z, cal.bits, codes, xsum, rowterm)
    return codes, xsum, rowterm


def cluster_gemm(cal: Calibration, lin: FoldedLinear, codes, rowterm, M, y=None, dtype=None):
    import torch
    if y is None:
        y = torch.empty((M, lin.N), dtype=dtype or torch.bfloat16, device=codes.device)
    B.rptq_cluster_gemm(codes, M, cal.bits, lin.Wq, lin.N, cal.cluster_off, cal.s, lin.sW, lin.zW, lin.colterm,
                        rowterm, y)
    return y


def cluster_gemm_quant(cal: Calibration, lin: FoldedLinear, codes, rowterm, M, next_site: Calibration, relu=True,
                       next_codes=None, next_rowterm=None, workspace=None):
    """The product of `lin` (folded with next_site=...) quantized for `next_site` in the output stage."""
    import torch
    dev = codes.device
    if next_codes is None:
        next_codes = torch.empty(B.rptq_codes_bytes(M, next_site.k_padded, next_site.bits), dtype=torch.uint8, device=dev)
    if next_rowterm is None:
        next_rowterm = torch.empty(M, dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty(max(16, B.rptq_cluster_gemm_quant_workspace_bytes(M, lin.N)), dtype=torch.uint8, device=dev)
    B.rptq_cluster_gemm_quant(codes, M, cal.bits, lin.Wq, lin.N, cal.cluster_off, cal.s, lin.sW, lin.zW, lin.colterm,
                              rowterm, relu, next_site.cluster_off, next_site.s, next_site.inv_s, next_site.z,
                              next_site.bits, next_codes, next_rowterm, workspace)
    return next_codes, next_rowterm


# ---- weights with one parameter pair per (output channel, input cluster): App. A.4 as printed ----
@dataclass
class FoldedLinearCw:
    N: int
    Wq: object
    sW: object            # [N, g]
    zW: object            # [N, g]
    wsum: object          # [N, g]
    scale_tab: object     # [g, N_p]
    cross_tab: object     # [N_p, 32]
    colterm: object       # [N]


def fold_linear_cw(cal: Calibration, W, perm_out=None) -> FoldedLinearCw:
    import torch
    N, K = (W.shape[0] if perm_out is None else len(perm_out)), W.shape[1]
    dev, g = W.device, cal.g_eff
    out = FoldedLinearCw(
        N=N,
        Wq=torch.empty(B.rptq_weight_bytes(N, cal.k_padded), dtype=torch.uint8, device=dev),
        sW=torch.empty((N, g), dtype=torch.float32, device=dev),
        zW=torch.empty((N, g), dtype=torch.int32, device=dev),
        wsum=torch.empty((N, g), dtype=torch.int32, device=dev),
        scale_tab=torch.empty(B.rptq_cw_scale_bytes(N, g) // 4, dtype=torch.float32, device=dev),
        cross_tab=torch.empty(B.rptq_cw_cross_bytes(N, g) // 4, dtype=torch.float32, device=dev),
        colterm=torch.empty(N, dtype=torch.float32, device=dev))
    B.rptq_fold_reorder_cw(cal.perm, cal.cluster_off, cal.s, cal.z, W, N, K, perm_out, cal.perm_pad, out.Wq, out.sW,
                           out.zW, out.wsum, out.scale_tab, out.cross_tab, out.colterm)
    return out


def cluster_rowsums(cal: Calibration, codes, M, rowsums=None):
    import torch
    if rowsums is None:
        rowsums = torch.empty(max(4, B.rptq_cw_rowsum_bytes(M, cal.g_eff) // 4), dtype=torch.float32, device=codes.device)
    B.rptq_cluster_rowsums(codes, M, cal.bits, cal.cluster_off, cal.s, cal.z, rowsums)
    return rowsums


def cluster_gemm_cw(cal: Calibration, lin: FoldedLinearCw, codes, rowsums, M, y=None, dtype=None):
    import torch
    if y is None:
        y = torch.empty((M, lin.N), dtype=dtype or torch.bfloat16, device=codes.device)
    B.rptq_cluster_gemm_cw(codes, M, cal.bits, lin.Wq, lin.N, cal.cluster_off, lin.scale_tab, lin.cross_tab, lin.colterm,
                           rowsums, y)
    return y
