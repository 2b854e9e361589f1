"""ctypes binding of librptq.so: one Python function per C entry point, same names.

Arguments are torch tensors (device memory) or numpy arrays / python sequences (host
tables); every function only checks dtypes, extracts pointers and calls the library.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

DTYPE_BF16 = 0
DTYPE_F32 = 1

EXPORTED_SYMBOLS = (
    "rptq_padded_k", "rptq_codes_bytes", "rptq_weight_bytes", "rptq_calibrate_workspace_bytes",
    "rptq_calibrate", "rptq_fold_reorder", "rptq_ln_quant", "rptq_ln_quant_scatter",
    "rptq_ln_quant_scatter_workspace_bytes", "rptq_cluster_gemm",
    "rptq_cluster_gemm_quant", "rptq_cluster_gemm_quant_workspace_bytes", "rptq_cluster_gemm_quant_static",
    "rptq_cluster_gemm_partials", "rptq_unpack_codes", "rptq_unpack_weights", "rptq_channel_minmax",
    "rptq_cw_scale_bytes", "rptq_cw_cross_bytes", "rptq_cw_rowsum_bytes", "rptq_fold_reorder_cw", "rptq_cluster_rowsums",
    "rptq_cluster_gemm_cw", "rptq_cluster_gemm_partials_cw",
    "rptq_cluster_channels", "rptq_cluster_heads", "rptq_kv_table_bytes", "rptq_kv_tables", "rptq_kv_quant",
    "rptq_kv_dequant", "rptq_dequant_codes", "rptq_dequant_weights", "rptq_gemm_bf16", "rptq_device_info", "rptq_strerror", "rptq_last_hip_error", "rptq_version",
)

_LIB = None


class RptqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = "%s failed: status %d" % (where, status)
        try:
            msg += " (%s)" % rptq_strerror(status)
            if status == -8:
                msg += " hip error %d" % load_library().rptq_last_hip_error()
        except Exception:
            pass
        super().__init__(msg)


def library_path() -> str:
    if os.environ.get("RPTQ_LIBRARY"):          # an alternative build of the same library
        return os.environ["RPTQ_LIBRARY"]
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "librptq.so")


def load_library():
    """Loads the built library; raises if it has not been built (no fallback exists)."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError("librptq.so is not built (%s): run `python -m paper_2304_01089_amd.build`" % path)
    lib = C.CDLL(path)
    vp, i32, i64, u64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float, C.c_size_t
    sig = {
        "rptq_padded_k": (i32, [vp, i32, vp]),
        "rptq_codes_bytes": (sz, [i64, i32, i32]),
        "rptq_weight_bytes": (sz, [i32, i32]),
        "rptq_calibrate_workspace_bytes": (sz, [i32]),
        "rptq_calibrate": (i32, [vp, vp, i32, i32, vp, vp, f32, i32, i32, i32, u64, i32,
                                 vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]),
        "rptq_fold_reorder": (i32, [vp, vp, i32, vp, vp, i32, vp, vp, vp, i32, i32, i32, i32, vp,
                                    vp, vp, vp, vp, vp, vp, vp, vp, vp]),
        "rptq_ln_quant": (i32, [vp, i64, i32, vp, vp, f32, i32, vp, vp, i32, vp, vp, vp, i32, vp, vp, vp, vp]),
        "rptq_ln_quant_scatter": (i32, [vp, i64, i32, vp, vp, f32, i32, vp, vp, i32, vp, vp, i32, vp, vp, sz, vp]),
        "rptq_ln_quant_scatter_workspace_bytes": (sz, [i64, i32, i32]),
        "rptq_dequant_codes": (i32, [vp, i64, i32, vp, i32, vp, vp, vp, vp]),
        "rptq_dequant_weights": (i32, [vp, i32, vp, i32, vp, vp, vp, vp]),
        "rptq_gemm_bf16": (i32, [vp, vp, i64, i32, i32, vp, i32, vp]),
        "rptq_cluster_gemm": (i32, [vp, i64, i32, vp, i32, vp, i32, vp, vp, vp, vp, vp, vp, i32, vp]),
        "rptq_cluster_gemm_quant": (i32, [vp, i64, i32, vp, i32, vp, i32, vp, vp, vp, vp, vp, i32,
                                          vp, i32, vp, vp, vp, i32, vp, vp, vp, sz, vp]),
        "rptq_cluster_gemm_quant_static": (i32, [vp, i64, i32, vp, i32, vp, i32, vp, vp, vp, vp, vp, i32,
                                                 vp, i32, vp, vp, vp, i32, vp, vp, vp]),
        "rptq_cluster_gemm_quant_workspace_bytes": (sz, [i64, i32]),
        "rptq_cluster_gemm_partials": (i32, [vp, i64, i32, vp, i32, vp, i32, vp, vp, vp, vp, vp, vp]),
        "rptq_unpack_codes": (i32, [vp, i64, vp, i32, i32, vp, vp]),
        "rptq_unpack_weights": (i32, [vp, i32, vp, i32, vp, vp]),
        "rptq_channel_minmax": (i32, [vp, vp, i32, i32, vp, vp, f32, i32, vp, vp, vp, sz, vp]),
        "rptq_cluster_channels": (i32, [vp, vp, i32, i32, i32, u64, i32, vp, vp, vp, vp, vp, vp, vp]),
        "rptq_cw_scale_bytes": (sz, [i32, i32]),
        "rptq_cw_cross_bytes": (sz, [i32, i32]),
        "rptq_cw_rowsum_bytes": (sz, [i64, i32]),
        "rptq_fold_reorder_cw": (i32, [vp, vp, i32, vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]),
        "rptq_cluster_rowsums": (i32, [vp, i64, i32, vp, i32, vp, vp, vp, vp]),
        "rptq_cluster_gemm_cw": (i32, [vp, i64, i32, vp, i32, vp, i32, vp, vp, vp, vp, vp, i32, vp]),
        "rptq_cluster_gemm_partials_cw": (i32, [vp, i64, i32, vp, i32, vp, i32, vp, vp, vp, vp, vp, vp]),
        "rptq_cluster_heads": (i32, [vp, vp, i32, i32, i32, i32, i32, u64, i32, vp, vp, vp, vp, vp, vp, vp]),
        "rptq_kv_table_bytes": (sz, [i32]),
        "rptq_kv_tables": (i32, [vp, vp, vp, vp, vp, i32, i32, i32, vp, vp]),
        "rptq_kv_quant": (i32, [vp, i64, i32, vp, i32, vp, vp]),
        "rptq_kv_dequant": (i32, [vp, i64, i32, vp, i32, vp, vp]),
        "rptq_device_info": (i32, [vp, vp, vp, vp]),
        "rptq_strerror": (C.c_char_p, [i32]),
        "rptq_last_hip_error": (i32, []),
        "rptq_version": (C.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _LIB = lib
    return lib


# --------------------------------------------------------------------------------------
# marshalling helpers
# --------------------------------------------------------------------------------------
def _dev(t, dtype=None, allow_none=False):
    """Device pointer of a torch tensor (None -> NULL)."""
    if t is None:
        if allow_none:
            return None
        raise ValueError("missing device tensor")
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError("expected dtype %s, got %s" % (dtype, t.dtype))
    return C.c_void_p(t.data_ptr())


def _host(a, dtype):
    arr = np.ascontiguousarray(a, dtype=dtype)
    return arr, arr.ctypes.data_as(C.c_void_p)


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(status: int, where: str):
    if status != 0:
        raise RptqError(status, where)


# --------------------------------------------------------------------------------------
# entry points
# --------------------------------------------------------------------------------------
def rptq_strerror(status: int) -> str:
    return load_library().rptq_strerror(int(status)).decode()


def rptq_version() -> str:
    return load_library().rptq_version().decode()


def rptq_device_info() -> dict:
    vals = [C.c_int32(0) for _ in range(4)]
    _check(load_library().rptq_device_info(*[C.byref(v) for v in vals]), "rptq_device_info")
    return dict(compute_units=vals[0].value, clock_khz=vals[1].value, memory_clock_khz=vals[2].value,
                memory_bus_bits=vals[3].value)


def rptq_padded_k(cluster_off) -> int:
    off, p = _host(cluster_off, np.int32)
    out = C.c_int32(0)
    _check(load_library().rptq_padded_k(p, len(off) - 1, C.byref(out)), "rptq_padded_k")
    return out.value


def rptq_codes_bytes(M: int, k_padded: int, bits: int) -> int:
    return load_library().rptq_codes_bytes(M, k_padded, bits)


def rptq_weight_bytes(N: int, k_padded: int) -> int:
    return load_library().rptq_weight_bytes(N, k_padded)


def rptq_calibrate_workspace_bytes(d: int) -> int:
    return load_library().rptq_calibrate_workspace_bytes(d)


def rptq_cluster_channels(ch_min, ch_max, g: int, bits: int, seed: int = 0, max_iter: int = 100):
    """Host-only K-Means + reorder index + parameters.  Returns a dict of numpy arrays."""
    cmin, pmin = _host(ch_min, np.float32)
    cmax, pmax = _host(ch_max, np.float32)
    d = cmin.shape[0]
    assign = np.empty(d, np.int32)
    perm = np.empty(d, np.int32)
    off = np.zeros(g + 1, np.int32)
    s = np.zeros(g, np.float32)
    inv_s = np.zeros(g, np.float32)
    z = np.zeros(g, np.int32)
    g_eff = C.c_int32(0)
    st = load_library().rptq_cluster_channels(
        pmin, pmax, d, g, bits, seed, max_iter, assign.ctypes.data_as(C.c_void_p), perm.ctypes.data_as(C.c_void_p),
        off.ctypes.data_as(C.c_void_p), s.ctypes.data_as(C.c_void_p), inv_s.ctypes.data_as(C.c_void_p),
        z.ctypes.data_as(C.c_void_p), C.byref(g_eff))
    _check(st, "rptq_cluster_channels")
    ge = g_eff.value
    return dict(ch_min=cmin, ch_max=cmax, assign=assign, perm=perm, cluster_off=off[:ge + 1].copy(),
                s=s[:ge].copy(), inv_s=inv_s[:ge].copy(), z=z[:ge].copy(), g_eff=ge)


def _batches(x_batches):
    import torch
    ptrs = (C.c_void_p * len(x_batches))()
    rows = (C.c_int64 * len(x_batches))()
    d = None
    for i, xb in enumerate(x_batches):
        if xb.dtype != torch.bfloat16 or xb.dim() != 2:
            raise ValueError("calibration batches must be bf16 [rows, d]")
        ptrs[i] = _dev(xb).value
        rows[i] = xb.shape[0]
        d = xb.shape[1] if d is None else d
        if xb.shape[1] != d:
            raise ValueError("calibration batches disagree on d")
    return ptrs, rows, d


def rptq_channel_minmax(x_batches, gamma, beta, eps: float, relu: bool, ch_min_dev, ch_max_dev, workspace,
                        stream=None):
    import torch
    ptrs, rows, d = _batches(x_batches)
    st = load_library().rptq_channel_minmax(
        ptrs, rows, len(x_batches), d, _dev(gamma, torch.float32, True), _dev(beta, torch.float32, True),
        float(eps), int(bool(relu)), _dev(ch_min_dev, torch.float32), _dev(ch_max_dev, torch.float32),
        _dev(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "rptq_channel_minmax")


def rptq_calibrate(x_batches, gamma, beta, eps: float, relu: bool, g: int, bits: int, seed: int = 0,
                   max_iter: int = 100, workspace=None, stream=None):
    """Sec. 4.1 calibration.  Returns a dict of host numpy arrays (see rptq.h)."""
    import torch
    ptrs, rows, d = _batches(x_batches)
    if workspace is None:
        workspace = torch.empty(rptq_calibrate_workspace_bytes(d), dtype=torch.uint8, device=x_batches[0].device)
    ch_min = np.empty(d, np.float32)
    ch_max = np.empty(d, np.float32)
    assign = np.empty(d, np.int32)
    perm = np.empty(d, np.int32)
    off = np.zeros(g + 1, np.int32)
    s = np.zeros(g, np.float32)
    inv_s = np.zeros(g, np.float32)
    z = np.zeros(g, np.int32)
    g_eff = C.c_int32(0)
    vp = C.c_void_p
    st = load_library().rptq_calibrate(
        ptrs, rows, len(x_batches), d, _dev(gamma, torch.float32, True), _dev(beta, torch.float32, True),
        float(eps), int(bool(relu)), g, bits, seed, max_iter,
        ch_min.ctypes.data_as(vp), ch_max.ctypes.data_as(vp), assign.ctypes.data_as(vp), perm.ctypes.data_as(vp),
        off.ctypes.data_as(vp), s.ctypes.data_as(vp), inv_s.ctypes.data_as(vp), z.ctypes.data_as(vp),
        C.byref(g_eff), _dev(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "rptq_calibrate")
    ge = g_eff.value
    return dict(ch_min=ch_min, ch_max=ch_max, assign=assign, perm=perm, cluster_off=off[:ge + 1].copy(),
                s=s[:ge].copy(), inv_s=inv_s[:ge].copy(), z=z[:ge].copy(), g_eff=ge)


def rptq_fold_reorder(gamma, beta, d: int, perm_in, cluster_off, sX, zX, W, N: int, K: int,
                      perm_out, perm_pad, gamma_pad, beta_pad, Wq_packed, sW, zW, wsum, colterm, stream=None):
    """perm_in / perm_out are host index arrays (numpy); W, the outputs and gamma/beta are device tensors."""
    import torch
    off, poff = _host(cluster_off, np.int32)
    g = len(off) - 1
    ph, pph = _host(perm_in, np.int32)
    sx, psx = _host(sX if sX is not None else np.ones(g), np.float32)
    zx, pzx = _host(zX if zX is not None else np.zeros(g), np.int32)
    po, ppo = (None, None) if perm_out is None else _host(perm_out, np.int32)
    w_dtype, w_rows = DTYPE_BF16, 0
    if W is not None:
        if W.dtype == torch.float32:
            w_dtype = DTYPE_F32
        elif W.dtype != torch.bfloat16:
            raise ValueError("W must be bf16 or fp32")
        if W.dim() != 2 or W.shape[1] != K:
            raise ValueError("W must be [rows, K]")
        w_rows = W.shape[0]
        if po is not None and po.shape[0] != N:
            raise ValueError("perm_out must have N entries")
    st = load_library().rptq_fold_reorder(
        _dev(gamma, torch.float32, True), _dev(beta, torch.float32, True), d,
        pph, poff, g, psx, pzx,
        _dev(W, None, True), w_dtype, w_rows, N, K, ppo,
        _dev(perm_pad, torch.int32), _dev(gamma_pad, torch.float32, True), _dev(beta_pad, torch.float32, True),
        _dev(Wq_packed, None, True), _dev(sW, torch.float32, True), _dev(zW, torch.int32, True),
        _dev(wsum, torch.int32, True), _dev(colterm, torch.float32, True), _stream(stream))
    _check(st, "rptq_fold_reorder")


def rptq_ln_quant(x, M: int, d: int, gamma_pad, beta_pad, eps: float, relu: bool, perm_pad, cluster_off,
                  s, inv_s, z, bits: int, codes_packed, xsum=None, rowterm=None, stream=None):
    import torch
    off, poff = _host(cluster_off, np.int32)
    sa, ps = _host(s, np.float32)
    ia, pi = _host(inv_s, np.float32)
    za, pz = _host(z, np.int32)
    st = load_library().rptq_ln_quant(
        _dev(x, torch.bfloat16), M, d, _dev(gamma_pad, torch.float32, True), _dev(beta_pad, torch.float32, True),
        float(eps), int(bool(relu)), _dev(perm_pad, torch.int32), poff, len(off) - 1, ps, pi, pz, bits,
        _dev(codes_packed), _dev(xsum, torch.int32, True), _dev(rowterm, torch.float32, True), _stream(stream))
    _check(st, "rptq_ln_quant")


def rptq_ln_quant_scatter_workspace_bytes(M: int, d: int, k_padded: int) -> int:
    return int(load_library().rptq_ln_quant_scatter_workspace_bytes(M, d, k_padded))


def rptq_ln_quant_scatter(x, M: int, d: int, gamma, beta, eps: float, relu: bool, perm_pad, cluster_off, inv_s, z,
                          bits: int, codes_packed, workspace, stream=None):
    import torch
    off, poff = _host(cluster_off, np.int32)
    ia, pi = _host(inv_s, np.float32)
    za, pz = _host(z, np.int32)
    st = load_library().rptq_ln_quant_scatter(
        _dev(x, torch.bfloat16), M, d, _dev(gamma, torch.float32, True), _dev(beta, torch.float32, True), float(eps),
        int(bool(relu)), _dev(perm_pad, torch.int32), poff, len(off) - 1, pi, pz, bits, _dev(codes_packed),
        _dev(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "rptq_ln_quant_scatter")


def rptq_dequant_codes(codes_packed, M: int, bits: int, cluster_off, sX, zX, x_hat, stream=None):
    import torch
    off, poff = _host(cluster_off, np.int32)
    sx, psx = _host(sX, np.float32)
    zx, pzx = _host(zX, np.int32)
    st = load_library().rptq_dequant_codes(_dev(codes_packed), M, bits, poff, len(off) - 1, psx, pzx,
                                           _dev(x_hat, torch.bfloat16), _stream(stream))
    _check(st, "rptq_dequant_codes")


def rptq_dequant_weights(Wq_packed, N: int, cluster_off, sW, zW, w_hat, stream=None):
    import torch
    off, poff = _host(cluster_off, np.int32)
    st = load_library().rptq_dequant_weights(_dev(Wq_packed), N, poff, len(off) - 1, _dev(sW, torch.float32),
                                             _dev(zW, torch.int32), _dev(w_hat, torch.bfloat16), _stream(stream))
    _check(st, "rptq_dequant_weights")


def rptq_gemm_bf16(x_hat, w_hat, M: int, N: int, K: int, y, stream=None):
    import torch
    if y.dtype == torch.float32:
        y_dtype = DTYPE_F32
    elif y.dtype == torch.bfloat16:
        y_dtype = DTYPE_BF16
    else:
        raise ValueError("y must be bf16 or fp32")
    st = load_library().rptq_gemm_bf16(_dev(x_hat, torch.bfloat16), _dev(w_hat, torch.bfloat16), M, N, K, _dev(y), y_dtype,
                                       _stream(stream))
    _check(st, "rptq_gemm_bf16")


def rptq_cluster_gemm(codes_packed, M: int, bits: int, Wq_packed, N: int, cluster_off, sX, sW, zW, colterm,
                      rowterm, y, stream=None):
    import torch
    off, poff = _host(cluster_off, np.int32)
    sx, psx = _host(sX, np.float32)
    if y.dtype == torch.float32:
        y_dtype = DTYPE_F32
    elif y.dtype == torch.bfloat16:
        y_dtype = DTYPE_BF16
    else:
        raise ValueError("y must be bf16 or fp32")
    st = load_library().rptq_cluster_gemm(
        _dev(codes_packed), M, bits, _dev(Wq_packed), N, poff, len(off) - 1, psx,
        _dev(sW, torch.float32), _dev(zW, torch.int32), _dev(colterm, torch.float32),
        _dev(rowterm, torch.float32), _dev(y), y_dtype, _stream(stream))
    _check(st, "rptq_cluster_gemm")


def rptq_cluster_gemm_quant_workspace_bytes(M: int, N: int) -> int:
    return int(load_library().rptq_cluster_gemm_quant_workspace_bytes(M, N))


def rptq_cluster_gemm_quant(codes_packed, M: int, bits: int, Wq_packed, N: int, cluster_off, sX, sW, zW, colterm,
                            rowterm, relu: bool, next_cluster_off, next_s, next_inv_s, next_z, next_bits: int,
                            next_codes, next_rowterm, workspace, stream=None):
    import torch
    off, poff = _host(cluster_off, np.int32)
    sx, psx = _host(sX, np.float32)
    noff, pnoff = _host(next_cluster_off, np.int32)
    ns, pns = _host(next_s, np.float32)
    ni, pni = _host(next_inv_s, np.float32)
    nz, pnz = _host(next_z, np.int32)
    st = load_library().rptq_cluster_gemm_quant(
        _dev(codes_packed), M, bits, _dev(Wq_packed), N, poff, len(off) - 1, psx,
        _dev(sW, torch.float32), _dev(zW, torch.int32), _dev(colterm, torch.float32),
        _dev(rowterm, torch.float32), int(bool(relu)), pnoff, len(noff) - 1, pns, pni, pnz, next_bits,
        _dev(next_codes), _dev(next_rowterm, torch.float32), _dev(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream))
    _check(st, "rptq_cluster_gemm_quant")


def rptq_cluster_gemm_quant_static(codes_packed, M: int, bits: int, Wq_packed, N: int, cluster_off, sX, sW, zW,
                                   colterm, rowterm, relu: bool, next_cluster_off, next_s, next_inv_s, next_z,
                                   next_bits: int, next_codes, next_rowterm, stream=None):
    import torch
    off, poff = _host(cluster_off, np.int32)
    sx, psx = _host(sX, np.float32)
    noff, pnoff = _host(next_cluster_off, np.int32)
    ns, pns = _host(next_s, np.float32)
    ni, pni = _host(next_inv_s, np.float32)
    nz, pnz = _host(next_z, np.int32)
    st = load_library().rptq_cluster_gemm_quant_static(
        _dev(codes_packed), M, bits, _dev(Wq_packed), N, poff, len(off) - 1, psx,
        _dev(sW, torch.float32), _dev(zW, torch.int32), _dev(colterm, torch.float32),
        _dev(rowterm, torch.float32), int(bool(relu)), pnoff, len(noff) - 1, pns, pni, pnz, next_bits,
        _dev(next_codes), _dev(next_rowterm, torch.float32), _stream(stream))
    _check(st, "rptq_cluster_gemm_quant_static")


def rptq_cluster_gemm_partials(codes_packed, M: int, bits: int, Wq_packed, N: int, cluster_off, zX, zW, xsum,
                               wsum, yq, stream=None):
    import torch
    off, poff = _host(cluster_off, np.int32)
    zx, pzx = _host(zX, np.int32)
    st = load_library().rptq_cluster_gemm_partials(
        _dev(codes_packed), M, bits, _dev(Wq_packed), N, poff, len(off) - 1, pzx, _dev(zW, torch.int32),
        _dev(xsum, torch.int32), _dev(wsum, torch.int32), _dev(yq, torch.int32), _stream(stream))
    _check(st, "rptq_cluster_gemm_partials")


def rptq_cw_scale_bytes(N: int, g: int) -> int:
    return int(load_library().rptq_cw_scale_bytes(N, g))


def rptq_cw_cross_bytes(N: int, g: int) -> int:
    return int(load_library().rptq_cw_cross_bytes(N, g))


def rptq_cw_rowsum_bytes(M: int, g: int) -> int:
    return int(load_library().rptq_cw_rowsum_bytes(M, g))


def rptq_fold_reorder_cw(perm_in, cluster_off, sX, zX, W, N: int, K: int, perm_out, perm_pad, Wq_packed, sW, zW, wsum,
                         scale_tab, cross_tab, colterm, stream=None):
    import torch
    off, poff = _host(cluster_off, np.int32)
    ph, pph = _host(perm_in, np.int32)
    sx, psx = _host(sX, np.float32)
    zx, pzx = _host(zX, np.int32)
    po, ppo = (None, None) if perm_out is None else _host(perm_out, np.int32)
    if W.dtype == torch.float32:
        w_dtype = DTYPE_F32
    elif W.dtype == torch.bfloat16:
        w_dtype = DTYPE_BF16
    else:
        raise ValueError("W must be bf16 or fp32")
    if W.dim() != 2 or W.shape[1] != K:
        raise ValueError("W must be [rows, K]")
    st = load_library().rptq_fold_reorder_cw(
        pph, poff, len(off) - 1, psx, pzx, _dev(W), w_dtype, W.shape[0], N, K, ppo, _dev(perm_pad, torch.int32),
        _dev(Wq_packed), _dev(sW, torch.float32), _dev(zW, torch.int32), _dev(wsum, torch.int32),
        _dev(scale_tab, torch.float32), _dev(cross_tab, torch.float32), _dev(colterm, torch.float32), _stream(stream))
    _check(st, "rptq_fold_reorder_cw")


def rptq_cluster_rowsums(codes_packed, M: int, bits: int, cluster_off, sX, zX, rowsums, stream=None):
    import torch
    off, poff = _host(cluster_off, np.int32)
    sx, psx = _host(sX, np.float32)
    zx, pzx = _host(zX, np.int32)
    st = load_library().rptq_cluster_rowsums(_dev(codes_packed), M, bits, poff, len(off) - 1, psx, pzx,
                                             _dev(rowsums, torch.float32), _stream(stream))
    _check(st, "rptq_cluster_rowsums")


def rptq_cluster_gemm_cw(codes_packed, M: int, bits: int, Wq_packed, N: int, cluster_off, scale_tab, cross_tab, colterm,
                         rowsums, y, stream=None):
    import torch
    off, poff = _host(cluster_off, np.int32)
    if y.dtype == torch.float32:
        y_dtype = DTYPE_F32
    elif y.dtype == torch.bfloat16:
        y_dtype = DTYPE_BF16
    else:
        raise ValueError("y must be bf16 or fp32")
    st = load_library().rptq_cluster_gemm_cw(
        _dev(codes_packed), M, bits, _dev(Wq_packed), N, poff, len(off) - 1, _dev(scale_tab, torch.float32),
        _dev(cross_tab, torch.float32), _dev(colterm, torch.float32), _dev(rowsums, torch.float32), _dev(y), y_dtype,
        _stream(stream))
    _check(st, "rptq_cluster_gemm_cw")


def rptq_cluster_gemm_partials_cw(codes_packed, M: int, bits: int, Wq_packed, N: int, cluster_off, zX, zW, xsum, wsum,
                                  yq, stream=None):
    import torch
    off, poff = _host(cluster_off, np.int32)
    zx, pzx = _host(zX, np.int32)
    st = load_library().rptq_cluster_gemm_partials_cw(
        _dev(codes_packed), M, bits, _dev(Wq_packed), N, poff, len(off) - 1, pzx, _dev(zW, torch.int32),
        _dev(xsum, torch.int32), _dev(wsum, torch.int32), _dev(yq, torch.int32), _stream(stream))
    _check(st, "rptq_cluster_gemm_partials_cw")


def rptq_cluster_heads(ch_min, ch_max, n_heads: int, g: int, bits: int, seed: int = 0, max_iter: int = 100):
    """Host-only per-head clustering.  ch_min / ch_max: lists of one (a tensor alone) or two (queries, keys)
    fp32 arrays [d].  Returns a dict of numpy arrays (see rptq.h)."""
    mins = [np.ascontiguousarray(a, dtype=np.float32) for a in ch_min]
    maxs = [np.ascontiguousarray(a, dtype=np.float32) for a in ch_max]
    nt, d = len(mins), mins[0].shape[0]
    pmin = (C.c_void_p * nt)(*[a.ctypes.data for a in mins])
    pmax = (C.c_void_p * nt)(*[a.ctypes.data for a in maxs])
    assign = np.empty(d, np.int32)
    perm = np.empty(d, np.int32)
    off = np.zeros((n_heads, g + 1), np.int32)
    s = np.zeros((nt, n_heads, g), np.float32)
    inv_s = np.zeros((nt, n_heads, g), np.float32)
    z = np.zeros((nt, n_heads, g), np.int32)
    g_eff = np.zeros(n_heads, np.int32)
    vp = C.c_void_p
    st = load_library().rptq_cluster_heads(
        pmin, pmax, nt, d, n_heads, g, bits, seed, max_iter, assign.ctypes.data_as(vp), perm.ctypes.data_as(vp),
        off.ctypes.data_as(vp), s.ctypes.data_as(vp), inv_s.ctypes.data_as(vp), z.ctypes.data_as(vp),
        g_eff.ctypes.data_as(vp))
    _check(st, "rptq_cluster_heads")
    return dict(assign=assign, perm=perm, cluster_off=off, s=s, inv_s=inv_s, z=z, g_eff=g_eff)


def rptq_kv_table_bytes(d: int) -> int:
    return int(load_library().rptq_kv_table_bytes(d))


def rptq_kv_tables(perm, cluster_off, s, inv_s, z, d: int, n_heads: int, g: int, table, stream=None):
    pa, pp = _host(perm, np.int32)
    oa, po = _host(cluster_off, np.int32)
    sa, ps = _host(s, np.float32)
    ia, pi = _host(inv_s, np.float32)
    za, pz = _host(z, np.int32)
    st = load_library().rptq_kv_tables(pp, po, ps, pi, pz, d, n_heads, g, _dev(table), _stream(stream))
    _check(st, "rptq_kv_tables")


def rptq_kv_quant(x, T: int, d: int, table, bits: int, codes, stream=None):
    import torch
    st = load_library().rptq_kv_quant(_dev(x, torch.bfloat16), T, d, _dev(table), bits, _dev(codes), _stream(stream))
    _check(st, "rptq_kv_quant")


def rptq_kv_dequant(codes, T: int, d: int, table, bits: int, out, stream=None):
    import torch
    st = load_library().rptq_kv_dequant(_dev(codes), T, d, _dev(table), bits, _dev(out, torch.bfloat16), _stream(stream))
    _check(st, "rptq_kv_dequant")


def rptq_unpack_codes(codes_packed, rows: int, cluster_off, bits: int, out, stream=None):
    import torch
    off, poff = _host(cluster_off, np.int32)
    st = load_library().rptq_unpack_codes(_dev(codes_packed), rows, poff, len(off) - 1, bits,
                                          _dev(out, torch.int8), _stream(stream))
    _check(st, "rptq_unpack_codes")


def rptq_unpack_weights(Wq_packed, N: int, cluster_off, out, stream=None):
    import torch
    off, poff = _host(cluster_off, np.int32)
    st = load_library().rptq_unpack_weights(_dev(Wq_packed), N, poff, len(off) - 1, _dev(out, torch.int8),
                                            _stream(stream))
    _check(st, "rptq_unpack_weights")
