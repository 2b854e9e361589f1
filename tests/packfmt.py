"""Numpy encoder/decoder of the packed layouts documented in include/rptq.h, written from
that text alone (shares nothing with the HIP sources or the oracle).  Used to feed the
GEMM kernels oracle-made codes and to decode what the quantization kernels wrote."""
import numpy as np

GROUP = 32
K_ALIGN = 256
N_ALIGN = 256


def padded_layout(cluster_off):
    off = np.asarray(cluster_off, dtype=np.int64)
    sizes = np.diff(off)
    padded = (sizes + GROUP - 1) // GROUP * GROUP
    pad_off = np.concatenate([[0], np.cumsum(padded)])
    k_p = int((pad_off[-1] + K_ALIGN - 1) // K_ALIGN * K_ALIGN)
    return pad_off, k_p


def to_padded(codes, cluster_off):
    """[rows, K] cluster order -> [rows, K_p] with zeros in pad positions."""
    pad_off, k_p = padded_layout(cluster_off)
    out = np.zeros((codes.shape[0], k_p), dtype=np.int64)
    for i in range(len(cluster_off) - 1):
        a, b = cluster_off[i], cluster_off[i + 1]
        out[:, pad_off[i]:pad_off[i] + (b - a)] = codes[:, a:b]
    return out


def from_padded(padded, cluster_off):
    pad_off, _ = padded_layout(cluster_off)
    parts = [padded[:, pad_off[i]:pad_off[i] + (cluster_off[i + 1] - cluster_off[i])]
             for i in range(len(cluster_off) - 1)]
    return np.concatenate(parts, axis=1)


def _pack4_groups(c):
    """[..., 8] codes -> [..., 4] bytes: byte b = c[b] << 4 | c[4+b] & 15."""
    c = c.astype(np.int64) & 15
    return ((c[..., 0:4] << 4) | c[..., 4:8]).astype(np.uint8)


def pack_codes(codes, cluster_off, bits):
    """Oracle codes [rows, K] -> packed bytes [rows, K_p*bits/8]."""
    return pack_groups(to_padded(codes, cluster_off), bits)


def pack_groups(p, bits):
    """Codes [rows, n] (n a multiple of 32, positions as given) -> the 32-code group formats."""
    p = np.asarray(p).astype(np.int64)
    rows, k_p = p.shape
    if bits == 8:
        return p.astype(np.int8).view(np.uint8).reshape(rows, k_p)
    if bits == 4:
        return _pack4_groups(p.reshape(rows, k_p // 8, 8)).reshape(rows, k_p // 2)
    f = (p & 7).reshape(rows, k_p // 32, 32)
    out = np.zeros((rows, k_p // 32, 12), dtype=np.int64)
    for b in range(4):
        out[..., 0 + b] = (f[..., b] << 5) | (f[..., 4 + b] << 2) | (f[..., 24 + b] >> 1)
        out[..., 4 + b] = (f[..., 8 + b] << 5) | (f[..., 12 + b] << 2) | (f[..., 28 + b] >> 1)
        out[..., 8 + b] = (f[..., 16 + b] << 5) | (f[..., 20 + b] << 2) | ((f[..., 28 + b] & 1) << 1) | (f[..., 24 + b] & 1)
    return out.astype(np.uint8).reshape(rows, k_p // 32 * 12)


def _sext(v, bits):
    v = v.astype(np.int64) & ((1 << bits) - 1)
    return np.where(v >= (1 << (bits - 1)), v - (1 << bits), v)


def unpack_codes(packed, cluster_off, bits):
    """Packed bytes -> (codes [rows, K] cluster order, pad codes [rows, n_pad])."""
    pad_off, k_p = padded_layout(cluster_off)
    p = unpack_groups(packed, k_p, bits)
    mask = np.ones(k_p, dtype=bool)
    for i in range(len(cluster_off) - 1):
        mask[pad_off[i]:pad_off[i] + (cluster_off[i + 1] - cluster_off[i])] = False
    return from_padded(p, cluster_off), p[:, mask]


def unpack_groups(packed, k_p, bits):
    """The 32-code group formats -> codes [rows, k_p]."""
    packed = np.asarray(packed, dtype=np.uint8)
    rows = packed.shape[0]
    if bits == 8:
        p = packed.view(np.int8).astype(np.int64).reshape(rows, k_p)
    elif bits == 4:
        by = packed.reshape(rows, k_p // 8, 4).astype(np.int64)
        p = np.concatenate([_sext(by >> 4, 4), _sext(by & 15, 4)], axis=2).reshape(rows, k_p)
    else:
        by = packed.reshape(rows, k_p // 32, 12).astype(np.int64)
        f = np.zeros((rows, k_p // 32, 32), dtype=np.int64)
        for b in range(4):
            f[..., b] = by[..., b] >> 5
            f[..., 4 + b] = (by[..., b] >> 2) & 7
            f[..., 8 + b] = by[..., 4 + b] >> 5
            f[..., 12 + b] = (by[..., 4 + b] >> 2) & 7
            f[..., 16 + b] = by[..., 8 + b] >> 5
            f[..., 20 + b] = (by[..., 8 + b] >> 2) & 7
            f[..., 24 + b] = ((by[..., b] & 3) << 1) | (by[..., 8 + b] & 1)
            f[..., 28 + b] = ((by[..., 4 + b] & 3) << 1) | ((by[..., 8 + b] >> 1) & 1)
        p = _sext(f, 3).reshape(rows, k_p)
    return p


def pack_weights(wq, cluster_off):
    """Oracle weight codes [N, K] cluster order -> packed fragment-major bytes."""
    p = to_padded(wq, cluster_off)
    N, k_p = p.shape
    n_p = (N + N_ALIGN - 1) // N_ALIGN * N_ALIGN
    full = np.zeros((n_p, k_p), dtype=np.int64)
    full[:N] = p
    # [rb, r, kb, sp, s2, h, v, 8 codes] -> [rb, kb, sp, h, r, s2, v, 4 bytes]   (slice s = 2 sp + s2)
    blk = full.reshape(n_p // 32, 32, k_p // 128, 2, 2, 2, 2, 8)
    by = _pack4_groups(blk)                                  # [rb, r, kb, sp, s2, h, v, 4]
    by = by.transpose(0, 2, 3, 5, 1, 4, 6, 7)                # [rb, kb, sp, h, r, s2, v, 4]
    return np.ascontiguousarray(by).reshape(-1)


def unpack_weights(packed, N, cluster_off):
    pad_off, k_p = padded_layout(cluster_off)
    n_p = (N + N_ALIGN - 1) // N_ALIGN * N_ALIGN
    by = np.asarray(packed, dtype=np.uint8).reshape(n_p // 32, k_p // 128, 2, 2, 32, 2, 2, 4).astype(np.int64)
    codes = np.concatenate([_sext(by >> 4, 4), _sext(by & 15, 4)], axis=7)     # [rb, kb, sp, h, r, s2, v, 8]
    full = codes.transpose(0, 4, 1, 2, 5, 3, 6, 7).reshape(n_p, k_p)
    return from_padded(full[:N], cluster_off), full[N:]
