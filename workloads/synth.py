"""Synthetic OPT-shaped activations, LayerNorm parameters and weights.

The recipe follows the channel-range structure the paper motivates in its
introduction and in the section on the challenges of activation quantization:
a few channels whose value range is far wider than the rest, and per-channel
ranges that sit away from zero.  Only shapes and that structure are
reproduced; no model weights or text corpora are involved.

Per site (one quantized activation tensor and the linear layers that read it):

* per-channel scale ``s_c = exp(N(0,1))``; ``round(0.01*d)`` channels chosen
  without replacement get ``s_c *= 30``; then the per-channel offset
  ``m_c ~ N(0, std = 2*s_c)`` (boosted scale);
* ``x[t,c] = bf16(m_c + s_c*N(0,1))``; calibration batches and the test batch
  share ``(m_c, s_c)`` and differ in the noise draw;
* LayerNorm ``gamma = exp(N(0,0.3))``, ``beta ~ N(0,0.1)`` in fp32;
* weights ``W ~ N(0, std=0.02)`` fp32 ``[N,K]``, generated in blocks of 256
  rows, each block from its own seed, so any subset of rows can be
  regenerated without drawing the whole matrix.

Everything is drawn from ``numpy.random.Generator(PCG64(seed))`` in the fixed
order listed above.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 20230401
CAL_ROWS = 128          # tokens per calibration batch
W_BLOCK_ROWS = 256      # rows per independently seeded weight block
W_STD = 0.02


# --------------------------------------------------------------------------
# bf16 helpers (storage format only: round-to-nearest-even on the top 16 bits)
# --------------------------------------------------------------------------
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 bf16 bit patterns (round to nearest even)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> the fp32 values they denote (exact)."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 array -> fp32 array holding bf16-representable values."""
    return bits_to_f32(bf16_bits(x))


# --------------------------------------------------------------------------
# configuration table (the five workloads)
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class SiteSpec:
    name: str
    d: int                      # channels of the quantized activation
    g: int                      # clusters
    gemms: Tuple[Tuple[str, int], ...]   # (name, N) linear layers reading it
    layernorm: bool = True      # False: ReLU site fed by a previous GEMM


@dataclass(frozen=True)
class LayerConfig:
    index: int
    name: str
    M: int
    bits: int
    n_cal: int
    sites: Tuple[SiteSpec, ...]


CONFIGS: Tuple[LayerConfig, ...] = (
    LayerConfig(0, "opt-125m linear W4A8", 128, 8, 4,
                (SiteSpec("ln", 768, 8, (("fc", 3072),)),)),
    LayerConfig(1, "opt-1.3b layer W4A4", 2048, 4, 16,
                (SiteSpec("ln_attn", 2048, 16, (("qkv", 6144),)),
                 SiteSpec("ln_ffn", 2048, 16, (("fc1", 8192),)))),
    LayerConfig(2, "opt-13b ffn W4A4", 4096, 4, 16,
                (SiteSpec("ln_ffn", 5120, 32, (("fc1", 20480),)),
                 SiteSpec("relu_fc2", 20480, 32, (("fc2", 5120),), layernorm=False))),
    LayerConfig(3, "opt-175b prefill W4A3", 8192, 3, 16,
                (SiteSpec("ln_attn", 12288, 32, (("qkv", 36864),)),
                 SiteSpec("ln_ffn", 12288, 32, (("fc1", 49152),)))),
    LayerConfig(4, "opt-175b decode W4A3", 16, 3, 16,
                (SiteSpec("ln_ffn", 12288, 32, (("fc1", 49152),)),)),
)


def site_seed(config_index: int, site_index: int) -> int:
    return BASE_SEED + 1000 * (config_index + 1) + site_index


# --------------------------------------------------------------------------
# generators
# --------------------------------------------------------------------------
@dataclass
class Site:
    d: int
    m_c: np.ndarray
    s_c: np.ndarray
    gamma: np.ndarray           # fp32 [d]
    beta: np.ndarray            # fp32 [d]
    cal: List[np.ndarray]       # bf16-representable fp32 [CAL_ROWS, d] each
    x: np.ndarray               # bf16-representable fp32 [M, d]
    seed: int = 0
    extra: dict = field(default_factory=dict)


def _channel_model(rng: np.random.Generator, d: int):
    s_c = np.exp(rng.normal(0.0, 1.0, d))
    n_out = int(round(0.01 * d))
    if n_out > 0:
        idx = rng.choice(d, size=n_out, replace=False)
        s_c[idx] *= 30.0
    m_c = rng.normal(0.0, 1.0, d) * (2.0 * s_c)
    return m_c, s_c


def _draw_rows(rng, m_c, s_c, rows: int) -> np.ndarray:
    d = m_c.shape[0]
    out = np.empty((rows, d), dtype=np.float32)
    step = max(1, (1 << 22) // d)
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        z = rng.standard_normal((r1 - r0, d))
        out[r0:r1] = (m_c + s_c * z).astype(np.float32)
    return round_to_bf16(out)


def make_site(seed: int, d: int, M: int, n_cal: int, cal_rows: int = CAL_ROWS) -> Site:
    """One LayerNorm site: channel model, gamma/beta, calibration batches, test batch."""
    rng = np.random.Generator(np.random.PCG64(seed))
    m_c, s_c = _channel_model(rng, d)
    gamma = np.exp(rng.normal(0.0, 0.3, d)).astype(np.float32)
    beta = rng.normal(0.0, 0.1, d).astype(np.float32)
    cal = [_draw_rows(rng, m_c, s_c, cal_rows) for _ in range(n_cal)]
    x = _draw_rows(rng, m_c, s_c, M)
    return Site(d, m_c, s_c, gamma, beta, cal, x, seed)


def extra_batch(site: Site, k: int, rows: int) -> np.ndarray:
    """A further batch of `rows` tokens from the site's channel model (noise stream k >= 1)."""
    rng = np.random.Generator(np.random.PCG64([site.seed, 7919, k]))
    return _draw_rows(rng, site.m_c, site.s_c, rows)


def weight_rows(seed: int, N: int, K: int, rows: np.ndarray) -> np.ndarray:
    """Selected rows of the seeded weight matrix W[N,K] (fp32), any order."""
    rows = np.asarray(rows, dtype=np.int64)
    out = np.empty((rows.shape[0], K), dtype=np.float32)
    blocks = rows // W_BLOCK_ROWS
    for b in np.unique(blocks):
        r0 = int(b) * W_BLOCK_ROWS
        nb = min(W_BLOCK_ROWS, N - r0)
        rng = np.random.Generator(np.random.PCG64([seed, int(b)]))
        blk = (rng.standard_normal((nb, K), dtype=np.float32) * np.float32(W_STD))
        sel = np.nonzero(blocks == b)[0]
        out[sel] = blk[rows[sel] - r0]
    return out


def weight_matrix(seed: int, N: int, K: int) -> np.ndarray:
    """The whole seeded weight matrix W[N,K] (fp32)."""
    out = np.empty((N, K), dtype=np.float32)
    for r0 in range(0, N, W_BLOCK_ROWS):
        nb = min(W_BLOCK_ROWS, N - r0)
        rng = np.random.Generator(np.random.PCG64([seed, r0 // W_BLOCK_ROWS]))
        out[r0:r0 + nb] = rng.standard_normal((nb, K), dtype=np.float32) * np.float32(W_STD)
    return out


def tiny_site(seed: int, d: int, M: int, n_cal: int = 2, cal_rows: int = 16) -> Site:
    """Small site with the same structure, for element-by-element checks."""
    return make_site(seed, d, M, n_cal, cal_rows)
