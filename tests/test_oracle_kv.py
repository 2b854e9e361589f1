"""Pins for the attention-site oracle: per-head clustering with a shared query/key index
(Sec. 4.2, Sec. 5.1), key/value-cache codes and their de-quantization (Eq. 1 and the line
under it)."""
from fractions import Fraction

import numpy as np
import pytest

import workloads as w
from oracle import kv_cache as kv
from oracle import rptq_oracle as o


def _qk(seed, T=40, H=3, dh=16):
    rng = np.random.default_rng(seed)
    D = H * dh
    sc = np.exp(rng.normal(0, 1, D))
    q = w.round_to_bf16((rng.normal(0, 2 * sc) + sc * rng.standard_normal((T, D))).astype(np.float32))
    k = w.round_to_bf16((rng.normal(0, 2 * sc) + 0.5 * sc * rng.standard_normal((T, D))).astype(np.float32))
    return q, k, H, dh


def _minmax(x):
    return (x.min(axis=0) + np.float32(0)).astype(np.float32), (x.max(axis=0) + np.float32(0)).astype(np.float32)


def test_shared_query_key_index_is_per_head_kmeans_on_the_four_number_points():
    q, k, H, dh = _qk(1)
    qmin, qmax = _minmax(q)
    kmin, kmax = _minmax(k)
    g, bits, seed = 4, 4, 9
    hc = kv.cluster_heads([qmin, kmin], [qmax, kmax], H, g, bits, seed)
    assert sorted(hc.perm.tolist()) == list(range(H * dh))
    for h in range(H):
        sl = slice(h * dh, (h + 1) * dh)
        # the point of a channel is (Qmax, Qmin, Kmax, Kmin), as the paper lists it
        pts = np.stack([qmax[sl], qmin[sl], kmax[sl], kmin[sl]], axis=1)
        raw, _, _ = o.kmeans_points(pts, g, seed + h)
        lab, ge = o.canonical_labels(raw)
        perm, off = o.reorder_index(lab, ge)
        assert ge == hc.g_eff[h]
        assert np.array_equal(hc.assign[sl], lab)
        assert np.array_equal(hc.perm[sl], perm + h * dh)              # channels never leave their head
        assert np.array_equal(hc.cluster_off[h, :ge + 1], off)
        # each tensor has its own Eq. 2 pair per cluster, from its own extrema
        for t, (mn, mx) in enumerate(((qmin, qmax), (kmin, kmax))):
            s, inv, z, _, _ = o.cluster_params(mn[sl], mx[sl], perm, off, bits)
            assert np.array_equal(hc.s[t, h, :ge], s) and np.array_equal(hc.z[t, h, :ge], z)
    # the product over channels does not see a reordering both operands share (exact on integers)
    qi = np.rint(q * 4).astype(np.int64)
    ki = np.rint(k * 4).astype(np.int64)
    for h in range(H):
        sl = slice(h * dh, (h + 1) * dh)
        assert np.array_equal(qi[:, hc.perm[sl]] @ ki[:, hc.perm[sl]].T, qi[:, sl] @ ki[:, sl].T)


def test_single_tensor_heads_use_the_two_number_points():
    q, k, H, dh = _qk(2)
    vmin, vmax = _minmax(k)
    hc = kv.cluster_heads([vmin], [vmax], H, 4, 3, seed=5)
    for h in range(H):
        sl = slice(h * dh, (h + 1) * dh)
        raw, _, _ = o.kmeans(vmin[sl], vmax[sl], 4, 5 + h)
        lab, ge = o.canonical_labels(raw)
        assert np.array_equal(hc.assign[sl], lab) and ge == hc.g_eff[h]


@pytest.mark.parametrize("bits", [3, 4, 8])
def test_cache_codes_are_the_pinned_quantizer_head_by_head(bits):
    q, k, H, dh = _qk(3)
    qmin, qmax = _minmax(q)
    kmin, kmax = _minmax(k)
    hc = kv.cluster_heads([qmin, kmin], [qmax, kmax], H, 4, bits, seed=2)
    codes = kv.kv_quant(k, hc, 1, bits)
    for h in range(H):
        sl = slice(h * dh, (h + 1) * dh)
        ge = int(hc.g_eff[h])
        ref, _, _ = o.ln_quant(k[:, sl], None, None, 1e-5, False, hc.perm[sl] - h * dh, hc.cluster_off[h, :ge + 1],
                               hc.inv_s[1, h, :ge], hc.z[1, h, :ge], bits)
        assert np.array_equal(codes[:, sl], ref)
    lo, hi = o.code_range(bits)
    assert codes.min() >= lo and codes.max() <= hi


def _bf16_nearest_even(fr: Fraction) -> Fraction:
    """Nearest bf16 (8 significant bits) to a rational, ties to even, by exact arithmetic."""
    if fr == 0:
        return Fraction(0)
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = 0
    while a >= 256:
        a /= 2
        e += 1
    while a < 128:
        a *= 2
        e -= 1
    fl = a.numerator // a.denominator
    rem = a - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return sign * Fraction(fl) * (Fraction(2) ** e)


def test_reading_the_cache_back_exact_arithmetic_and_error_bound():
    q, k, H, dh = _qk(4, T=30)
    kmin, kmax = _minmax(k)
    bits = 4
    hc = kv.cluster_heads([kmin], [kmax], H, 4, bits, seed=1)
    codes = kv.kv_quant(k, hc, 0, bits)
    back = kv.kv_dequant(codes, hc, 0)
    s, _, z = kv.position_tables(hc, 0)
    rng = np.random.default_rng(0)
    for _ in range(300):
        t, j = int(rng.integers(0, codes.shape[0])), int(rng.integers(0, codes.shape[1]))
        exact = Fraction(float(s[j])) * (int(codes[t, j]) - int(z[j]))       # s (x_q - z), exactly
        f32 = Fraction(float(np.float32(float(exact))))                      # one rounding to fp32 (float() of a 46-bit product is exact)
        assert Fraction(float(back[t, j])) == _bf16_nearest_even(f32)
    # original channel order on request
    orig = kv.kv_dequant(codes, hc, 0, original_order=True)
    assert np.array_equal(orig[:, hc.perm], back)
    # round trip: within half a step (plus the bf16 rounding of the result) wherever Eq. 1 did not clamp
    lo, hi = o.code_range(bits)
    inner = (codes > lo) & (codes < hi)
    err = np.abs(back.astype(np.float64) - k[:, hc.perm].astype(np.float64))
    bound = 0.5 * s[None, :].astype(np.float64) * (1 + 2.0 ** -20) + np.abs(back) * 2.0 ** -8
    assert (err[inner] <= bound[inner]).all()
