"""Pins for the oracle's quantizer (Eq. 1) and Min-Max rule (Eq. 2)."""
from fractions import Fraction

import numpy as np
import pytest

from conftest import read_golden
from oracle import rptq_oracle as o


def test_code_range_printed_for_four_bits():
    # The text under Eq. 1 prints the 4-bit range.
    assert o.code_range(4) == (-8, 7)
    assert o.code_range(3) == (-4, 3)
    assert o.code_range(8) == (-128, 127)


def test_eq2_worked_examples():
    for kind, xmin, xmax, s, z in [r for r in read_golden("eq2_examples.txt") if r[0] == "params"]:
        s32, inv32, zz = o.minmax_params(np.float32(xmin), np.float32(xmax), 4)
        assert float(s32) == float(s)
        assert int(zz) == int(z)
        assert float(inv32) == float(np.float32(1.0 / float(s)))


def test_eq1_worked_examples():
    for kind, x, s, z, code, xhat in [r for r in read_golden("eq2_examples.txt") if r[0] == "quant"]:
        inv = np.float32(1.0 / float(s))
        q = o.quantize(np.float32(x), inv, int(z), 4)
        assert int(q) == int(code), (x, s, z)
        assert float(o.dequantize(q, float(s), int(z))) == float(xhat)


def test_zero_point_not_bounded_by_code_range():
    # a range far from zero gives |z| beyond the code range (second worked example)
    _, _, z = o.minmax_params(np.float32(80), np.float32(100), 4)
    assert int(z) == -72


@pytest.mark.parametrize("k", [3, 4, 8])
def test_dequantization_error_bound(k):
    rng = np.random.default_rng(k)
    for _ in range(20):
        lo = np.float32(rng.normal(0, 10))
        hi = np.float32(lo + abs(rng.normal(0, 10)) + 0.1)
        s, inv, z = o.minmax_params(lo, hi, k)
        x = rng.uniform(lo, hi, 4000).astype(np.float32)
        q = o.quantize(x, inv, z, k)
        assert q.min() >= -(1 << (k - 1)) and q.max() <= (1 << (k - 1)) - 1
        xh = o.dequantize(q, s, z)
        err = np.abs(xh - x.astype(np.float64))
        s64 = float(s)
        unclamped = (np.rint(x.astype(np.float64) / s64) + int(z) >= -(1 << (k - 1))) & (
            np.rint(x.astype(np.float64) / s64) + int(z) <= (1 << (k - 1)) - 1)
        assert err[unclamped].max() <= 0.5 * s64 * (1 + 1e-3)   # fp32 product slack
        # rounding of z shifts the grid by at most half a step and the top code
        # is cut by the 2^k divisor: never worse than 2.5 steps inside the range
        assert err.max() <= 2.5 * s64 * (1 + 1e-5)
        # monotone in x
        order = np.argsort(x, kind="stable")
        assert (np.diff(q[order]) >= 0).all()


def test_against_exact_rational_quantizer():
    """Eq. 1 with true division in exact rationals; the fp32-reciprocal product may
    only differ where x/s sits on a rounding tie (never by more than one code)."""
    rng = np.random.default_rng(7)
    lo, hi = np.float32(-3.7), np.float32(11.2)
    k = 4
    s, inv, z = o.minmax_params(lo, hi, k)
    x = rng.uniform(-6, 14, 3000).astype(np.float32)
    q = o.quantize(x, inv, z, k)
    sf = Fraction(float(s))
    n_diff = 0
    for xi, qi in zip(x.tolist(), q.tolist()):
        r = Fraction(xi) / sf
        fl = r.numerator // r.denominator
        frac = r - fl
        rn = fl + (1 if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and fl % 2 == 1) else 0)
        ref = max(-8, min(7, rn + int(z)))
        n_diff += ref != qi
        assert abs(ref - qi) <= 1
    assert n_diff <= 2


def test_degenerate_group():
    s, inv, z = o.minmax_params(np.float32(0.0), np.float32(0.0), 4)
    assert float(s) == 1.0 and float(inv) == 1.0 and int(z) == 0
    s, inv, z = o.minmax_params(np.float32(2.5), np.float32(2.5), 4)
    assert float(s) == 1.0 and int(z) == -2          # round half to even
    assert int(o.quantize(np.float32(0.0), inv, 0, 4)) == 0


def test_saturation_far_outside_range():
    s, inv, z = o.minmax_params(np.float32(-1), np.float32(1), 3)
    q = o.quantize(np.array([-3e38, -1e9, 1e9, 3e38], dtype=np.float32), inv, z, 3)
    assert q.tolist() == [-4, -4, 3, 3]


@pytest.mark.parametrize("k,relu", [(3, True), (4, True), (4, False), (8, True)])
def test_bf16_rounding_then_quantizer_is_monotone(k, relu):
    """The parity test of the product that quantizes for the next site brackets a code between the
    oracle's codes of H - tol and H + tol.  That is only valid because rounding to bf16 (nearest
    even), ReLU and Eq. 1 with the reciprocal multiply are each non-decreasing: checked here on
    sorted inputs that include ties of both roundings, per cluster."""
    import workloads as w
    rng = np.random.default_rng(31 + k)
    g, per = 5, 4000
    s = np.exp(rng.normal(size=g)).astype(np.float32)
    inv_s = (1.0 / s.astype(np.float64)).astype(np.float32)
    z = rng.integers(-9, 10, size=g).astype(np.int32)
    off = np.arange(g + 1, dtype=np.int32) * per
    cols = []
    for i in range(g):
        qmax = 2 ** (k - 1)
        x = rng.uniform(-1.5 * qmax, 1.5 * qmax, size=per - 200) * s[i]
        ties = (np.arange(-100, 100) + 0.5) * s[i]                      # Eq. 1's rounding ties
        cols.append(np.sort(np.concatenate([x, ties])).astype(np.float64))
    H = np.concatenate(cols)[None, :]                                   # one row, clusters side by side
    h = w.round_to_bf16(H.astype(np.float32))
    codes, _, _ = o.ln_quant(h, None, None, 1e-5, relu, None, off, inv_s, z, k)
    codes = codes[0].astype(np.int64)
    for i in range(g):
        seg = codes[off[i]:off[i + 1]]
        assert (np.diff(seg) >= 0).all()
        assert seg.min() >= -(2 ** (k - 1)) and seg.max() <= 2 ** (k - 1) - 1
    hb = h[0].astype(np.float64)
    for i in range(g):
        assert (np.diff(hb[off[i]:off[i + 1]]) >= 0).all()
