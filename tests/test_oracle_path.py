"""Pins for the oracle's fused reorder, per-cluster quantization, weight
quantization and the two forms of the cluster-wise product."""
import numpy as np
import pytest

import workloads as w
from oracle import rptq_oracle as o


def _setup(seed=21, d=48, M=12, g=4, bits=4, N=10):
    s = w.tiny_site(seed, d, M, n_cal=3, cal_rows=24)
    cal = o.calibrate(s.cal, s.gamma, s.beta, 1e-5, False, g, bits, seed=seed)
    W = w.weight_matrix(seed + 1, N, d)
    return s, cal, W


@pytest.mark.parametrize("bits", [3, 4, 8])
def test_fused_reorder_equals_explicit_permute_then_quantize(bits):
    s, cal, _ = _setup(bits=bits)
    codes, xsum, fr = o.ln_quant(s.x, s.gamma, s.beta, 1e-5, False, cal.perm, cal.cluster_off,
                                 cal.inv_s, cal.z, bits)
    # explicit: LN in original order, physically permute, quantize cluster by cluster
    y, _ = o.layernorm_f32(s.x, s.gamma, s.beta, 1e-5)
    yt = y[:, cal.perm]
    for i in range(cal.g_eff):
        a, b = cal.cluster_off[i], cal.cluster_off[i + 1]
        ref = o.quantize(yt[:, a:b], cal.inv_s[i], cal.z[i], bits)
        assert np.array_equal(codes[:, a:b], ref)
        assert np.array_equal(xsum[:, i], ref.sum(axis=1))
    # fused: gamma/beta gathered, LN run on the reordered row
    gr, br = o.fold_layernorm(s.gamma, s.beta, cal.perm)
    yf, fr2 = o.layernorm_f32(s.x[:, cal.perm], gr, br, 1e-5)
    ok = ~(fr | fr2)
    sizes = np.diff(cal.cluster_off)
    cf = o.quantize(yf, np.repeat(cal.inv_s, sizes)[None], np.repeat(cal.z, sizes)[None], bits)
    assert ok.sum() >= ok.size - 1
    assert np.array_equal(cf[ok], codes[ok])


def test_one_cluster_is_per_tensor_and_c_clusters_is_per_channel():
    s, _, _ = _setup()
    bits = 4
    cmin, cmax = o.calibrate_minmax(s.cal, s.gamma, s.beta, 1e-5)
    y, _ = o.layernorm_f32(s.x, s.gamma, s.beta, 1e-5)
    # g = 1
    cal1 = o.calibrate(s.cal, s.gamma, s.beta, 1e-5, False, 1, bits)
    assert cal1.g_eff == 1 and np.array_equal(cal1.perm, np.arange(s.d))
    c1, _, _ = o.ln_quant(s.x, s.gamma, s.beta, 1e-5, False, cal1.perm, cal1.cluster_off, cal1.inv_s, cal1.z, bits)
    st, invt, zt = o.minmax_params(cmin.min(), cmax.max(), bits)
    assert np.array_equal(c1, o.quantize(y, invt, zt, bits))
    # g = C (distinct points): every channel its own cluster
    calC = o.calibrate(s.cal, s.gamma, s.beta, 1e-5, False, s.d, bits)
    assert calC.g_eff == s.d
    cC, _, _ = o.ln_quant(s.x, s.gamma, s.beta, 1e-5, False, calC.perm, calC.cluster_off, calC.inv_s, calC.z, bits)
    sc, invc, zc = o.minmax_params(cmin, cmax, bits)
    ref = o.quantize(y, invc[None], zc[None], bits)
    assert np.array_equal(cC, ref[:, calC.perm])


def test_calibration_outputs_are_a_partition():
    s, cal, _ = _setup(g=5)
    assert sorted(cal.perm.tolist()) == list(range(s.d))
    assert cal.cluster_off[0] == 0 and cal.cluster_off[-1] == s.d
    assert (np.diff(cal.cluster_off) > 0).all()
    assert cal.assign[0] == 0
    for i in range(cal.g_eff):
        mem = cal.perm[cal.cluster_off[i]:cal.cluster_off[i + 1]]
        assert (cal.assign[mem] == i).all() and (np.diff(mem) > 0).all()
    # calibration rows never clamp by more than the top-code cut of Eq. 2
    for xb in s.cal:
        codes, _, _ = o.ln_quant(xb, s.gamma, s.beta, 1e-5, False, cal.perm, cal.cluster_off, cal.inv_s, cal.z, 4)
        assert codes.min() >= -8 and codes.max() <= 7


def test_weight_quantization_per_output_channel():
    s, cal, W = _setup()
    wq, sW, invW, zW = o.quantize_weights(W, cal.perm)
    assert wq.min() >= -8 and wq.max() <= 7
    for r in range(W.shape[0]):                              # Eq. 2 / Eq. 1 row by row
        sr, invr, zr = o.minmax_params(W[r].min(), W[r].max(), 4)
        assert float(sr) == float(sW[r]) and int(zr) == int(zW[r])
        assert np.array_equal(wq[r], o.quantize(W[r][cal.perm], invr, zr, 4))
    # column reorder commutes with per-row quantization; row reorder permutes rows
    wq0, _, _, _ = o.quantize_weights(W, np.arange(s.d))
    assert np.array_equal(wq, wq0[:, cal.perm])
    po = np.random.default_rng(0).permutation(W.shape[0])
    wq2, sW2, _, zW2 = o.quantize_weights(W, cal.perm, po)
    assert np.array_equal(wq2, wq[po]) and np.array_equal(sW2, sW[po]) and np.array_equal(zW2, zW[po])
    # a row's extremes land on the extreme codes (within the 2^k divisor cut)
    assert (wq.min(axis=1) == -8).all() and (wq.max(axis=1) >= 6).all()


def _brute_force_gemm(xq, wq, off, sX, zX, sW, zW):
    g = len(off) - 1
    M, N = xq.shape[0], wq.shape[0]
    Yq = [[[0] * N for _ in range(M)] for _ in range(g)]
    Y = np.zeros((M, N))
    for t in range(M):
        for n in range(N):
            acc = 0.0
            for i in range(g):
                tot = 0
                for c in range(int(off[i]), int(off[i + 1])):
                    tot += (int(xq[t, c]) - int(zX[i])) * (int(wq[n, c]) - int(zW[n]))
                Yq[i][t][n] = tot
                acc += float(sX[i]) * float(sW[n]) * tot
            Y[t, n] = acc
    return np.array(Yq, dtype=np.int64), Y


@pytest.mark.parametrize("bits", [3, 4, 8])
def test_integer_form_against_brute_force_and_dequantized_form(bits):
    s, cal, W = _setup(bits=bits)
    codes, xsum, _ = o.ln_quant(s.x, s.gamma, s.beta, 1e-5, False, cal.perm, cal.cluster_off, cal.inv_s, cal.z, bits)
    wq, sW, _, zW = o.quantize_weights(W, cal.perm)
    P, Yq, Y = o.cluster_gemm_int(codes, wq, cal.cluster_off, cal.s, cal.z, sW, zW)
    Yq_ref, Y_ref = _brute_force_gemm(codes, wq, cal.cluster_off, cal.s, cal.z, sW, zW)
    assert np.array_equal(Yq, Yq_ref)
    scale = np.abs(Y_ref).max()
    assert np.abs(Y - Y_ref).max() <= 1e-12 * scale
    Y1 = o.cluster_gemm_dequant(codes, wq, cal.cluster_off, cal.s, cal.z, sW, zW)   # method 1
    assert np.abs(Y - Y1).max() <= 1e-12 * scale
    # raw products are the plain integer matrix product of each cluster's slice
    for i in range(cal.g_eff):
        a, b = cal.cluster_off[i], cal.cluster_off[i + 1]
        assert np.array_equal(P[i], codes[:, a:b].astype(np.int64) @ wq[:, a:b].astype(np.int64).T)


def test_product_invariant_to_order_inside_clusters_and_cluster_relabelling():
    s, cal, W = _setup(g=3)
    bits = 4
    codes, _, _ = o.ln_quant(s.x, s.gamma, s.beta, 1e-5, False, cal.perm, cal.cluster_off, cal.inv_s, cal.z, bits)
    wq, sW, _, zW = o.quantize_weights(W, cal.perm)
    _, _, Y = o.cluster_gemm_int(codes, wq, cal.cluster_off, cal.s, cal.z, sW, zW)
    rng = np.random.default_rng(1)
    shuffle = np.concatenate([cal.cluster_off[i] + rng.permutation(cal.cluster_off[i + 1] - cal.cluster_off[i])
                              for i in range(cal.g_eff)])
    _, _, Y2 = o.cluster_gemm_int(codes[:, shuffle], wq[:, shuffle], cal.cluster_off, cal.s, cal.z, sW, zW)
    assert np.abs(Y - Y2).max() <= 1e-12 * np.abs(Y).max()
    # swap the first two clusters wholesale
    a, b, c = cal.cluster_off[0], cal.cluster_off[1], cal.cluster_off[2]
    order = np.concatenate([np.arange(b, c), np.arange(a, b), np.arange(c, s.d)])
    off2 = np.array([0, c - b, c - a + 0, s.d])
    sw = [1, 0, 2]
    _, _, Y3 = o.cluster_gemm_int(codes[:, order], wq[:, order], off2, cal.s[sw], cal.z[sw], sW, zW)
    assert np.abs(Y - Y3).max() <= 1e-12 * np.abs(Y).max()


def test_quantized_product_approximates_the_float_layer():
    """End to end: the A8 path tracks the unquantized LayerNorm + linear layer, and
    clustering helps (more clusters, lower error) on the outlier-channel inputs."""
    s = w.tiny_site(31, 256, 64, n_cal=4, cal_rows=64)
    W = w.weight_matrix(32, 40, 256)
    y, _ = o.layernorm_f32(s.x, s.gamma, s.beta, 1e-5)
    errs = []
    for g in (1, 8):
        cal = o.calibrate(s.cal, s.gamma, s.beta, 1e-5, False, g, 4, seed=1)
        codes, _, _ = o.ln_quant(s.x, s.gamma, s.beta, 1e-5, False, cal.perm, cal.cluster_off, cal.inv_s, cal.z, 4)
        sizes = np.diff(cal.cluster_off)
        xh = o.dequantize(codes, np.repeat(cal.s, sizes)[None], np.repeat(cal.z, sizes)[None])
        errs.append(np.linalg.norm(xh - y[:, cal.perm]) / np.linalg.norm(y))
    assert errs[1] < 0.5 * errs[0]


# ---------------------------------------------------------------------------
# App. A.4 with its own weight parameters: one (s, z) per (output channel, input cluster)
# ---------------------------------------------------------------------------
def test_per_cluster_weight_quantization_is_eq_1_2_on_every_block():
    s, cal, W = _setup(seed=31, d=40, M=6, g=4, N=7)
    wq, sW, inv, zW = o.quantize_weights_per_cluster(W, cal.perm, cal.cluster_off)
    Wt = W[:, cal.perm]
    for n in range(W.shape[0]):
        for i in range(cal.g_eff):
            a, b = cal.cluster_off[i], cal.cluster_off[i + 1]
            blk = Wt[n, a:b].astype(np.float64)
            lo, hi = blk.min(), blk.max()
            if hi == lo:
                s_ref, z_ref = 1.0, -np.rint(lo)
            else:
                s_ref = (hi - lo) / 16.0                              # Eq. 2 with k = 4
                z_ref = -np.rint((hi + lo) / (2.0 * s_ref))
            assert float(sW[n, i]) == float(np.float32(s_ref)) and int(zW[n, i]) == int(z_ref)
            r = (Wt[n, a:b] * inv[n, i]).astype(np.float32).astype(np.float64)
            assert np.array_equal(wq[n, a:b], np.clip(np.rint(r) + z_ref, -8, 7))
            # a block's own range is never wider than its row's: the de-quantization error shrinks
            back = o.dequantize(wq[n, a:b], sW[n, i], zW[n, i])
            assert np.abs(back - blk).max() <= 2.5 * float(sW[n, i]) + 1e-12
    # one cluster: the per-row scheme
    wq1, s1, _, z1 = o.quantize_weights_per_cluster(W, cal.perm, np.array([0, W.shape[1]]))
    wqr, sr, _, zr = o.quantize_weights(W, cal.perm)
    assert np.array_equal(wq1, wqr) and np.array_equal(s1[:, 0], sr) and np.array_equal(z1[:, 0], zr)


def test_per_cluster_weight_product_both_methods_and_brute_force():
    s, cal, W = _setup(seed=33, d=36, M=5, g=3, N=6)
    codes, _, _ = o.ln_quant(s.x, s.gamma, s.beta, 1e-5, False, cal.perm, cal.cluster_off, cal.inv_s, cal.z, 4)
    wq, sW, _, zW = o.quantize_weights_per_cluster(W, cal.perm, cal.cluster_off)
    Yq, Y = o.cluster_gemm_int_pc(codes, wq, cal.cluster_off, cal.s, cal.z, sW, zW)
    Y1 = o.cluster_gemm_dequant_pc(codes, wq, cal.cluster_off, cal.s, cal.z, sW, zW)
    assert np.allclose(Y, Y1, rtol=1e-12, atol=1e-12 * np.abs(Y1).max())
    # triple loop over (token, output, cluster) of the zero-point-corrected integer products
    for t in range(codes.shape[0]):
        for n in range(wq.shape[0]):
            tot = 0.0
            for i in range(cal.g_eff):
                a, b = cal.cluster_off[i], cal.cluster_off[i + 1]
                acc = 0
                for c in range(a, b):
                    acc += (int(codes[t, c]) - int(cal.z[i])) * (int(wq[n, c]) - int(zW[n, i]))
                assert acc == Yq[i, t, n]
                tot += float(cal.s[i]) * float(sW[n, i]) * acc
            assert abs(tot - Y[t, n]) <= 1e-12 * max(1.0, abs(tot))
    # when every cluster of a row carries the row's pair, this is the per-row product
    wqr, sr, _, zr = o.quantize_weights(W, cal.perm)
    _, Yq_r, Y_r = o.cluster_gemm_int(codes, wqr, cal.cluster_off, cal.s, cal.z, sr, zr)
    Yq_b, Y_b = o.cluster_gemm_int_pc(codes, wqr, cal.cluster_off, cal.s, cal.z,
                                      np.repeat(sr[:, None], cal.g_eff, axis=1), np.repeat(zr[:, None], cal.g_eff, axis=1))
    assert np.array_equal(Yq_r, Yq_b) and np.allclose(Y_r, Y_b, rtol=1e-13, atol=0)


# ---------------------------------------------------------------------------
# App. A.4, first method, on bf16 operands
# ---------------------------------------------------------------------------
def _bf16_nearest_even_exact(v: float) -> float:
    """Nearest bf16 (8 significant bits) to a double, ties to even, by exact rational arithmetic."""
    from fractions import Fraction
    fr = Fraction(v)
    if fr == 0:
        return 0.0
    sign = -1 if fr < 0 else 1
    fr = abs(fr)
    e = 0
    while fr >= 256:
        fr /= 2
        e += 1
    while fr < 128:
        fr *= 2
        e -= 1
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return float(sign * Fraction(fl) * (Fraction(2) ** e))


def test_bf16_rounding_is_nearest_even():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal(400) * np.exp(rng.normal(0, 4, 400))).astype(np.float32)
    # ties: 8-bit significands with the next bit set and nothing below it, both parities
    ties = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.5 + 2.0 ** -8), 255.5 * 2.0 ** 10, 254.5 * 2.0 ** -20],
                    dtype=np.float32)
    got = o.round_to_bf16(np.concatenate([x, ties]))
    for v, gv in zip(np.concatenate([x, ties]), got):
        assert float(gv) == _bf16_nearest_even_exact(float(v))
    assert float(got[-5]) == 1.0 and float(got[-4]) == 1.0 + 2.0 ** -6      # 1 + 2^-8 -> even below, 1 + 3*2^-8 -> even above


def test_method_1_on_bf16_operands_against_the_exact_method_1():
    s, cal, W = _setup(seed=31, d=64, M=9, g=4, bits=4, N=12)
    codes, _, _ = o.ln_quant(s.x, s.gamma, s.beta, 1e-5, False, cal.perm, cal.cluster_off, cal.inv_s, cal.z, 4)
    wq, sW, _, zW = o.quantize_weights(W, cal.perm)
    exact = o.cluster_gemm_dequant(codes, wq, cal.cluster_off, cal.s, cal.z, sW, zW)
    xh, wh, Y = o.cluster_gemm_dequant_bf16(codes, wq, cal.cluster_off, cal.s, cal.z, sW, zW)
    # every operand is the bf16 nearest to its exact value s (q - z) rounded once to fp32
    sizes = np.diff(cal.cluster_off)
    sx = np.repeat(cal.s, sizes)
    zx = np.repeat(cal.z, sizes)
    for t, j in ((0, 0), (3, 17), (8, 63), (5, 40)):
        f32 = float(np.float32(float(sx[j]) * (int(codes[t, j]) - int(zx[j]))))
        assert float(xh[t, j]) == _bf16_nearest_even_exact(f32)
    for n, j in ((0, 0), (11, 63), (4, 9)):
        f32 = float(np.float32(float(sW[n]) * (int(wq[n, j]) - int(zW[n]))))
        assert float(wh[n, j]) == _bf16_nearest_even_exact(f32)
    # the product of the rounded operands lies within the rounding bound of two bf16 factors of the exact product
    xe = sx[None, :].astype(np.float64) * (codes.astype(np.float64) - zx[None, :])
    we = sW[:, None].astype(np.float64) * (wq.astype(np.float64) - zW[:, None])
    bound = (2.0 ** -8 + 2.0 ** -16) * (np.abs(xe) @ np.abs(we).T)
    assert np.all(np.abs(Y - exact) <= bound)
    assert np.abs(Y - exact).max() > 0          # and the rounding is really there

    # scales that are powers of two and small integers: every de-quantized value is a bf16 number, so the
    # bf16 form is the exact first method
    sX2 = np.array([0.5, 2.0, 0.125, 1.0], dtype=np.float32)
    sW2 = (2.0 ** np.arange(-6, 6)).astype(np.float32)
    xh2, wh2, Y2 = o.cluster_gemm_dequant_bf16(codes, wq, cal.cluster_off, sX2, cal.z, sW2, zW)
    assert np.abs(codes - np.repeat(cal.z, sizes)[None, :]).max() < 256
    assert np.array_equal(Y2, o.cluster_gemm_dequant(codes, wq, cal.cluster_off, sX2, cal.z, sW2, zW))
