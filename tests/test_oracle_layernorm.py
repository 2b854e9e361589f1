"""Pins for the oracle's LayerNorm and calibration min/max."""
import numpy as np
import torch

import workloads as w
from oracle import rptq_oracle as o


def _site(seed=3, d=96, M=40):
    return w.tiny_site(seed, d, M)


def test_matches_library_layernorm_fp64():
    s = _site()
    y, _ = o.layernorm_f32(s.x, s.gamma, s.beta, 1e-5)
    ref = torch.nn.functional.layer_norm(
        torch.from_numpy(s.x.astype(np.float64)), (s.d,),
        torch.from_numpy(s.gamma.astype(np.float64)),
        torch.from_numpy(s.beta.astype(np.float64)), 1e-5).numpy()
    scale = np.abs(ref).max()
    assert np.abs(y.astype(np.float64) - ref).max() <= 4e-7 * scale


def test_constant_row_gives_beta():
    s = _site()
    x = np.full((3, s.d), 1.5, dtype=np.float32)
    y, _ = o.layernorm_f32(x, s.gamma, s.beta, 1e-5)
    assert np.array_equal(y, np.broadcast_to(s.beta, y.shape))


def test_unit_gamma_zero_beta_statistics():
    s = _site(seed=5, d=512, M=16)
    y, _ = o.layernorm_f32(s.x, np.ones(s.d, np.float32), np.zeros(s.d, np.float32), 0.0)
    y = y.astype(np.float64)
    assert np.abs(y.mean(axis=1)).max() < 1e-6
    assert np.abs(y.var(axis=1) - 1.0).max() < 1e-5


def test_eps_enters_under_the_root():
    x = np.array([[1.0, -1.0, 1.0, -1.0]], dtype=np.float32)       # mean 0, var 1
    y, _ = o.layernorm_f32(x, np.ones(4, np.float32), np.zeros(4, np.float32), 3.0)
    assert np.allclose(y, x * 0.5)                                  # 1/sqrt(1+3)


def test_permutation_equivariance():
    s = _site(seed=9)
    rng = np.random.default_rng(0)
    p = rng.permutation(s.d)
    y, fr = o.layernorm_f32(s.x, s.gamma, s.beta, 1e-5)
    yp, frp = o.layernorm_f32(s.x[:, p], s.gamma[p], s.beta[p], 1e-5)
    ok = ~(fr | frp)
    assert ok.sum() >= ok.size - 2
    assert np.array_equal(y[ok][:, p], yp[ok])


def test_calibration_minmax_is_plain_min_max():
    s = _site(seed=11, d=64, M=8)
    cmin, cmax = o.calibrate_minmax(s.cal, s.gamma, s.beta, 1e-5, False)
    allrows = np.concatenate(s.cal, axis=0)
    y, _ = o.layernorm_f32(allrows, s.gamma, s.beta, 1e-5)
    for c in range(s.d):                      # brute force per channel
        assert cmin[c] == min(y[:, c].tolist())
        assert cmax[c] == max(y[:, c].tolist())
    # non-LN site with ReLU: minimum can never be negative
    rmin, rmax = o.calibrate_minmax(s.cal, None, None, 1e-5, True)
    assert (rmin >= 0).all()
    assert np.array_equal(rmax, np.maximum(allrows.max(axis=0), 0))
