"""The first method of App. A.4 on the HIP path (de-quantize both operands to bf16, bf16 matrix cores,
fp32 accumulation) against the oracle: the de-quantized operands bit for bit, the product within the
tolerance of fp32 accumulation."""
import numpy as np
import pytest

import workloads as w
from oracle import rptq_oracle as o

import packfmt
from test_gpu_parity import Case, dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def rp():
    import paper_2304_01089_amd as rp_
    rp_.load_library()            # raises if the HIP library is not built: no fallback
    assert torch.cuda.is_available()
    return rp_


M1_CASES = {
    "tiny_a4": dict(seed=41, d=96, M=37, g=4, bits=4, N=40),
    "tiny_a3": dict(seed=42, d=200, M=70, g=5, bits=3, N=132),
    "tiny_a8": dict(seed=43, d=64, M=5, g=2, bits=8, N=36),
    "relu_site": dict(seed=44, d=320, M=40, g=6, bits=4, N=48, ln=False, relu=True),
    # several 128 x 128 tiles with ragged edges in both directions, many K steps
    "mid_a3": dict(seed=45, d=1024, M=300, g=16, bits=3, N=520, n_cal=4, cal_rows=64),
    "mid_a4": dict(seed=46, d=2048, M=257, g=16, bits=4, N=388, n_cal=4, cal_rows=64),
    "one_row": dict(seed=47, d=512, M=1, g=4, bits=3, N=64),
}
_cache = {}


def get_case(name):
    if name not in _cache:
        _cache[name] = Case(**M1_CASES[name])
    return _cache[name]


def _bits(t):
    """bf16 device tensor -> uint16 bit patterns on the host."""
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("name", list(M1_CASES))
def test_method_1_operands_and_product(rp, name):
    c = get_case(name)
    cal = c.cal
    k_p = rp.rptq_padded_k(cal.cluster_off)
    pad_off, _ = packfmt.padded_layout(cal.cluster_off)
    codes = dev(packfmt.pack_codes(c.codes, cal.cluster_off, c.bits).reshape(-1))
    Wq = dev(packfmt.pack_weights(c.wq, cal.cluster_off))
    xh_ref, wh_ref, Y = o.cluster_gemm_dequant_bf16(c.codes, c.wq, cal.cluster_off, cal.s, cal.z, c.sW, c.zW)

    x_hat = torch.full((c.M, k_p), float("nan"), dtype=torch.bfloat16, device="cuda")
    w_hat = torch.full((c.N, k_p), float("nan"), dtype=torch.bfloat16, device="cuda")
    rp.rptq_dequant_codes(codes, c.M, c.bits, cal.cluster_off, cal.s, cal.z, x_hat)
    rp.rptq_dequant_weights(Wq, c.N, cal.cluster_off, dev(c.sW), dev(c.zW.astype(np.int32)), w_hat)
    torch.cuda.synchronize()
    # operands: the oracle's bf16 values bit for bit at the real positions, zero at the pad positions
    xb, wb = _bits(x_hat), _bits(w_hat)
    real = np.zeros(k_p, dtype=bool)
    for i in range(cal.g_eff):
        real[pad_off[i]:pad_off[i] + (cal.cluster_off[i + 1] - cal.cluster_off[i])] = True
    assert np.array_equal(xb[:, real], w.bf16_bits(xh_ref))
    assert np.array_equal(wb[:, real], w.bf16_bits(wh_ref))
    assert (xb[:, ~real] == 0).all() and (wb[:, ~real] == 0).all()

    # product: fp32 accumulation of exact products in some order: |error| <= K_p 2^-24 sum |terms|, far inside the
    # 1e-3 reading; measured against the oracle's exact product of the same bf16 operands
    y32 = torch.full((c.M, c.N), float("nan"), dtype=torch.float32, device="cuda")
    rp.rptq_gemm_bf16(x_hat, w_hat, c.M, c.N, k_p, y32)
    torch.cuda.synchronize()
    got = y32.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    tol = 1e-3 * np.maximum(np.abs(Y), np.sqrt((Y * Y).mean(axis=1, keepdims=True)))
    assert (np.abs(got - Y) <= tol).all(), float((np.abs(got - Y) / tol).max())
    bound = k_p * 2.0 ** -24 * (np.abs(xh_ref).astype(np.float64) @ np.abs(wh_ref).astype(np.float64).T)
    assert (np.abs(got - Y) <= bound + 1e-30).all()
    y16 = torch.empty((c.M, c.N), dtype=torch.bfloat16, device="cuda")
    rp.rptq_gemm_bf16(x_hat, w_hat, c.M, c.N, k_p, y16)
    torch.cuda.synchronize()
    g16 = y16.float().cpu().numpy().astype(np.float64)
    ref16 = w.round_to_bf16(Y.astype(np.float32)).astype(np.float64)
    assert (np.abs(g16 - ref16) <= np.maximum(np.abs(ref16), 1e-30) * 2.0 ** -7 + tol).all()

    # against the second method (the exact value both methods approximate the same layer with): the first method's
    # extra error is the bf16 rounding of its operands
    _, _, Y2 = c.gemm()
    xe = np.abs(xh_ref).astype(np.float64) @ np.abs(wh_ref).astype(np.float64).T
    assert (np.abs(got - Y2) <= (2.0 ** -8 + 2.0 ** -15) * xe + bound).all()
    rms2 = np.sqrt((Y2 * Y2).mean())
    print("%s: first method on bf16 operands deviates from the exact product by up to %.2e of its rms (fp32 accumulation alone: %.2e)"
          % (name, np.abs(got - Y2).max() / rms2, np.abs(got - Y).max() / rms2))


def test_method_1_validation(rp):
    x = torch.zeros((8, 256), dtype=torch.bfloat16, device="cuda")
    wt = torch.zeros((8, 256), dtype=torch.bfloat16, device="cuda")
    y = torch.zeros((8, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(rp.RptqError):
        rp.rptq_gemm_bf16(x, wt, 8, 8, 200, y)        # K not a multiple of 64
    with pytest.raises(rp.RptqError):
        rp.rptq_gemm_bf16(x, wt, 8, 6, 256, y)        # N not a multiple of 4
    rp.rptq_gemm_bf16(x, wt, 0, 8, 256, y)            # no rows: nothing to do
