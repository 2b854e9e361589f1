"""Parity of the HIP path against the CPU oracle, element by element, through the C ABI.

Stage-isolated: every stage is fed the oracle's output of the previous stage, so the
bit-exact comparisons do not inherit float noise from upstream.  Codes, permutations,
cluster assignments and int32 per-cluster sums must match exactly; de-quantized fp32
outputs within 1e-3 of max(|ref|, rms of the ref row)."""
import numpy as np
import pytest

import workloads as w
from oracle import rptq_oracle as o

import packfmt

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
EPS = 1e-5


@pytest.fixture(scope="module")
def rp():
    import paper_2304_01089_amd as rp_
    rp_.load_library()            # raises if the HIP library is not built: no fallback
    assert torch.cuda.is_available()
    return rp_


def dev_bf16(x):
    return torch.from_numpy(w.bf16_bits(x).view(np.int16)).cuda().view(torch.bfloat16)


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


class Case:
    """One site + linear layer: synthetic inputs, oracle results for every stage."""

    def __init__(self, seed, d, M, g, bits, N, n_cal=3, cal_rows=32, ln=True, relu=False):
        self.d, self.M, self.g, self.bits, self.N, self.ln, self.relu = d, M, g, bits, N, ln, relu
        self.site = w.make_site(seed, d, M, n_cal, cal_rows)
        s = self.site
        self.gamma = s.gamma if ln else None
        self.beta = s.beta if ln else None
        self.cal = o.calibrate(s.cal, self.gamma, self.beta, EPS, relu, g, bits, seed=seed)
        self.W = w.weight_matrix(seed + 7, N, d)
        c = self.cal
        self.codes, self.xsum, self.fragile = o.ln_quant(s.x, self.gamma, self.beta, EPS, relu, c.perm,
                                                         c.cluster_off, c.inv_s, c.z, bits)
        self.wq, self.sW, _, self.zW = o.quantize_weights(self.W, c.perm)
        self.wsum = np.stack([self.wq[:, c.cluster_off[i]:c.cluster_off[i + 1]].sum(axis=1)
                              for i in range(c.g_eff)], axis=1)

    def gemm(self):
        c = self.cal
        return o.cluster_gemm_int(self.codes, self.wq, c.cluster_off, c.s, c.z, self.sW, self.zW)


CASES = {
    "tiny_a4": dict(seed=11, d=96, M=37, g=4, bits=4, N=40),
    "tiny_a3": dict(seed=12, d=200, M=70, g=5, bits=3, N=130),
    "tiny_a8": dict(seed=13, d=64, M=5, g=2, bits=8, N=33),
    "one_cluster": dict(seed=14, d=256, M=33, g=1, bits=4, N=64),
    "relu_site": dict(seed=15, d=320, M=40, g=6, bits=4, N=48, ln=False, relu=True),
    "cfg0": dict(seed=w.site_seed(0, 0), d=768, M=128, g=8, bits=8, N=3072, n_cal=4, cal_rows=128),
    "mid_a3": dict(seed=16, d=1024, M=300, g=16, bits=3, N=520, n_cal=4, cal_rows=64),
    "mid_a4": dict(seed=17, d=2048, M=257, g=16, bits=4, N=384, n_cal=4, cal_rows=64),
    "decode_a3": dict(seed=18, d=1536, M=16, g=32, bits=3, N=1024, n_cal=4, cal_rows=64),
    # a row too wide for three LDS row buffers (two buffers, one more barrier per row), four
    # input chunks and four units per thread
    "wide_relu": dict(seed=19, d=24576, M=9, g=8, bits=4, N=32, n_cal=2, cal_rows=16, ln=False, relu=True),
    "one_row": dict(seed=20, d=512, M=1, g=4, bits=3, N=64),
    # the depth of the large workloads on the 64-token tile (two row tiles, the second ragged; two
    # column tiles): the int32 accumulators run over all of K without being cleared, so the
    # literal per-cluster integers are pinned at K = 12288 (3 bit) and K = 20480 (4 bit)
    "deep_a3": dict(seed=21, d=12288, M=72, g=32, bits=3, N=512, n_cal=2, cal_rows=64),
    "deep_relu_a4": dict(seed=22, d=20480, M=72, g=32, bits=4, N=512, n_cal=2, cal_rows=64, ln=False, relu=True),
}
_cache = {}


def get_case(name):
    if name not in _cache:
        _cache[name] = Case(**CASES[name])
    return _cache[name]


ALL = list(CASES)


# ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("name", ALL)
def test_calibrate_matches_oracle(rp, name):
    c = get_case(name)
    batches = [dev_bf16(b) for b in c.site.cal]
    gamma = dev(c.gamma) if c.ln else None
    beta = dev(c.beta) if c.ln else None
    r = rp.rptq_calibrate(batches, gamma, beta, EPS, c.relu, c.g, c.bits, seed=CASES[name]["seed"])
    ref = c.cal
    assert np.array_equal(r["ch_min"], ref.ch_min)
    assert np.array_equal(r["ch_max"], ref.ch_max)
    assert r["g_eff"] == ref.g_eff
    for key in ("assign", "perm", "cluster_off", "s", "inv_s", "z"):
        assert np.array_equal(r[key], getattr(ref, key)), key


def _folded_site(rp, c):
    cal = c.cal
    k_p = rp.rptq_padded_k(cal.cluster_off)
    perm_pad = torch.empty(k_p, dtype=torch.int32, device="cuda")
    gpad = torch.empty(k_p, dtype=torch.float32, device="cuda") if c.ln else None
    bpad = torch.empty(k_p, dtype=torch.float32, device="cuda") if c.ln else None
    rp.rptq_fold_reorder(dev(c.gamma) if c.ln else None, dev(c.beta) if c.ln else None, c.d, cal.perm,
                         cal.cluster_off, None, None, None, 0, c.d, None, perm_pad, gpad, bpad,
                         None, None, None, None, None)
    return k_p, perm_pad, gpad, bpad


@pytest.mark.parametrize("name", ALL)
def test_ln_quant_codes_bit_exact(rp, name):
    c = get_case(name)
    cal = c.cal
    k_p, perm_pad, gpad, bpad = _folded_site(rp, c)
    pad_off, k_p_ref = packfmt.padded_layout(cal.cluster_off)
    assert k_p == k_p_ref
    # folded LayerNorm parameters: gamma' = gamma[S], beta' = beta[S] in the padded layout
    pp = perm_pad.cpu().numpy()
    ref_pp = np.full(k_p, -1, dtype=np.int32)
    for i in range(cal.g_eff):
        n = cal.cluster_off[i + 1] - cal.cluster_off[i]
        ref_pp[pad_off[i]:pad_off[i] + n] = cal.perm[cal.cluster_off[i]:cal.cluster_off[i + 1]]
    assert np.array_equal(pp, ref_pp)
    if c.ln:
        gr, br = o.fold_layernorm(c.gamma, c.beta, cal.perm)
        assert np.array_equal(gpad.cpu().numpy()[ref_pp >= 0], gr)
        assert np.array_equal(bpad.cpu().numpy()[ref_pp >= 0], br)

    x = dev_bf16(c.site.x)
    codes = torch.empty(rp.rptq_codes_bytes(c.M, k_p, c.bits), dtype=torch.uint8, device="cuda")
    xsum = torch.empty((c.M, cal.g_eff), dtype=torch.int32, device="cuda")
    rowterm = torch.empty(c.M, dtype=torch.float32, device="cuda")
    rp.rptq_ln_quant(x, c.M, c.d, gpad, bpad, EPS, c.relu, perm_pad, cal.cluster_off, cal.s, cal.inv_s, cal.z,
                     c.bits, codes, xsum, rowterm)
    torch.cuda.synchronize()
    packed = codes.cpu().numpy().reshape(c.M, -1)
    got, pads = packfmt.unpack_codes(packed, cal.cluster_off, c.bits)       # decoded from the documented layout
    assert (pads == 0).all()
    ok = ~c.fragile
    assert ok.sum() >= c.M - max(2, c.M // 100)
    assert np.array_equal(got[ok], c.codes[ok])
    assert np.abs(got - c.codes).max() <= 1                                  # fragile rows: at most one step
    # the library's own unpacker agrees with the documented layout
    out = torch.empty((c.M, c.d), dtype=torch.int8, device="cuda")
    rp.rptq_unpack_codes(codes, c.M, cal.cluster_off, c.bits, out)
    assert np.array_equal(out.cpu().numpy().astype(np.int64), got)
    # per-cluster code sums and the de-quantized row sum
    gx = xsum.cpu().numpy().astype(np.int64)
    assert np.array_equal(gx[ok], c.xsum[ok])
    sizes = np.diff(cal.cluster_off)
    ref_rt = (cal.s.astype(np.float64)[None, :] * (gx - sizes[None, :] * cal.z[None, :])).sum(axis=1)
    scale = np.abs(cal.s.astype(np.float64)[None, :] * (gx - sizes[None, :] * cal.z[None, :])).sum(axis=1)
    assert np.abs(rowterm.cpu().numpy() - ref_rt).max() <= 1e-6 * scale.max()


def _folded_linear(rp, c, w_dtype=torch.float32):
    cal = c.cal
    k_p, perm_pad, _, _ = _folded_site(rp, c)
    N = c.N
    Wq = torch.zeros(rp.rptq_weight_bytes(N, k_p), dtype=torch.uint8, device="cuda")
    sW = torch.empty(N, dtype=torch.float32, device="cuda")
    zW = torch.empty(N, dtype=torch.int32, device="cuda")
    wsum = torch.empty((N, cal.g_eff), dtype=torch.int32, device="cuda")
    colterm = torch.empty(N, dtype=torch.float32, device="cuda")
    rp.rptq_fold_reorder(None, None, c.d, cal.perm, cal.cluster_off, cal.s, cal.z,
                         dev(c.W, w_dtype), N, c.d, None, perm_pad, None, None, Wq, sW, zW, wsum, colterm)
    torch.cuda.synchronize()
    return k_p, Wq, sW, zW, wsum, colterm


@pytest.mark.parametrize("name", ALL)
def test_fold_reorder_weights_bit_exact(rp, name):
    c = get_case(name)
    cal = c.cal
    k_p, Wq, sW, zW, wsum, colterm = _folded_linear(rp, c)
    got, extra = packfmt.unpack_weights(Wq.cpu().numpy(), c.N, cal.cluster_off)
    assert np.array_equal(got, c.wq) and (extra == 0).all()
    assert np.array_equal(sW.cpu().numpy(), c.sW)
    assert np.array_equal(zW.cpu().numpy().astype(np.int64), c.zW)
    assert np.array_equal(wsum.cpu().numpy().astype(np.int64), c.wsum)
    ref_ct = (cal.s.astype(np.float64) * cal.z)[None, :] * c.wsum
    assert np.abs(colterm.cpu().numpy() - ref_ct.sum(axis=1)).max() <= 1e-6 * max(np.abs(ref_ct).sum(axis=1).max(), 1e-30)
    out = torch.empty((c.N, c.d), dtype=torch.int8, device="cuda")
    rp.rptq_unpack_weights(Wq, c.N, cal.cluster_off, out)
    assert np.array_equal(out.cpu().numpy().astype(np.int64), c.wq)


def _gemm_inputs(rp, c):
    """Oracle-made operands, packed by the test-side encoder."""
    cal = c.cal
    k_p = rp.rptq_padded_k(cal.cluster_off)
    codes = dev(packfmt.pack_codes(c.codes, cal.cluster_off, c.bits).reshape(-1))
    Wq = dev(packfmt.pack_weights(c.wq, cal.cluster_off))
    sizes = np.diff(cal.cluster_off)
    sx64 = cal.s.astype(np.float64)
    rowterm = (sx64[None, :] * (c.xsum - sizes[None, :] * cal.z[None, :])).sum(axis=1)
    colterm = ((sx64 * cal.z)[None, :] * c.wsum).sum(axis=1)
    return (k_p, codes, Wq, dev(c.sW), dev(c.zW.astype(np.int32)), dev(colterm.astype(np.float32)),
            dev(rowterm.astype(np.float32)), dev(c.xsum.astype(np.int32)), dev(c.wsum.astype(np.int32)))


@pytest.mark.parametrize("name", ALL)
def test_cluster_gemm_partial_sums_bit_exact(rp, name):
    c = get_case(name)
    cal = c.cal
    k_p, codes, Wq, sW, zW, colterm, rowterm, xsum, wsum = _gemm_inputs(rp, c)
    yq = torch.full((cal.g_eff, c.M, c.N), 123456789, dtype=torch.int32, device="cuda")
    rp.rptq_cluster_gemm_partials(codes, c.M, c.bits, Wq, c.N, cal.cluster_off, cal.z, zW, xsum, wsum, yq)
    torch.cuda.synchronize()
    _, Yq, _ = c.gemm()
    assert np.array_equal(yq.cpu().numpy().astype(np.int64), Yq)


@pytest.mark.parametrize("name", ALL)
def test_cluster_gemm_output_within_tolerance(rp, name):
    c = get_case(name)
    cal = c.cal
    k_p, codes, Wq, sW, zW, colterm, rowterm, _, _ = _gemm_inputs(rp, c)
    _, _, Y = c.gemm()
    tol = 1e-3 * np.maximum(np.abs(Y), np.sqrt((Y * Y).mean(axis=1, keepdims=True)))
    y32 = torch.full((c.M, c.N), float("nan"), dtype=torch.float32, device="cuda")
    rp.rptq_cluster_gemm(codes, c.M, c.bits, Wq, c.N, cal.cluster_off, cal.s, sW, zW, colterm, rowterm, y32)
    torch.cuda.synchronize()
    got = y32.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert (np.abs(got - Y) <= tol).all(), float((np.abs(got - Y) / tol).max())
    # bf16 output: the same value rounded to bf16, at most one bf16 step from the rounded oracle
    y16 = torch.empty((c.M, c.N), dtype=torch.bfloat16, device="cuda")
    rp.rptq_cluster_gemm(codes, c.M, c.bits, Wq, c.N, cal.cluster_off, cal.s, sW, zW, colterm, rowterm, y16)
    torch.cuda.synchronize()
    g16 = y16.float().cpu().numpy().astype(np.float64)
    ref16 = w.round_to_bf16(Y.astype(np.float32)).astype(np.float64)
    ulp = np.maximum(np.abs(ref16), 1e-30) * 2.0 ** -7
    assert (np.abs(g16 - ref16) <= ulp + tol).all()


@pytest.mark.parametrize("name", ["tiny_a4", "mid_a3", "cfg0", "relu_site"])
def test_chained_path_end_to_end(rp, name):
    """calibrate -> fold -> ln_quant -> gemm entirely on the HIP path, against the oracle's Y."""
    c = get_case(name)
    batches = [dev_bf16(b) for b in c.site.cal]
    gamma = dev(c.gamma) if c.ln else None
    beta = dev(c.beta) if c.ln else None
    cal = rp.calibrate_site(batches, gamma, beta, EPS, c.relu, c.g, c.bits, seed=CASES[name]["seed"])
    lin = rp.fold_linear(cal, dev(c.W))
    codes, _, rowterm = rp.ln_quant(cal, dev_bf16(c.site.x), EPS, c.relu)
    y = rp.cluster_gemm(cal, lin, codes, rowterm, c.M, dtype=torch.float32)
    torch.cuda.synchronize()
    _, _, Y = c.gemm()
    ok = ~c.fragile
    tol = 1e-3 * np.maximum(np.abs(Y), np.sqrt((Y * Y).mean(axis=1, keepdims=True)))
    assert (np.abs(y.cpu().numpy().astype(np.float64) - Y)[ok] <= tol[ok]).all()


def test_bf16_weights_accepted(rp):
    c = get_case("tiny_a4")
    Wb = w.round_to_bf16(c.W)
    wq, sW, _, zW = o.quantize_weights(Wb, c.cal.perm)
    cc = Case(**CASES["tiny_a4"])
    cc.W = Wb
    k_p, Wq, sWd, zWd, _, _ = _folded_linear(rp, cc, torch.bfloat16)
    got, _ = packfmt.unpack_weights(Wq.cpu().numpy(), c.N, c.cal.cluster_off)
    assert np.array_equal(got, wq) and np.array_equal(sWd.cpu().numpy(), sW)


def test_empty_batch_is_a_no_op(rp):
    c = get_case("tiny_a4")
    cal = c.cal
    k_p, perm_pad, gpad, bpad = _folded_site(rp, c)
    x = torch.zeros((1, c.d), dtype=torch.bfloat16, device="cuda")        # M = 0 rows of a valid buffer
    codes = torch.full((16,), 7, dtype=torch.uint8, device="cuda")
    rp.rptq_ln_quant(x, 0, c.d, gpad, bpad, EPS, False, perm_pad, cal.cluster_off, cal.s, cal.inv_s, cal.z,
                     c.bits, codes, None, None)
    y = torch.full((4,), 3.0, dtype=torch.float32, device="cuda")
    k_p, pc, Wq, sW, zW, colterm, rowterm, _, _ = _gemm_inputs(rp, c)
    rp.rptq_cluster_gemm(pc, 0, c.bits, Wq, c.N, cal.cluster_off, cal.s, sW, zW, colterm, rowterm, y)
    torch.cuda.synchronize()
    assert (codes.cpu().numpy() == 7).all() and (y.cpu().numpy() == 3.0).all()


def test_deterministic_across_runs(rp):
    c = get_case("mid_a4")
    cal = c.cal
    k_p, codes, Wq, sW, zW, colterm, rowterm, _, _ = _gemm_inputs(rp, c)
    outs = []
    for _ in range(2):
        y = torch.empty((c.M, c.N), dtype=torch.float32, device="cuda")
        rp.rptq_cluster_gemm(codes, c.M, c.bits, Wq, c.N, cal.cluster_off, cal.s, sW, zW, colterm, rowterm, y)
        outs.append(y.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])


@pytest.mark.parametrize("name", ["tiny_a4", "tiny_a3", "tiny_a8", "relu_site", "mid_a3", "mid_a4", "one_row", "deep_a3"])
def test_scatter_on_write_variant_gives_the_same_codes(rp, name):
    """Sec. 4.2's own wording of the fused reorder (LayerNorm in the original order, the reorder index
    offsets the write address) as a second implementation: packed codes identical to rptq_ln_quant's."""
    c = get_case(name)
    cal = c.cal
    k_p, perm_pad, gpad, bpad = _folded_site(rp, c)
    x = dev_bf16(c.site.x)
    codes = torch.empty(rp.rptq_codes_bytes(c.M, k_p, c.bits), dtype=torch.uint8, device="cuda")
    rp.rptq_ln_quant(x, c.M, c.d, gpad, bpad, EPS, c.relu, perm_pad, cal.cluster_off, cal.s, cal.inv_s, cal.z,
                     c.bits, codes, None, None)
    ws = torch.empty(rp.rptq_ln_quant_scatter_workspace_bytes(c.M, c.d, k_p) + 256, dtype=torch.uint8, device="cuda")
    ws = ws[(-ws.data_ptr()) % 256:]
    codes2 = torch.full_like(codes, 0x5A)
    rp.rptq_ln_quant_scatter(x, c.M, c.d, dev(c.gamma) if c.ln else None, dev(c.beta) if c.ln else None, EPS, c.relu,
                             perm_pad, cal.cluster_off, cal.inv_s, cal.z, c.bits, codes2, ws)
    torch.cuda.synchronize()
    assert torch.equal(codes, codes2)
    got, pads = packfmt.unpack_codes(codes2.cpu().numpy().reshape(c.M, -1), cal.cluster_off, c.bits)
    ok = ~c.fragile
    assert (pads == 0).all() and np.array_equal(got[ok], c.codes[ok])
