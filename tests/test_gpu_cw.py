"""The product with one weight parameter pair per (output channel, input cluster) - App. A.4 as
printed - on the HIP path against the oracle: folded weights, parameters and tables bit for
bit, per-cluster row sums bit for bit, the literal integers Yq_i bit for bit, outputs to 1e-3."""
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
    rp_.load_library()
    assert torch.cuda.is_available()
    return rp_


def dev_bf16(x):
    return torch.from_numpy(w.bf16_bits(x).view(np.int16)).cuda().view(torch.bfloat16)


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    return (t.to(dtype) if dtype is not None else t).cuda()


def tol_of(Y):
    return 1e-3 * np.maximum(np.abs(Y), np.sqrt((Y * Y).mean(axis=-1, keepdims=True)))


def tab_col(i):
    return (i & 1) * 16 + (i >> 1)


CASES = {
    "tiny_a4": dict(seed=41, d=96, M=37, g=4, bits=4, N=40),
    "tiny_a3": dict(seed=42, d=200, M=70, g=5, bits=3, N=130),
    "tiny_a8": dict(seed=43, d=64, M=5, g=2, bits=8, N=33),
    "mid_a4": dict(seed=44, d=2048, M=257, g=16, bits=4, N=384),
    "mid_a3": dict(seed=45, d=1024, M=300, g=32, bits=3, N=520),
    "decode_a3": dict(seed=46, d=1536, M=16, g=32, bits=3, N=1024),
    "relu_site": dict(seed=47, d=320, M=40, g=6, bits=4, N=48, ln=False, relu=True),
    # every block of one cluster lies far from zero relative to its width: zero points of millions
    "far_from_zero_blocks": dict(seed=48, d=128, M=33, g=6, bits=4, N=72, narrow=True),
}


@pytest.mark.parametrize("name", list(CASES))
def test_clusterwise_weight_parameters_against_oracle(rp, name):
    kw = dict(CASES[name])
    ln, relu, narrow = kw.pop("ln", True), kw.pop("relu", False), kw.pop("narrow", False)
    seed, d, M, g, bits, N = (kw[k] for k in ("seed", "d", "M", "g", "bits", "N"))
    site = w.make_site(seed, d, M, 3, 32)
    gamma, beta = (site.gamma, site.beta) if ln else (None, None)
    cal = o.calibrate(site.cal, gamma, beta, EPS, relu, g, bits, seed=seed)
    W = w.weight_matrix(seed + 7, N, d)
    if narrow:
        sizes_ = np.diff(cal.cluster_off)
        i_small = int(np.argmin(np.where(sizes_ >= 2, sizes_, 1 << 30)))
        chans = cal.perm[cal.cluster_off[i_small]:cal.cluster_off[i_small + 1]]
        W[:, chans] = (np.float32(0.03) + np.float32(4e-9) * np.arange(len(chans) * N, dtype=np.float32).reshape(N, -1) % 7)
    codes, xsum, fragile = o.ln_quant(site.x, gamma, beta, EPS, relu, cal.perm, cal.cluster_off, cal.inv_s, cal.z, bits)
    wq, sW, _, zW = o.quantize_weights_per_cluster(W, cal.perm, cal.cluster_off)
    if narrow:
        assert np.abs(zW).max() > 1 << 22
    Yq, Y = o.cluster_gemm_int_pc(codes, wq, cal.cluster_off, cal.s, cal.z, sW, zW)
    ge = cal.g_eff
    sizes = np.diff(cal.cluster_off)
    wsum = np.stack([wq[:, a:b].sum(axis=1) for a, b in zip(cal.cluster_off[:-1], cal.cluster_off[1:])], axis=1)

    # device: calibrate + fold with per-block parameters
    batches = [dev_bf16(b) for b in site.cal]
    k1 = rp.calibrate_site(batches, dev(gamma) if ln else None, dev(beta) if ln else None, EPS, relu, g, bits, seed=seed)
    assert np.array_equal(k1.perm, cal.perm) and np.array_equal(k1.s, cal.s) and np.array_equal(k1.z, cal.z)
    lin = rp.fold_linear_cw(k1, dev(W))
    gw = torch.empty((N, d), dtype=torch.int8, device="cuda")
    rp.rptq_unpack_weights(lin.Wq, N, k1.cluster_off, gw)
    assert np.array_equal(gw.cpu().numpy().astype(np.int64), wq)
    dec, extra = packfmt.unpack_weights(lin.Wq.cpu().numpy(), N, cal.cluster_off)
    assert np.array_equal(dec, wq) and (extra == 0).all()
    assert np.array_equal(lin.sW.cpu().numpy(), sW)
    assert np.array_equal(lin.zW.cpu().numpy().astype(np.int64), zW)
    assert np.array_equal(lin.wsum.cpu().numpy().astype(np.int64), wsum)
    n_p = (N + 255) // 256 * 256
    st = lin.scale_tab.cpu().numpy().reshape(ge, n_p)
    want_st = (cal.s.astype(np.float64)[:, None] * sW.astype(np.float64).T).astype(np.float32)
    assert np.array_equal(st[:, :N], want_st)
    ct = lin.cross_tab.cpu().numpy().reshape(n_p, 32)
    want_ct = np.zeros((N, 32), dtype=np.float32)
    for i in range(ge):
        want_ct[:, tab_col(i)] = (-(sW[:, i].astype(np.float64) * zW[:, i])).astype(np.float32)
    assert np.array_equal(ct[:N], want_ct) and (ct[N:] == 0).all()
    ref_col = ((cal.s.astype(np.float64) * cal.z)[None, :] * sW.astype(np.float64) * wsum).sum(axis=1)
    scale_col = np.abs((cal.s.astype(np.float64) * cal.z)[None, :] * sW.astype(np.float64) * wsum).sum(axis=1).max()
    assert np.abs(lin.colterm.cpu().numpy() - ref_col).max() <= 1e-6 * max(scale_col, 1e-30)

    # online: oracle-made codes (packed by the test-side encoder) -> per-cluster row sums -> product
    pc = dev(packfmt.pack_codes(codes, cal.cluster_off, bits).reshape(-1))
    rs = rp.cluster_rowsums(k1, pc, M)
    torch.cuda.synchronize()
    got_rs = rs.cpu().numpy()[:M * 32].reshape(M, 32)
    want_rs = np.zeros((M, 32), dtype=np.float32)
    for i in range(ge):
        want_rs[:, tab_col(i)] = (float(cal.s[i]) * (xsum[:, i].astype(np.float64) - float(sizes[i]) * float(cal.z[i]))).astype(np.float32)
    assert np.array_equal(got_rs, want_rs)

    yq = torch.full((ge, M, N), 123456789, dtype=torch.int32, device="cuda")
    rp.rptq_cluster_gemm_partials_cw(pc, M, bits, lin.Wq, N, cal.cluster_off, cal.z, lin.zW, dev(xsum.astype(np.int32)),
                                     lin.wsum, yq)
    torch.cuda.synchronize()
    # (int32 output: equal modulo 2^32, which is plain equality unless a block's zero point is huge)
    assert np.array_equal(yq.cpu().numpy(), Yq.astype(np.int32))
    assert narrow or np.array_equal(yq.cpu().numpy().astype(np.int64), Yq)

    y32 = rp.cluster_gemm_cw(k1, lin, pc, rs, M, dtype=torch.float32)
    torch.cuda.synchronize()
    err = np.abs(y32.cpu().numpy().astype(np.float64) - Y)
    print("%s: max err/tol %.4f" % (name, float((err / tol_of(Y)).max())))
    assert (err <= tol_of(Y)).all()
    y16 = rp.cluster_gemm_cw(k1, lin, pc, rs, M, dtype=torch.bfloat16)
    ref16 = w.round_to_bf16(Y.astype(np.float32)).astype(np.float64)
    assert (np.abs(y16.float().cpu().numpy().astype(np.float64) - ref16) <= np.abs(ref16) * 2.0 ** -7 + tol_of(Y)).all()


def test_clusterwise_config1_sized_product(rp):
    """configs[1]'s qkv product (2048 x 6144 x 2048, 16 clusters, A4) with per-block weight parameters:
    every output against the first method of App. A.4, the literal integers on a block of rows."""
    cfg = w.CONFIGS[1]
    spec = cfg.sites[0]
    seed, M, d, bits, g = w.site_seed(1, 0), cfg.M, spec.d, cfg.bits, spec.g
    N = spec.gemms[0][1]
    site = w.make_site(seed, d, M, cfg.n_cal)
    cal = o.calibrate(site.cal, site.gamma, site.beta, EPS, False, g, bits, seed=seed)
    W = w.weight_matrix(seed + 500, N, d)
    codes, xsum, fragile = o.ln_quant(site.x, site.gamma, site.beta, EPS, False, cal.perm, cal.cluster_off, cal.inv_s, cal.z, bits)
    wq, sW, _, zW = o.quantize_weights_per_cluster(W, cal.perm, cal.cluster_off)
    Y = o.cluster_gemm_dequant_pc(codes, wq, cal.cluster_off, cal.s, cal.z, sW, zW)
    k1 = rp.calibrate_site([dev_bf16(b) for b in site.cal], dev(site.gamma), dev(site.beta), EPS, False, g, bits, seed=seed)
    lin = rp.fold_linear_cw(k1, dev(W))
    pcodes, _, _ = rp.ln_quant(k1, dev_bf16(site.x), EPS)          # the whole path on the device
    rs = rp.cluster_rowsums(k1, pcodes, M)
    y = rp.cluster_gemm_cw(k1, lin, pcodes, rs, M, dtype=torch.float32)
    torch.cuda.synchronize()
    ok = ~fragile
    err = np.abs(y.cpu().numpy().astype(np.float64) - Y)
    print("configs[1] qkv, per-block weight parameters: max err/tol %.4f" % float((err / tol_of(Y))[ok].max()))
    assert (err[ok] <= tol_of(Y)[ok]).all()
    rows = 192
    Yq, _ = o.cluster_gemm_int_pc(codes[:rows], wq, cal.cluster_off, cal.s, cal.z, sW, zW)
    pc = dev(packfmt.pack_codes(codes[:rows], cal.cluster_off, bits).reshape(-1))
    yq = torch.empty((cal.g_eff, rows, N), dtype=torch.int32, device="cuda")
    rp.rptq_cluster_gemm_partials_cw(pc, rows, bits, lin.Wq, N, cal.cluster_off, cal.z, lin.zW,
                                     dev(xsum[:rows].astype(np.int32)), lin.wsum, yq)
    torch.cuda.synchronize()
    assert np.array_equal(yq.cpu().numpy().astype(np.int64), Yq)


def test_clusterwise_config3_fc1_sampled(rp):
    """configs[3]'s fc1 (8192 x 49152 x 12288, 32 clusters, A3) at full size with per-block weight
    parameters: every output of sampled tokens against whole rows computed by the oracle."""
    cfg = w.CONFIGS[3]
    spec = cfg.sites[1]
    seed, M, d, bits, g = w.site_seed(3, 1), cfg.M, spec.d, cfg.bits, spec.g
    N = spec.gemms[0][1]
    rows = 512
    site = w.make_site(seed, d, rows, cfg.n_cal)
    cal = o.calibrate(site.cal, site.gamma, site.beta, EPS, False, g, bits, seed=seed)
    k1 = rp.calibrate_site([dev_bf16(b) for b in site.cal], dev(site.gamma), dev(site.beta), EPS, False, g, bits, seed=seed)
    assert np.array_equal(k1.perm, cal.perm) and np.array_equal(k1.z, cal.z)
    x = dev_bf16(site.x).repeat(M // rows, 1).contiguous()
    pcodes, _, _ = rp.ln_quant(k1, x, EPS)
    rs = rp.cluster_rowsums(k1, pcodes, M)
    rng = np.random.default_rng(33)
    ts = np.unique(np.concatenate([[0, M - 1], rng.integers(0, M, 10)]))
    rc, _, fragile = o.ln_quant(site.x[ts % rows], site.gamma, site.beta, EPS, False, cal.perm, cal.cluster_off, cal.inv_s, cal.z, bits)
    Wd = torch.empty((N, d), dtype=torch.float32, device="cuda")
    Y = np.empty((len(ts), N), dtype=np.float64)
    for r0 in range(0, N, 4096):
        Wc = w.weight_rows(seed + 500, N, d, np.arange(r0, r0 + 4096))
        Wd[r0:r0 + 4096] = torch.from_numpy(Wc).cuda()
        wq, sW, _, zW = o.quantize_weights_per_cluster(Wc, cal.perm, cal.cluster_off)
        Y[:, r0:r0 + 4096] = o.cluster_gemm_dequant_pc(rc, wq, cal.cluster_off, cal.s, cal.z, sW, zW)
    lin = rp.fold_linear_cw(k1, Wd)
    del Wd
    y = rp.cluster_gemm_cw(k1, lin, pcodes, rs, M, dtype=torch.bfloat16)
    torch.cuda.synchronize()
    yrows = y[torch.from_numpy(ts).cuda()].float().cpu().numpy().astype(np.float64)
    ok = ~fragile
    tol = tol_of(Y) + np.abs(Y) * 2.0 ** -7
    err = np.abs(yrows - Y)
    print("configs[3] fc1, per-block weight parameters: max err/tol %.3f" % float((err / tol)[ok].max()))
    assert (err[ok] <= tol[ok]).all()
