"""Parity at the workloads' full sizes, in the launch configuration bench.py times.

configs[1] is compared element by element; the larger workloads (configs[3], the bench
workload, and configs[4]) are checked on sampled tokens: their codes, and every output of
every product for those tokens, each computed by the oracle from the same seeded inputs.  Also the chained fc1 -> ReLU -> fc2 path of
configs[2] at reduced width, with fc1's rows permuted offline by fc2's reorder index."""
import numpy as np
import pytest

import workloads as w
from oracle import rptq_oracle as o

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


def tol_of(Y):
    return 1e-3 * np.maximum(np.abs(Y), np.sqrt((Y * Y).mean(axis=-1, keepdims=True)))


def test_config1_full_size_elementwise(rp):
    cfg = w.CONFIGS[1]
    for si, spec in enumerate(cfg.sites):
        seed = w.site_seed(1, si)
        site = w.make_site(seed, spec.d, cfg.M, cfg.n_cal)
        gamma, beta = torch.from_numpy(site.gamma).cuda(), torch.from_numpy(site.beta).cuda()
        cal = rp.calibrate_site([dev_bf16(b) for b in site.cal], gamma, beta, EPS, False, spec.g, cfg.bits, seed=seed)
        ref = o.calibrate(site.cal, site.gamma, site.beta, EPS, False, spec.g, cfg.bits, seed=seed)
        assert np.array_equal(ref.perm, cal.perm) and np.array_equal(ref.cluster_off, cal.cluster_off)
        assert np.array_equal(ref.s, cal.s) and np.array_equal(ref.z, cal.z)
        codes, xsum, rowterm = rp.ln_quant(cal, dev_bf16(site.x), EPS, want_xsum=True)
        got = torch.empty((cfg.M, spec.d), dtype=torch.int8, device="cuda")
        rp.rptq_unpack_codes(codes, cfg.M, cal.cluster_off, cfg.bits, got)
        rc, rx, fragile = o.ln_quant(site.x, site.gamma, site.beta, EPS, False, ref.perm, ref.cluster_off, ref.inv_s, ref.z, cfg.bits)
        ok = ~fragile
        assert ok.sum() >= cfg.M - 8
        assert np.array_equal(got.cpu().numpy()[ok], rc[ok])
        assert np.array_equal(xsum.cpu().numpy()[ok], rx[ok])
        for li, (name, N) in enumerate(spec.gemms):
            W = w.weight_matrix(seed + 500 + li, N, spec.d)
            lin = rp.fold_linear(cal, torch.from_numpy(W).cuda())
            wq, sW, _, zW = o.quantize_weights(W, ref.perm)
            gw = torch.empty((N, spec.d), dtype=torch.int8, device="cuda")
            rp.rptq_unpack_weights(lin.Wq, N, cal.cluster_off, gw)
            assert np.array_equal(gw.cpu().numpy(), wq)
            y = rp.cluster_gemm(cal, lin, codes, rowterm, cfg.M, dtype=torch.float32)
            _, _, Y = o.cluster_gemm_int(rc, wq, ref.cluster_off, ref.s, ref.z, sW, zW)
            d = np.abs(y.cpu().numpy().astype(np.float64) - Y)
            assert (d[ok] <= tol_of(Y)[ok]).all()
            y16 = rp.cluster_gemm(cal, lin, codes, rowterm, cfg.M, dtype=torch.bfloat16)   # the dtype bench.py times
            d16 = np.abs(y16.float().cpu().numpy().astype(np.float64) - Y)
            assert (d16[ok] <= tol_of(Y)[ok] + np.abs(Y[ok]) * 2.0 ** -7).all()


W_CHUNK = 4096


def oracle_rows_and_device_weights(seed, N, d, ref, rc):
    """One pass over the seeded weight matrix in row blocks: every block goes to the device
    (fp32) and through the oracle - Eq. 1-2 per output row, then the cluster-wise product
    of App. A.4 for the sampled tokens `rc` - so the oracle's result covers whole rows."""
    Wd = torch.empty((N, d), dtype=torch.float32, device="cuda")
    Y = np.empty((rc.shape[0], N), dtype=np.float64)
    for r0 in range(0, N, W_CHUNK):
        r1 = min(N, r0 + W_CHUNK)
        Wc = w.weight_rows(seed, N, d, np.arange(r0, r1))
        Wd[r0:r1] = torch.from_numpy(Wc).cuda()
        wq, sW, _, zW = o.quantize_weights(Wc, ref.perm)
        _, _, Y[:, r0:r1] = o.cluster_gemm_int(rc, wq, ref.cluster_off, ref.s, ref.z, sW, zW)
    return Wd, Y


@pytest.mark.parametrize("ci,si", [(3, 0), (3, 1), (4, 0)])
def test_large_configs_sampled(rp, ci, si):
    """configs[3] (both products: qkv 36864 x 12288, fc1 49152 x 12288) and configs[4] at full
    size and in bench.py's launch configuration: the codes of sampled tokens bit for bit, and
    for those tokens every output of the product, against whole rows computed by the oracle
    (which also supply the row rms of the tolerance: nothing the device computed sets it)."""
    cfg = w.CONFIGS[ci]
    spec = cfg.sites[si]
    seed = w.site_seed(ci, si)
    rows = min(cfg.M, 512)                                    # distinct rows generated on the host
    site = w.make_site(seed, spec.d, rows, cfg.n_cal)
    gamma, beta = torch.from_numpy(site.gamma).cuda(), torch.from_numpy(site.beta).cuda()
    cal = rp.calibrate_site([dev_bf16(b) for b in site.cal], gamma, beta, EPS, False, spec.g, cfg.bits, seed=seed)
    ref = o.calibrate(site.cal, site.gamma, site.beta, EPS, False, spec.g, cfg.bits, seed=seed)
    assert np.array_equal(ref.perm, cal.perm) and np.array_equal(ref.z, cal.z) and np.array_equal(ref.s, cal.s)
    reps = (cfg.M + rows - 1) // rows
    x = dev_bf16(site.x).repeat(reps, 1)[:cfg.M].contiguous()            # full M rows on the device
    codes, _, rowterm = rp.ln_quant(cal, x, EPS)
    rng = np.random.default_rng(10 * ci + si)
    ts = np.unique(np.concatenate([[0, cfg.M - 1], rng.integers(0, cfg.M, 14)]))
    rc, rx, fragile = o.ln_quant(site.x[ts % rows], site.gamma, site.beta, EPS, False, ref.perm, ref.cluster_off,
                                 ref.inv_s, ref.z, cfg.bits)
    got = torch.empty((cfg.M, spec.d), dtype=torch.int8, device="cuda")
    rp.rptq_unpack_codes(codes, cfg.M, cal.cluster_off, cfg.bits, got)
    g = got[torch.from_numpy(ts).cuda()].cpu().numpy()
    del got
    ok = ~fragile
    assert ok.sum() >= len(ts) - 2
    assert np.array_equal(g[ok], rc[ok])
    tsd = torch.from_numpy(ts).cuda()
    for li, (name, N) in enumerate(spec.gemms):
        Wd, Y = oracle_rows_and_device_weights(seed + 500 + li, N, spec.d, ref, rc)
        lin = rp.fold_linear(cal, Wd)
        del Wd
        y = rp.cluster_gemm(cal, lin, codes, rowterm, cfg.M, dtype=torch.bfloat16)      # bench dtype
        torch.cuda.synchronize()
        yrows = y[tsd].float().cpu().numpy().astype(np.float64)
        del y, lin
        tol = tol_of(Y) + np.abs(Y) * 2.0 ** -7                  # 1e-3 (row rms from the oracle) + one bf16 step
        err = np.abs(yrows - Y)
        print("configs[%d] %s %dx%dx%d: %d tokens x %d outputs, max err/tol %.3f" % (
            ci, name, cfg.M, N, spec.d, int(ok.sum()), N, float((err / tol)[ok].max())))
        assert (err[ok] <= tol[ok]).all()


def test_chained_ffn_with_output_reorder(rp):
    """LN -> fc1 (rows permuted by fc2's reorder index) -> ReLU + quantize -> fc2."""
    d, dff, M, bits, g = 256, 1024, 200, 4, 8
    seed = 77
    site = w.make_site(seed, d, M, 4, 64)
    W1 = w.weight_matrix(seed + 1, dff, d)
    W2 = w.weight_matrix(seed + 2, d, dff)
    # oracle pass 1: site 1
    c1 = o.calibrate(site.cal, site.gamma, site.beta, EPS, False, g, bits, seed=seed)
    # calibration of the ReLU site runs on the unquantized model
    def fp_hidden(x):
        y, _ = o.layernorm_f32(x, site.gamma, site.beta, EPS)
        return w.round_to_bf16((y.astype(np.float64) @ W1.astype(np.float64).T).astype(np.float32))
    hcal = [fp_hidden(b) for b in site.cal]
    c2 = o.calibrate(hcal, None, None, EPS, True, g, bits, seed=seed + 1)
    # device: calibrate both sites, fold fc1 with perm_out = site 2's reorder index
    gamma, beta = torch.from_numpy(site.gamma).cuda(), torch.from_numpy(site.beta).cuda()
    k1 = rp.calibrate_site([dev_bf16(b) for b in site.cal], gamma, beta, EPS, False, g, bits, seed=seed)
    k2 = rp.calibrate_site([dev_bf16(h) for h in hcal], None, None, EPS, True, g, bits, seed=seed + 1)
    assert np.array_equal(k1.perm, c1.perm) and np.array_equal(k2.perm, c2.perm) and np.array_equal(k2.z, c2.z)
    lin1 = rp.fold_linear(k1, torch.from_numpy(W1).cuda(), perm_out=k2.perm)
    # site 2's input arrives already in its cluster order: its own gather is the identity
    codes1, _, rt1 = rp.ln_quant(k1, dev_bf16(site.x), EPS)
    h = rp.cluster_gemm(k1, lin1, codes1, rt1, M, dtype=torch.bfloat16)            # [M, dff] in site-2 order
    # oracle for fc1 with permuted rows
    rc1, _, fr1 = o.ln_quant(site.x, site.gamma, site.beta, EPS, False, c1.perm, c1.cluster_off, c1.inv_s, c1.z, bits)
    wq1, sW1, _, zW1 = o.quantize_weights(W1, c1.perm, c2.perm)
    _, _, H = o.cluster_gemm_int(rc1, wq1, c1.cluster_off, c1.s, c1.z, sW1, zW1)
    hd = h.float().cpu().numpy().astype(np.float64)
    ok = ~fr1
    assert (np.abs(hd - H)[ok] <= (tol_of(H) + np.abs(H) * 2.0 ** -7)[ok]).all()
    # stage 2 on identical inputs: the oracle's hidden tensor, rounded to bf16, goes to both sides
    # (the device's own h agrees with it only to the product's tolerance, and a code may flip on that)
    h32 = w.round_to_bf16(H.astype(np.float32))
    ident = rp.identity_site(k2)
    codes2, _, rt2 = rp.ln_quant(ident, dev_bf16(h32), EPS, relu=True)
    got2 = torch.empty((M, dff), dtype=torch.int8, device="cuda")
    rp.rptq_unpack_codes(codes2, M, k2.cluster_off, bits, got2)
    rc2, _, _ = o.ln_quant(h32, None, None, EPS, True, None, c2.cluster_off, c2.inv_s, c2.z, bits)
    assert np.array_equal(got2.cpu().numpy(), rc2)
    lin2 = rp.fold_linear(k2, torch.from_numpy(W2).cuda())
    y = rp.cluster_gemm(k2, lin2, codes2, rt2, M, dtype=torch.float32)
    wq2, sW2, _, zW2 = o.quantize_weights(W2, c2.perm)
    _, _, Y = o.cluster_gemm_int(rc2, wq2, c2.cluster_off, c2.s, c2.z, sW2, zW2)
    assert (np.abs(y.cpu().numpy().astype(np.float64) - Y) <= tol_of(Y)).all()
