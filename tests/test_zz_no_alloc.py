"""rptq_cluster_gemm_quant_static (the entry point for callers that cannot allocate) against
rptq_cluster_gemm_quant on the same inputs: identical codes and row sums, on two calls in a
row, the second with a smaller input (the scratch array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest

import workloads as w
from oracle import rptq_oracle as o

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")
EPS = 1e-5


def dev_bf16(x):
    return torch.from_numpy(w.bf16_bits(x).view(np.int16)).cuda().view(torch.bfloat16)


def test_static_scratch_entry_point_matches_the_workspace_one():
    import paper_2304_01089_amd as rp
    rp.load_library()
    assert torch.cuda.is_available()
    d, dff, M, bits, g, seed = 256, 1504, 333, 4, 8, 1207
    site = w.make_site(seed, d, M, 3, 64)
    W1 = w.weight_matrix(seed + 1, dff, d)

    def fp_hidden(x):
        y, _ = o.layernorm_f32(x, site.gamma, site.beta, EPS)
        return w.round_to_bf16(y @ W1.T)
    gamma, beta = torch.from_numpy(site.gamma).cuda(), torch.from_numpy(site.beta).cuda()
    k1 = rp.calibrate_site([dev_bf16(b) for b in site.cal], gamma, beta, EPS, False, g, bits, seed=seed)
    k2 = rp.calibrate_site([dev_bf16(fp_hidden(b)) for b in site.cal], None, None, EPS, True, g, 3, seed=seed + 1)
    lin1 = rp.fold_linear(k1, torch.from_numpy(W1).cuda(), next_site=k2)
    codes1, _, rt1 = rp.ln_quant(k1, dev_bf16(site.x), EPS)

    def both(rows):
        """The two entry points on the first `rows` tokens."""
        outs = []
        for static in (False, True):
            codes2 = torch.full((rp.rptq_codes_bytes(rows, k2.k_padded, k2.bits),), 0x5A, dtype=torch.uint8, device="cuda")
            rt2 = torch.full((rows,), float("nan"), dtype=torch.float32, device="cuda")
            args = (codes1, rows, bits, lin1.Wq, lin1.N, k1.cluster_off, k1.s, lin1.sW, lin1.zW, lin1.colterm, rt1, True,
                    k2.cluster_off, k2.s, k2.inv_s, k2.z, k2.bits, codes2, rt2)
            if static:
                rp.rptq_cluster_gemm_quant_static(*args)
            else:
                ws = torch.empty(rp.rptq_cluster_gemm_quant_workspace_bytes(rows, lin1.N), dtype=torch.uint8, device="cuda")
                rp.rptq_cluster_gemm_quant(*args, ws)
            torch.cuda.synchronize()
            outs.append((codes2, rt2))
        return outs

    for rows in (M, 77):                                 # the second call is smaller: stale entries stay behind it
        (ca, ra), (cb, rb) = both(rows)
        assert torch.equal(ca, cb), rows
        assert torch.equal(ra, rb), rows                 # same kernels, same summation order: bit-equal
        assert torch.isfinite(rb).all()

    # a call that needs more than the array holds is refused before anything is launched
    lib = rp.load_library()
    need = rp.rptq_cluster_gemm_quant_workspace_bytes(1 << 20, lin1.N)
    assert need > (8 << 20)
    with pytest.raises(rp.RptqError) as e:
        rp.rptq_cluster_gemm_quant_static(codes1, 1 << 20, bits, lin1.Wq, lin1.N, k1.cluster_off, k1.s, lin1.sW, lin1.zW,
                                          lin1.colterm, rt1, True, k2.cluster_off, k2.s, k2.inv_s, k2.z, k2.bits,
                                          codes1, rt1)
    assert e.value.status == -7
