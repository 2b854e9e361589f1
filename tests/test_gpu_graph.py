"""The online entry points under HIP graph capture: they make no allocation, no
synchronization and no memset, so a recorded step must replay to exactly what the eager
calls give.  Replays are separated by eager work and synchronizations, and every replay
is checked."""
import numpy as np
import pytest

import workloads as w
from oracle import rptq_oracle as o

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")
EPS = 1e-5


def dev_bf16(x):
    return torch.from_numpy(w.bf16_bits(x).view(np.int16)).cuda().view(torch.bfloat16)


def test_recorded_step_replays_to_the_eager_result():
    import paper_2304_01089_amd as rp
    rp.load_library()
    d, dff, M, bits, g, seed = 256, 1024, 96, 4, 8, 909
    site = w.make_site(seed, d, M, 3, 64)
    W1 = w.weight_matrix(seed + 1, dff, d)
    W2 = w.weight_matrix(seed + 2, d, dff)

    def fp_hidden(x):
        y, _ = o.layernorm_f32(x, site.gamma, site.beta, EPS)
        return w.round_to_bf16(y @ W1.T)
    gamma, beta = torch.from_numpy(site.gamma).cuda(), torch.from_numpy(site.beta).cuda()
    k1 = rp.calibrate_site([dev_bf16(b) for b in site.cal], gamma, beta, EPS, False, g, bits, seed=seed)
    k2 = rp.calibrate_site([dev_bf16(fp_hidden(b)) for b in site.cal], None, None, EPS, True, g, bits, seed=seed + 1)
    lin1 = rp.fold_linear(k1, torch.from_numpy(W1).cuda(), next_site=k2)
    lin2 = rp.fold_linear(k2, torch.from_numpy(W2).cuda())

    x = dev_bf16(site.x).clone()
    codes1 = torch.empty(rp.rptq_codes_bytes(M, k1.k_padded, bits), dtype=torch.uint8, device="cuda")
    codes2 = torch.empty(rp.rptq_codes_bytes(M, k2.k_padded, bits), dtype=torch.uint8, device="cuda")
    rt1 = torch.empty(M, dtype=torch.float32, device="cuda")
    rt2 = torch.empty(M, dtype=torch.float32, device="cuda")
    ws = torch.empty(rp.rptq_cluster_gemm_quant_workspace_bytes(M, lin1.N), dtype=torch.uint8, device="cuda")
    y = torch.empty((M, d), dtype=torch.bfloat16, device="cuda")
    outs = (codes1, codes2, rt1, rt2, y)

    def step():
        rp.rptq_ln_quant(x, M, d, k1.gamma_pad, k1.beta_pad, EPS, False, k1.perm_pad, k1.cluster_off, k1.s, k1.inv_s,
                         k1.z, bits, codes1, None, rt1)
        rp.rptq_cluster_gemm_quant(codes1, M, bits, lin1.Wq, lin1.N, k1.cluster_off, k1.s, lin1.sW, lin1.zW,
                                   lin1.colterm, rt1, True, k2.cluster_off, k2.s, k2.inv_s, k2.z, bits, codes2, rt2, ws)
        rp.rptq_cluster_gemm(codes2, M, bits, lin2.Wq, d, k2.cluster_off, k2.s, lin2.sW, lin2.zW, lin2.colterm, rt2, y)

    step()                                    # eager first: one-time driver set-up happens outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for k in range(1, 4):
        x.copy_(dev_bf16(w.extra_batch(site, k, M)))
        graph.replay()
        torch.cuda.synchronize()
        replayed = [t.clone() for t in outs]
        for t in outs:                        # eager work between replays
            t.zero_()
        step()
        torch.cuda.synchronize()
        for a, b in zip(replayed, outs):
            assert torch.equal(a, b)
        assert y.float().abs().sum().item() > 0
