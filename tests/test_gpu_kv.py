"""Key/value-cache codes and the shared query/key index on the HIP path against the oracle
(Sec. 4.2 last paragraph, Sec. 5.1): per-head clustering bit for bit, cache codes bit for bit
(decoded with the test-side codec of the documented formats), read-back bit for bit."""
import numpy as np
import pytest

import workloads as w
from oracle import kv_cache as kvo
from oracle import rptq_oracle as o

import packfmt

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def rp():
    import paper_2304_01089_amd as rp_
    rp_.load_library()
    assert torch.cuda.is_available()
    return rp_


def dev_bf16(x):
    return torch.from_numpy(w.bf16_bits(x).view(np.int16)).cuda().view(torch.bfloat16)


def qk_tensors(seed, T, H, dh):
    """Synthetic query / key activations with the per-channel range structure of the site model."""
    rng = np.random.default_rng(seed)
    D = H * dh
    sc = np.exp(rng.normal(0, 1, D))
    sc[rng.choice(D, max(1, D // 100), replace=False)] *= 30.0
    q = w.round_to_bf16((rng.normal(0, 2 * sc) + sc * rng.standard_normal((T, D))).astype(np.float32))
    k = w.round_to_bf16((rng.normal(0, 2 * sc) + 0.5 * sc * rng.standard_normal((T, D))).astype(np.float32))
    return q, k


def minmax(x):
    return (x.min(axis=0) + np.float32(0)).astype(np.float32), (x.max(axis=0) + np.float32(0)).astype(np.float32)


CASES = [
    ("opt_heads_a4", 300, 12, 128, 4, 4),        # 1.5 wave tiles per row (ragged tile), several rows per wave
    ("opt_heads_a3", 130, 8, 128, 3, 4),
    ("small_heads_a4", 70, 5, 64, 4, 4),         # d = 320: one partial tile
    ("a8", 33, 4, 128, 8, 4),
    ("one_row_a3", 1, 16, 64, 3, 3),
    ("whole_tile_heads", 20, 3, 1024, 4, 8),     # a head as wide as a wave tile
]


@pytest.mark.parametrize("name,T,H,dh,bits,g", CASES)
def test_cache_codes_and_read_back_bit_exact(rp, name, T, H, dh, bits, g):
    seed = 7000 + sum(map(ord, name))
    q, k = qk_tensors(seed, T, H, dh)
    d = H * dh
    qmin, qmax = minmax(q)
    kmin, kmax = minmax(k)
    ref = kvo.cluster_heads([qmin, kmin], [qmax, kmax], H, g, bits, seed)
    got = rp.rptq_cluster_heads([qmin, kmin], [qmax, kmax], H, g, bits, seed)
    for key in ("assign", "perm", "cluster_off", "g_eff", "s", "inv_s", "z"):
        assert np.array_equal(got[key], getattr(ref, key)), key

    for tensor, x in ((0, q), (1, k)):               # queries are quantized the same way when a scheme asks for it
        table = torch.empty(rp.rptq_kv_table_bytes(d), dtype=torch.uint8, device="cuda")
        rp.rptq_kv_tables(got["perm"], got["cluster_off"], got["s"][tensor], got["inv_s"][tensor], got["z"][tensor],
                          d, H, g, table)
        codes = torch.full((T * d * bits // 8,), 0xA5, dtype=torch.uint8, device="cuda")
        rp.rptq_kv_quant(dev_bf16(x), T, d, table, bits, codes)
        torch.cuda.synchronize()
        dec = packfmt.unpack_groups(codes.cpu().numpy().reshape(T, -1), d, bits)
        want = kvo.kv_quant(x, ref, tensor, bits)
        assert np.array_equal(dec, want)

        # read-back: oracle-made codes, packed by the test-side encoder
        packed = torch.from_numpy(packfmt.pack_groups(want, bits).reshape(-1)).cuda()
        out = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
        rp.rptq_kv_dequant(packed, T, d, table, bits, out)
        torch.cuda.synchronize()
        back = kvo.kv_dequant(want, ref, tensor)
        assert np.array_equal(out.float().cpu().numpy(), back)


def test_value_cache_alone_uses_two_number_points(rp):
    _, v = qk_tensors(11, 64, 6, 128)
    vmin, vmax = minmax(v)
    ref = kvo.cluster_heads([vmin], [vmax], 6, 4, 4, 3)
    got = rp.rptq_cluster_heads([vmin], [vmax], 6, 4, 4, 3)
    for key in ("assign", "perm", "cluster_off", "g_eff", "s", "inv_s", "z"):
        assert np.array_equal(got[key], getattr(ref, key)), key


def test_full_width_cache_sampled(rp):
    """The width of an OPT-175b layer's cache (96 heads x 128) at 8192 tokens, 3 bits: sampled rows."""
    T, H, dh, bits, g = 8192, 96, 128, 3, 4
    d = H * dh
    q, k = qk_tensors(99, 256, H, dh)
    kmin, kmax = minmax(k)
    qmin, qmax = minmax(q)
    ref = kvo.cluster_heads([qmin, kmin], [qmax, kmax], H, g, bits, 5)
    got = rp.rptq_cluster_heads([qmin, kmin], [qmax, kmax], H, g, bits, 5)
    assert np.array_equal(got["perm"], ref.perm) and np.array_equal(got["z"], ref.z)
    table = torch.empty(rp.rptq_kv_table_bytes(d), dtype=torch.uint8, device="cuda")
    rp.rptq_kv_tables(got["perm"], got["cluster_off"], got["s"][1], got["inv_s"][1], got["z"][1], d, H, g, table)
    x = dev_bf16(k).repeat(T // 256, 1).contiguous()
    codes = torch.empty(T * d * bits // 8, dtype=torch.uint8, device="cuda")
    rp.rptq_kv_quant(x, T, d, table, bits, codes)
    out = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
    rp.rptq_kv_dequant(codes, T, d, table, bits, out)
    torch.cuda.synchronize()
    rng = np.random.default_rng(1)
    ts = np.unique(np.concatenate([[0, T - 1], rng.integers(0, T, 30)]))
    want = kvo.kv_quant(k[ts % 256], ref, 1, bits)
    dec = packfmt.unpack_groups(codes.view(T, -1)[torch.from_numpy(ts).cuda()].cpu().numpy(), d, bits)
    assert np.array_equal(dec, want)
    assert np.array_equal(out[torch.from_numpy(ts).cuda()].float().cpu().numpy(), kvo.kv_dequant(want, ref, 1))
