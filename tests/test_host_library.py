"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, its
host logic (sizes, validation, clustering) agrees with the oracle, and the packed-layout
codec used by the GPU tests round-trips.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2304_01089_amd as rp
import workloads as w
from oracle import rptq_oracle as o

import packfmt

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(rp.library_path()):
        from paper_2304_01089_amd.build import build_library
        build_library()
    return rp.load_library()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "rptq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(rptq_[a-z_0-9]+)\s*\(", header))
    assert declared == set(rp.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name
    assert rp.rptq_version().startswith("rptq-gfx950")


def test_size_queries():
    assert rp.rptq_padded_k([0, 5, 40, 100]) == 256            # 32 + 64 + 64 = 160 -> 256
    assert rp.rptq_padded_k([0, 128]) == 256
    assert rp.rptq_padded_k([0, 129]) == 256
    assert rp.rptq_codes_bytes(10, 256, 4) == 10 * 128
    assert rp.rptq_codes_bytes(10, 256, 3) == 10 * 96
    assert rp.rptq_codes_bytes(10, 256, 8) == 10 * 256
    assert rp.rptq_codes_bytes(10, 256, 5) == 0
    assert rp.rptq_weight_bytes(300, 256) == 512 * 128
    assert rp.rptq_calibrate_workspace_bytes(768) == 768 * 16
    for off in ([0, 5, 40, 100], [0, 1, 2, 3, 700], [0, 33]):
        assert rp.rptq_padded_k(off) == packfmt.padded_layout(off)[1]


def test_validation_happens_before_any_device_work(lib):
    with pytest.raises(rp.RptqError) as e:
        rp.rptq_padded_k([0, 5, 5, 9])                          # not strictly increasing
    assert e.value.status == -5
    with pytest.raises(rp.RptqError) as e:
        rp.rptq_padded_k([1, 5])
    assert e.value.status == -5
    with pytest.raises(rp.RptqError) as e:
        rp.rptq_padded_k(list(range(0, 66 * 4, 4)))             # 65 clusters
    assert e.value.status == -2
    # NULL pointers and bad bits are refused by the entry points themselves
    i32, vp = ctypes.c_int32, ctypes.c_void_p
    off = (i32 * 2)(0, 64)
    one = (ctypes.c_float * 1)(1.0)
    zero = (i32 * 1)(0)
    dummy = vp(4096)
    assert lib.rptq_ln_quant(None, 4, 64, None, None, 1e-5, 0, dummy, off, 1, one, one, zero, 4, dummy, None, None, None) == -1
    assert lib.rptq_ln_quant(dummy, 4, 64, None, None, 1e-5, 0, dummy, off, 1, one, one, zero, 5, dummy, None, None, None) == -3
    assert lib.rptq_ln_quant(dummy, 4, 72, None, None, 1e-5, 0, dummy, off, 1, one, one, zero, 4, dummy, None, None, None) == -2
    assert lib.rptq_ln_quant(vp(4100), 4, 64, None, None, 1e-5, 0, dummy, off, 1, one, one, zero, 4, dummy, None, None, None) == -4
    big = (i32 * 1)(1 << 22)
    assert lib.rptq_ln_quant(dummy, 4, 64, None, None, 1e-5, 0, dummy, off, 1, one, one, big, 4, dummy, None, None, None) == -6
    # a LayerNorm row wider than one workgroup covers (K_p > 15360) is refused before any launch
    wide = (i32 * 2)(0, 16384)
    assert lib.rptq_ln_quant(dummy, 4, 16384, dummy, dummy, 1e-5, 0, dummy, wide, 1, one, one, zero, 4, dummy, None, None, None) == -2
    assert lib.rptq_cluster_gemm(dummy, 4, 4, dummy, 8, off, 1, one, dummy, dummy, dummy, None, dummy, 1, None) == -1
    assert lib.rptq_cluster_gemm(dummy, 4, 4, dummy, 0, off, 1, one, dummy, dummy, dummy, dummy, dummy, 1, None) == -2
    # the quantizing output stage: code widths as everywhere, the product's width must be the
    # next site's padded width, the workspace must be large enough
    off256 = (i32 * 2)(0, 256)
    gq = lambda N, nb, ws: lib.rptq_cluster_gemm_quant(dummy, 4, 4, dummy, N, off, 1, one, dummy, dummy, dummy, dummy, 1,
                                                      off256, 1, one, one, zero, nb, dummy, dummy, dummy, ws, None)
    assert gq(256, 5, 1 << 20) == -3
    assert gq(512, 4, 1 << 20) == -2
    assert gq(256, 4, 8) == -7
    assert rp.rptq_cluster_gemm_quant_workspace_bytes(100, 256) == 2 * 100 * 8
    perm = (i32 * 4)(0, 1, 1, 3)
    off4 = (i32 * 2)(0, 4)
    assert lib.rptq_fold_reorder(None, None, 4, perm, off4, 1, None, None, None, 0, 0, 0, 4, None,
                                 dummy, None, None, None, None, None, None, None, None) == -5
    assert b"permutation" in lib.rptq_strerror(-5)


def test_fold_reorder_validates_its_index_arrays_on_the_host(lib):
    """Both index arrays are host arrays: a bad entry is refused before any device work, so an
    out-of-range source row or channel can never reach a kernel."""
    i32, vp, f32 = ctypes.c_int32, ctypes.c_void_p, ctypes.c_float
    dummy = vp(4096)
    K, N, rows = 64, 8, 8
    off = (i32 * 2)(0, K)
    sx, zx = (f32 * 1)(0.5), (i32 * 1)(3)
    ident = (i32 * K)(*range(K))

    def fold(perm_in=ident, perm_out=None, n=N, w_rows=rows, sx=sx, zx=zx, W=dummy, w_dtype=1):
        return lib.rptq_fold_reorder(None, None, K, perm_in, off, 1, sx, zx, W, w_dtype, w_rows, n, K, perm_out,
                                     dummy, None, None, dummy, dummy, dummy, dummy, dummy, None)
    bad = list(range(K)); bad[5] = K
    assert fold(perm_in=(i32 * K)(*bad)) == -5                      # channel index out of range
    bad[5] = -1
    assert fold(perm_in=(i32 * K)(*bad)) == -5
    bad[5] = 6
    assert fold(perm_in=(i32 * K)(*bad)) == -5                      # a channel twice
    assert fold(perm_out=(i32 * N)(0, 1, 2, 3, 4, 5, rows, 0)) == -5    # source row beyond W
    assert fold(perm_out=(i32 * N)(0, 1, 2, 3, 4, 5, -2, 0)) == -5      # only -1 marks a pad row
    assert fold(n=N + 1, w_rows=rows, perm_out=None) == -2              # no output index: N rows of W must exist
    assert fold(w_rows=0) == -2
    assert fold(w_dtype=7) == -2
    assert fold(sx=(f32 * 1)(float("nan"))) == -6
    assert fold(zx=(i32 * 1)(1 << 22)) == -6
    assert fold(perm_in=None) == -1
    # a misaligned device pointer is the first thing checked after the host arrays
    assert lib.rptq_fold_reorder(None, None, K, ident, off, 1, sx, zx, vp(4100), 1, rows, N, K, None,
                                 dummy, None, None, dummy, dummy, dummy, dummy, dummy, None) == -4


def test_accumulator_headroom_bound_is_declared_and_enforced(lib):
    """The product kernels never clear their int32 accumulators: |sum| <= 2^14 * K_p.  The header
    states the bound K_p <= RPTQ_MAX_K_PADDED and every cluster table is checked against it."""
    header = open(os.path.join(ROOT, "include", "rptq.h")).read()
    max_kp = int(re.search(r"#define RPTQ_MAX_K_PADDED (\d+)", header).group(1))
    max_ch = int(re.search(r"#define RPTQ_MAX_CHANNELS (\d+)", header).group(1))
    max_g = int(re.search(r"#define RPTQ_MAX_CLUSTERS (\d+)", header).group(1))
    assert (1 << 14) * max_kp <= 1 << 30
    # the widest table the other limits admit still fits
    worst = max_ch + max_g * 31
    assert (worst + 255) // 256 * 256 <= max_kp
    off = np.concatenate([[0], np.arange(1, max_g) * 33, [max_ch]]).astype(np.int32)
    assert rp.rptq_padded_k(off) <= max_kp
    with pytest.raises(rp.RptqError) as e:
        rp.rptq_padded_k([0, max_ch + 1])
    assert e.value.status == -2
    assert b"capture" in lib.rptq_strerror(-9)


@pytest.mark.parametrize("cfg,g,bits,seed", [(0, 8, 8, 1), (0, 16, 4, 2), (0, 32, 3, 3), (0, 1, 4, 0)])
def test_host_clustering_matches_oracle(cfg, g, bits, seed):
    c = w.CONFIGS[cfg]
    s = w.make_site(w.site_seed(cfg, 0), c.sites[0].d, 8, c.n_cal)
    cmin, cmax = o.calibrate_minmax(s.cal, s.gamma, s.beta)
    raw, _, _ = o.kmeans(cmin, cmax, g, seed)
    assign, ge = o.canonical_labels(raw)
    perm, off = o.reorder_index(assign, ge)
    ss, inv, z, _, _ = o.cluster_params(cmin, cmax, perm, off, bits)
    r = rp.rptq_cluster_channels(cmin, cmax, g, bits, seed)
    assert r["g_eff"] == ge
    for key, ref in (("assign", assign), ("perm", perm), ("cluster_off", off), ("s", ss), ("inv_s", inv), ("z", z)):
        assert np.array_equal(r[key], ref), key


def test_host_clustering_degenerate_points():
    cmin = np.array([0, 0, 0, 1, 1, 1, 0, 1], dtype=np.float32)
    cmax = np.array([2, 2, 2, 5, 5, 5, 2, 5], dtype=np.float32)
    r = rp.rptq_cluster_channels(cmin, cmax, 4, 4, 3)
    raw, _, _ = o.kmeans(cmin, cmax, 4, 3)
    assign, ge = o.canonical_labels(raw)
    assert r["g_eff"] == ge == 2 and np.array_equal(r["assign"], assign)


@pytest.mark.parametrize("bits", [3, 4, 8])
def test_packed_code_codec_round_trip(bits):
    rng = np.random.default_rng(bits)
    off = np.array([0, 5, 70, 71, 200])
    lo, hi = o.code_range(bits)
    codes = rng.integers(lo, hi + 1, (7, 200))
    packed = packfmt.pack_codes(codes, off, bits)
    assert packed.shape == (7, rp.rptq_codes_bytes(7, rp.rptq_padded_k(off), bits) // 7)
    back, pads = packfmt.unpack_codes(packed, off, bits)
    assert np.array_equal(back, codes) and (pads == 0).all()


def test_packed_weight_codec_round_trip():
    rng = np.random.default_rng(0)
    off = np.array([0, 31, 64, 130])
    wq = rng.integers(-8, 8, (70, 130))
    packed = packfmt.pack_weights(wq, off)
    assert packed.size == rp.rptq_weight_bytes(70, rp.rptq_padded_k(off))
    back, extra = packfmt.unpack_weights(packed, 70, off)
    assert np.array_equal(back, wq) and (extra == 0).all()


def test_head_clustering_matches_oracle_and_tables_are_validated(lib):
    from oracle import kv_cache as kvo
    rng = np.random.default_rng(3)
    H, dh, g, bits = 5, 32, 4, 4
    d = H * dh
    qmin = rng.normal(-3, 2, d).astype(np.float32)
    qmax = (qmin + np.abs(rng.normal(4, 3, d))).astype(np.float32)
    kmin = rng.normal(-1, 1, d).astype(np.float32)
    kmax = (kmin + np.abs(rng.normal(2, 1, d))).astype(np.float32)
    ref = kvo.cluster_heads([qmin, kmin], [qmax, kmax], H, g, bits, 17)
    got = rp.rptq_cluster_heads([qmin, kmin], [qmax, kmax], H, g, bits, 17)
    for key in ("assign", "perm", "cluster_off", "g_eff", "s", "inv_s", "z"):
        assert np.array_equal(got[key], getattr(ref, key)), key
    ref1 = kvo.cluster_heads([kmin], [kmax], H, g, 3, 2)
    got1 = rp.rptq_cluster_heads([kmin], [kmax], H, g, 3, 2)
    for key in ("assign", "perm", "cluster_off", "s", "z"):
        assert np.array_equal(got1[key], getattr(ref1, key)), key
    # table construction refuses what the kernels could not survive, before any device work
    i32, vp, f32 = ctypes.c_int32, ctypes.c_void_p, ctypes.c_float
    dummy = vp(4096)

    def tables(perm=got["perm"], off=got["cluster_off"], s=got["s"][1], z=got["z"][1], d_=d, heads=H):
        pa = np.ascontiguousarray(perm, np.int32)
        oa = np.ascontiguousarray(off, np.int32)
        sa = np.ascontiguousarray(s, np.float32)
        za = np.ascontiguousarray(z, np.int32)
        return lib.rptq_kv_tables(pa.ctypes.data_as(vp), oa.ctypes.data_as(vp), sa.ctypes.data_as(vp),
                                  sa.ctypes.data_as(vp), za.ctypes.data_as(vp), d_, heads, g, dummy, None)
    bad = got["perm"].copy()
    bad[0], bad[dh] = bad[dh], bad[0]                          # two channels swap heads
    assert tables(perm=bad) == -5
    bad = got["perm"].copy()
    bad[3] = bad[4]
    assert tables(perm=bad) == -5                              # not a permutation
    off = got["cluster_off"].copy()
    off[2, g] = dh - 1
    assert tables(off=off) == -5                               # a head's offsets must end at its width
    sb = got["s"][1].copy()
    sb[0, 0] = np.nan
    assert tables(s=sb) == -6
    assert tables(d_=d + 8) == -2
    assert lib.rptq_kv_quant(dummy, 4, d, dummy, 5, dummy, None) == -3
    assert lib.rptq_kv_dequant(dummy, 4, d + 8, dummy, 4, dummy, None) == -2
    assert lib.rptq_kv_quant(None, 4, d, dummy, 4, dummy, None) == -1


def test_first_method_entry_points_validate_on_the_host(lib):
    """rptq_gemm_bf16 / rptq_dequant_* refuse bad shapes and null pointers before any HIP call."""
    import ctypes
    fake = ctypes.c_void_p(4096)                       # an aligned non-null address: never dereferenced
    off = (ctypes.c_int32 * 3)(0, 40, 64)
    sx = (ctypes.c_float * 2)(0.5, 0.25)
    zx = (ctypes.c_int32 * 2)(1, -2)
    assert lib.rptq_gemm_bf16(fake, fake, 8, 8, 200, fake, rp.DTYPE_F32, None) == -2       # K not a multiple of 64
    assert lib.rptq_gemm_bf16(fake, fake, 8, 6, 256, fake, rp.DTYPE_F32, None) == -2       # N not a multiple of 4
    assert lib.rptq_gemm_bf16(fake, fake, 8, 8, 256, fake, 7, None) == -2                  # unknown output type
    assert lib.rptq_gemm_bf16(None, fake, 8, 8, 256, fake, rp.DTYPE_F32, None) == -1
    assert lib.rptq_dequant_codes(fake, 4, 5, off, 2, sx, zx, fake, None) == -3            # bits
    assert lib.rptq_dequant_codes(fake, -1, 4, off, 2, sx, zx, fake, None) == -2
    bad = (ctypes.c_float * 2)(0.5, float("nan"))
    assert lib.rptq_dequant_codes(fake, 4, 4, off, 2, bad, zx, fake, None) == -6           # scale not finite
    assert lib.rptq_dequant_weights(fake, 0, off, 2, fake, fake, fake, None) == -2
    assert lib.rptq_dequant_weights(None, 4, off, 2, fake, fake, fake, None) == -1
