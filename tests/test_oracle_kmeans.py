"""Pins for the oracle's K-Means, reorder index and per-cluster parameters."""
import itertools

import numpy as np
import pytest

from conftest import read_golden
from oracle import rptq_oracle as o


def test_splitmix64_published_vectors():
    rows = read_golden("splitmix64.txt")
    gen = o.SplitMix64(int(rows[0][0]))
    for seed, idx, val in rows:
        assert gen.next_u64() == int(val, 16)


def _sse(px, py, labels):
    tot = 0.0
    for l in set(labels.tolist()):
        m = labels == l
        tot += ((px[m] - px[m].mean()) ** 2 + (py[m] - py[m].mean()) ** 2).sum()
    return tot


def _brute_force_partition(px, py, g):
    """Optimal-SSE partition of C points into exactly g non-empty groups."""
    C = len(px)
    best, best_lab = None, None
    for lab in itertools.product(range(g), repeat=C):
        if len(set(lab)) != g:
            continue
        lab = np.array(lab)
        e = _sse(px, py, lab)
        if best is None or e < best - 1e-12:
            best, best_lab = e, lab
    return best_lab, best


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("g", [2, 3])
def test_matches_brute_force_on_separated_blobs(seed, g):
    rng = np.random.default_rng(100 + seed)
    centres = np.array([[-50.0, -40.0], [0.0, 5.0], [60.0, 90.0]])[:g]
    sizes = rng.multinomial(8 - g, np.ones(g) / g) + 1
    pts = np.concatenate([c + rng.normal(0, 0.5, (n, 2)) for c, n in zip(centres, sizes)])
    pts = pts[rng.permutation(len(pts))].astype(np.float32)
    px, py = pts[:, 0].astype(np.float64), pts[:, 1].astype(np.float64)
    raw, cen, _ = o.kmeans(pts[:, 0], pts[:, 1], g, seed=seed)
    got, g_eff = o.canonical_labels(raw)
    ref, _ = _brute_force_partition(px, py, g)
    ref, _ = o.canonical_labels(ref)
    assert g_eff == g
    assert np.array_equal(got, ref)


def _interval_dp(v, g):
    """Textbook optimal 1-D k-means: contiguous intervals of the sorted values."""
    v = np.sort(v)
    n = len(v)
    cost = np.zeros((n, n))
    for a in range(n):
        for b in range(a, n):
            seg = v[a:b + 1]
            cost[a, b] = ((seg - seg.mean()) ** 2).sum()
    D = np.full((g + 1, n + 1), np.inf)
    D[0, 0] = 0.0
    for j in range(1, g + 1):
        for e in range(1, n + 1):
            for st in range(j - 1, e):
                D[j, e] = min(D[j, e], D[j - 1, st] + cost[st, e - 1])
    return D[g, n]


def test_one_dimensional_case_reaches_interval_optimum():
    # a ReLU site: every channel minimum is 0, so the points lie on a line
    rng = np.random.default_rng(5)
    vmax = np.concatenate([rng.normal(1, 0.05, 7), rng.normal(10, 0.3, 6), rng.normal(40, 1.0, 5)]).astype(np.float32)
    vmax = vmax[rng.permutation(len(vmax))]
    vmin = np.zeros_like(vmax)
    raw, _, _ = o.kmeans(vmin, vmax, 3, seed=2)
    lab, g_eff = o.canonical_labels(raw)
    assert g_eff == 3
    got = _sse(vmin.astype(np.float64), vmax.astype(np.float64), lab)
    assert got <= _interval_dp(vmax.astype(np.float64), 3) * (1 + 1e-9) + 1e-12
    # clusters are contiguous intervals of the sorted values
    order = np.argsort(vmax)
    changes = (np.diff(lab[order]) != 0).sum()
    assert changes == 2


def _kmeans_python_loops(ch_min, ch_max, g, seed, max_iter=100):
    """The same rule with explicit sequential loops (pins numpy's cumsum/bincount order)."""
    px = [float(np.float32(v)) for v in ch_min]
    py = [float(np.float32(v)) for v in ch_max]
    C = len(px)
    rng = o.SplitMix64(seed)

    def sq(i, cx, cy):
        dx = px[i] - cx
        dy = py[i] - cy
        return dx * dx + dy * dy

    first = min(int(rng.uniform() * C), C - 1)
    cen = [(px[first], py[first])]
    d2 = [sq(i, *cen[0]) for i in range(C)]
    while len(cen) < g:
        cum, acc = [], 0.0
        for v in d2:
            acc = acc + v
            cum.append(acc)
        if not cum[-1] > 0.0:
            break
        target = rng.uniform() * cum[-1]
        nxt = C - 1
        for i in range(C):
            if cum[i] > target:
                nxt = i
                break
        cen.append((px[nxt], py[nxt]))
        d2 = [min(d2[i], sq(i, *cen[-1])) for i in range(C)]
    gk = len(cen)
    labels = [-1] * C

    def assign():
        out = []
        for i in range(C):
            best, bk = None, 0
            for kk in range(gk):
                dd = sq(i, *cen[kk])
                if best is None or dd < best:
                    best, bk = dd, kk
            out.append(bk)
        return out

    for _ in range(max_iter):
        new = assign()
        if new == labels:
            break
        labels = new
        cnt = [0] * gk
        sx = [0.0] * gk
        sy = [0.0] * gk
        for i in range(C):
            cnt[labels[i]] += 1
            sx[labels[i]] = sx[labels[i]] + px[i]
            sy[labels[i]] = sy[labels[i]] + py[i]
        for kk in range(gk):
            if cnt[kk] > 0:
                cen[kk] = (sx[kk] / cnt[kk], sy[kk] / cnt[kk])
        empties = [kk for kk in range(gk) if cnt[kk] == 0]
        if empties:
            own = [sq(i, *cen[labels[i]]) for i in range(C)]
            for kk in empties:
                far = max(range(C), key=lambda i: (own[i], -i))
                cen[kk] = (px[far], py[far])
                own[far] = -1.0
            labels = [-1] * C
    if -1 in labels:
        labels = assign()
    return np.array(labels), np.array(cen)


@pytest.mark.parametrize("seed,C,g", [(0, 40, 4), (1, 97, 8), (2, 64, 16), (3, 30, 30), (4, 50, 1)])
def test_numpy_and_loop_versions_agree_bit_for_bit(seed, C, g):
    rng = np.random.default_rng(seed)
    sc = np.exp(rng.normal(0, 1, C))
    mid = rng.normal(0, 2 * sc)
    cmin = (mid - 3 * sc).astype(np.float32)
    cmax = (mid + 3 * sc).astype(np.float32)
    raw, cen, _ = o.kmeans(cmin, cmax, g, seed=seed)
    lab2, cen2 = _kmeans_python_loops(cmin, cmax, g, seed)
    assert np.array_equal(raw, lab2)
    assert np.array_equal(cen, cen2)


def test_lloyd_fixed_point_invariants():
    rng = np.random.default_rng(12)
    C, g = 300, 8
    cmin = rng.normal(-2, 3, C).astype(np.float32)
    cmax = (cmin + np.abs(rng.normal(4, 3, C))).astype(np.float32)
    raw, cen, n_iter = o.kmeans(cmin, cmax, g, seed=9)
    assert n_iter < 100
    px, py = cmin.astype(np.float64), cmax.astype(np.float64)
    d = (px[:, None] - cen[None, :, 0]) ** 2 + (py[:, None] - cen[None, :, 1]) ** 2
    assert np.array_equal(np.argmin(d, axis=1), raw)            # every point nearest its own centre
    for kk in range(g):                                         # every centre is its members' mean
        m = raw == kk
        assert m.any()
        assert np.allclose(cen[kk], [px[m].mean(), py[m].mean()], rtol=1e-12, atol=1e-12)


def test_duplicate_points_give_fewer_clusters():
    cmin = np.array([0, 0, 0, 1, 1, 1], dtype=np.float32)
    cmax = np.array([2, 2, 2, 5, 5, 5], dtype=np.float32)
    raw, cen, _ = o.kmeans(cmin, cmax, 4, seed=3)
    lab, g_eff = o.canonical_labels(raw)
    assert g_eff == 2
    assert lab.tolist() == [0, 0, 0, 1, 1, 1]


def test_canonical_labels_and_reorder_index():
    raw = np.array([5, 2, 5, 7, 2, 2, 7, 5])
    lab, g_eff = o.canonical_labels(raw)
    assert g_eff == 3 and lab.tolist() == [0, 1, 0, 2, 1, 1, 2, 0]
    perm, off = o.reorder_index(lab, g_eff)
    assert perm.tolist() == [0, 2, 7, 1, 4, 5, 3, 6]             # S = [S^1, S^2, S^3]
    assert off.tolist() == [0, 3, 6, 8]
    assert sorted(perm.tolist()) == list(range(8))              # union of the S^i is every channel


def test_cluster_params_special_cases():
    rng = np.random.default_rng(4)
    C = 12
    cmin = rng.normal(-1, 1, C).astype(np.float32)
    cmax = (cmin + 1 + rng.random(C)).astype(np.float32)
    # one cluster: per-tensor Eq. 2
    perm, off = o.reorder_index(np.zeros(C, int), 1)
    s, inv, z, lo, hi = o.cluster_params(cmin, cmax, perm, off, 4)
    s1, inv1, z1 = o.minmax_params(cmin.min(), cmax.max(), 4)
    assert float(s[0]) == float(s1) and int(z[0]) == int(z1)
    # one cluster per channel: per-channel Eq. 2
    perm, off = o.reorder_index(np.arange(C), C)
    s, inv, z, lo, hi = o.cluster_params(cmin, cmax, perm, off, 4)
    sc, invc, zc = o.minmax_params(cmin, cmax, 4)
    assert np.array_equal(s, sc) and np.array_equal(z, zc) and np.array_equal(perm, np.arange(C))


# ---------------------------------------------------------------------------
# kmeans_points: the same rule in any dimension (the shared query/key index, Sec. 4.2)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("seed,C,g", [(0, 40, 4), (1, 97, 8), (2, 64, 16), (4, 50, 1), (5, 33, 33)])
def test_points_version_equals_the_two_dimensional_one_bit_for_bit(seed, C, g):
    rng = np.random.default_rng(seed)
    sc = np.exp(rng.normal(0, 1, C))
    mid = rng.normal(0, 2 * sc)
    cmin = (mid - 3 * sc).astype(np.float32)
    cmax = (mid + 3 * sc).astype(np.float32)
    raw, cen, n_it = o.kmeans(cmin, cmax, g, seed=seed)
    raw2, cen2, n_it2 = o.kmeans_points(np.stack([cmin, cmax], axis=1), g, seed=seed)
    assert np.array_equal(raw, raw2) and np.array_equal(cen, cen2) and n_it == n_it2


def _sse_nd(P, labels):
    return sum((((P[labels == l] - P[labels == l].mean(axis=0)) ** 2).sum()) for l in set(labels.tolist()))


@pytest.mark.parametrize("seed", range(5))
@pytest.mark.parametrize("g", [2, 3])
def test_points_version_matches_brute_force_in_four_dimensions(seed, g):
    rng = np.random.default_rng(300 + seed)
    centres = np.array([[-50.0, -60.0, 5.0, -4.0], [0.0, -5.0, 40.0, 20.0], [60.0, 30.0, -30.0, -45.0]])[:g]
    sizes = rng.multinomial(8 - g, np.ones(g) / g) + 1
    pts = np.concatenate([c + rng.normal(0, 0.5, (n, 4)) for c, n in zip(centres, sizes)])
    pts = pts[rng.permutation(len(pts))].astype(np.float32)
    raw, cen, _ = o.kmeans_points(pts, g, seed=seed)
    got, g_eff = o.canonical_labels(raw)
    P = pts.astype(np.float64)
    best, best_lab = None, None
    for lab in itertools.product(range(g), repeat=len(P)):
        if len(set(lab)) != g:
            continue
        lab = np.array(lab)
        e = _sse_nd(P, lab)
        if best is None or e < best - 1e-12:
            best, best_lab = e, lab
    ref, _ = o.canonical_labels(best_lab)
    assert g_eff == g and np.array_equal(got, ref)


def test_points_version_python_loops_bit_for_bit():
    """Sequential float64 loops in four dimensions (pins the order of the distance terms and of the member sums)."""
    rng = np.random.default_rng(77)
    C, g, seed, D = 60, 5, 11, 4
    pts = (rng.normal(0, 3, (C, D)) * np.exp(rng.normal(0, 1, (C, 1)))).astype(np.float32)
    raw, cen, _ = o.kmeans_points(pts, g, seed=seed)
    P = [[float(v) for v in row] for row in pts]
    gen = o.SplitMix64(seed)

    def sq(i, c):
        acc = None
        for j in range(D):
            dj = P[i][j] - c[j]
            t = dj * dj
            acc = t if acc is None else acc + t
        return acc
    first = min(int(gen.uniform() * C), C - 1)
    cs = [list(P[first])]
    d2 = [sq(i, cs[0]) for i in range(C)]
    while len(cs) < g:
        acc, cum = 0.0, []
        for v in d2:
            acc = acc + v
            cum.append(acc)
        target = gen.uniform() * cum[-1]
        nxt = next((i for i in range(C) if cum[i] > target), C - 1)
        cs.append(list(P[nxt]))
        d2 = [min(d2[i], sq(i, cs[-1])) for i in range(C)]
    labels = [-1] * C
    for _ in range(100):
        new = []
        for i in range(C):
            best, bk = None, 0
            for kk in range(g):
                dd = sq(i, cs[kk])
                if best is None or dd < best:
                    best, bk = dd, kk
            new.append(bk)
        if new == labels:
            break
        labels = new
        for kk in range(g):
            mem = [i for i in range(C) if labels[i] == kk]
            assert mem                                           # (no empty cluster on this input)
            for j in range(D):
                acc = 0.0
                for i in mem:
                    acc = acc + P[i][j]
                cs[kk][j] = acc / len(mem)
    assert labels == raw.tolist()
    assert np.array_equal(np.array(cs), cen)


def test_points_version_lloyd_invariants():
    rng = np.random.default_rng(8)
    pts = rng.normal(0, 2, (200, 4)).astype(np.float32)
    raw, cen, n_iter = o.kmeans_points(pts, 6, seed=4)
    P = pts.astype(np.float64)
    d = ((P[:, None, :] - cen[None, :, :]) ** 2).sum(axis=2)
    assert n_iter < 100 and np.array_equal(np.argmin(d, axis=1), raw)
    for kk in range(6):
        assert np.allclose(cen[kk], P[raw == kk].mean(axis=0), rtol=1e-12, atol=1e-12)
