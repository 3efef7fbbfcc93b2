"""Pins of the oracle's per-layer statistics and bit-width assigners (paper Sec. "Layer-wise
Adaptive Quantization", problem definition and Algorithm 1)."""
import math

import numpy as np
import pytest

from oracle import adaptive
from paper_2111_08617_amd import workloads as wl


# ---------------------------------------------------------------- statistics

def test_sqnorms_closed_forms_and_exact_sum(oracle):
    rng = np.random.default_rng(1)
    off = np.array([0, 5, 5, 1005, 5000], np.int64)
    x = rng.standard_normal(5000).astype(np.float32)
    x[:5] = [3, -4, 0, 12, 0]                                   # 9 + 16 + 144
    got = oracle.layer_sqnorms(x, off)
    assert got[0] == 169.0 and got[1] == 0.0
    for l in (2, 3):
        seg = x[off[l]:off[l + 1]].astype(np.float64)
        exact = math.fsum((seg * seg).tolist())                 # squares of binary32 values are exact in binary64
        assert abs(got[l] - exact) <= 2 ** -52 * exact
    h = x.astype(np.float16)
    goth = oracle.layer_sqnorms(h, off, dt=wl.F16)
    seg = h[off[3]:off[4]].astype(np.float64)
    assert abs(goth[3] - math.fsum((seg * seg).tolist())) <= 2 ** -52 * goth[3]
    ints = np.arange(-500, 500, dtype=np.float32)               # sum k^2 closed form
    assert oracle.layer_sqnorms(ints, np.array([0, 1000], np.int64))[0] == 500 * 501 * 1001 / 6 + 499 * 500 * 999 / 6


@pytest.mark.parametrize("scheme", [0, 1])
def test_sqerrors_against_the_definition(oracle, scheme):
    """||x - deq(Q(x))||^2 per layer from the oracle's own dequantizer and an exact sum; zero on
    pass-through layers and exact grids; below unit^2 per element; about unit^2/6 per element for
    uniform positions (E p(1-p) = 1/6)."""
    w = wl.tiny_mixed(seed=7)
    if scheme:
        w.bits = np.where(w.bits == 1, 2, w.bits).astype(np.uint8)
    g = w.gradient()
    q = oracle.qsgd_quantize if scheme else oracle.quantize
    p, m = q(g, w.offsets, w.bits, w.bucket, 5)
    deq = (oracle.qsgd_dequant_reduce if scheme else oracle.dequant_reduce)([p], [m], w.offsets, w.bits, w.bucket)["sum32"]
    got = oracle.layer_sqerrors(g, p, m, w.offsets, w.bits, w.bucket, scheme=scheme)
    for l in range(w.L):
        a, b = w.offsets[l], w.offsets[l + 1]
        d = g[a:b].astype(np.float64) - deq[a:b].astype(np.float64)     # exact differences
        exact = math.fsum((d * d).tolist())
        assert abs(got[l] - exact) <= 1e-14 * exact + 1e-300
        if w.bits[l] == 0:
            assert got[l] == 0.0
    # statistical size on one big uniform layer
    rng = np.random.default_rng(3)
    n, B, b = 1 << 16, 128, 4
    x = rng.uniform(-1, 1, n).astype(np.float32)
    off, bits = np.array([0, n], np.int64), np.array([b], np.uint8)
    p, m = q(x, off, bits, B, 9)
    err = oracle.layer_sqerrors(x, p, m, off, bits, B, scheme=scheme)[0]
    unit = np.repeat(m.reshape(n // B, -1)[:, 0].astype(np.float64), B)
    assert err <= (unit ** 2).sum()
    assert abs(err / ((unit ** 2).sum() / 6) - 1) < 0.05
    grid = (rng.integers(0, 16, n) * 2.0 ** -6).astype(np.float32)
    grid[::B], grid[1::B] = 0, 15 * 2.0 ** -6
    if scheme:
        grid = (rng.integers(-7, 8, n) * 2.0 ** -6).astype(np.float32)
        grid[::B] = 7 * 2.0 ** -6
    p, m = q(grid, off, bits, B, 9)
    assert oracle.layer_sqerrors(grid, p, m, off, bits, B, scheme=scheme)[0] == 0.0


def test_fewer_bits_give_a_larger_error(oracle):
    rng = np.random.default_rng(4)
    n, B = 1 << 15, 128
    x = rng.standard_normal(n).astype(np.float32)
    off = np.array([0, n], np.int64)
    errs = []
    for b in (2, 3, 4, 6, 8):
        bits = np.array([b], np.uint8)
        p, m = oracle.quantize(x, off, bits, B, 1)
        errs.append(oracle.layer_sqerrors(x, p, m, off, bits, B)[0])
    assert all(a > 3 * b for a, b in zip(errs, errs[1:]))       # one more bit: about 4x less


# ---------------------------------------------------------------- assigners

def blobs(rng, centres, per):
    pts = []
    for cx, cy in centres:
        pts += [(cx + 0.01 * rng.standard_normal(), cy + 0.01 * rng.standard_normal()) for _ in range(per)]
    return pts


def test_kmeans_recovers_separated_groups_and_orders_them_by_norm_minus_size():
    rng = np.random.default_rng(0)
    # (size, norm): big & quiet, middle, small & loud
    centres = [(0.9, 0.1), (0.5, 0.5), (0.1, 0.9)]
    pts = blobs(rng, centres, 7)
    perm = rng.permutation(len(pts))
    sizes = np.array([1e6 * (0.05 + pts[i][0]) for i in perm])
    norms = np.array([10.0 * (0.05 + pts[i][1]) for i in perm])
    bits = adaptive.kmeans_bits(sizes, norms, np.full(len(pts), 4), [2, 4, 8])
    want = np.array([[2, 4, 8][i // 7] for i in perm], np.uint8)
    assert np.array_equal(bits, want)
    # a filtered layer and an empty layer stay at 0 and do not move the others
    bits2 = adaptive.kmeans_bits(np.append(sizes, [64, 0]), np.append(norms, [1e9, 0.0]),
                                 np.append(np.full(len(pts), 4), [0, 4]), [2, 4, 8])
    assert np.array_equal(bits2[:-2], want) and bits2[-2] == 0 and bits2[-1] == 0


def test_kmeans_result_is_a_lloyd_fixed_point():
    rng = np.random.default_rng(5)
    M = 60
    sizes = np.exp(rng.uniform(5, 17, M))
    norms = np.exp(rng.normal(0, 1.5, M))
    bits, d = adaptive.kmeans_bits(sizes, norms, np.full(M, 4), [2, 3, 4, 8], details=True)
    x, y, lab = np.array(d["x"]), np.array(d["y"]), np.array(d["label"])
    cx, cy = np.array(d["cx"]), np.array(d["cy"])
    assert x.min() == 0 and x.max() == 1 and y.min() == 0 and y.max() == 1
    dist = (x[:, None] - cx[None]) ** 2 + (y[:, None] - cy[None]) ** 2
    assert np.array_equal(dist.argmin(1), lab)                  # every point sits with its nearest centroid
    for c in set(lab.tolist()):
        assert np.allclose([x[lab == c].mean(), y[lab == c].mean()], [cx[c], cy[c]], rtol=0, atol=1e-12)
    key = {c: cy[c] - cx[c] for c in set(lab.tolist())}
    for i in range(M):
        for j in range(M):
            if key[lab[i]] < key[lab[j]]:
                assert bits[i] <= bits[j]                       # bit-widths follow the centroid order


def test_kmeans_agrees_with_a_library_lloyd_from_the_same_start():
    KMeans = pytest.importorskip("sklearn.cluster").KMeans
    rng = np.random.default_rng(11)
    M, k = 80, 4
    sizes = np.exp(rng.uniform(5, 17, M))
    norms = np.exp(rng.normal(0, 1.5, M))
    _, d = adaptive.kmeans_bits(sizes, norms, np.full(M, 4), [1, 2, 4, 8], details=True)
    P = np.stack([d["x"], d["y"]], 1)
    key = P[:, 1] - P[:, 0]
    order = sorted(range(M), key=lambda i: (key[i], i))
    start = P[[order[((2 * c + 1) * M) // (2 * k)] for c in range(k)]]
    km = KMeans(n_clusters=k, init=start, n_init=1, max_iter=100, tol=0.0, algorithm="lloyd").fit(P)
    assert np.array_equal(km.labels_, np.array(d["label"]))
    assert np.allclose(km.cluster_centers_, np.stack([d["cx"], d["cy"]], 1), atol=1e-9)


def test_kmeans_small_and_degenerate_inputs():
    assert adaptive.kmeans_bits([], [], [], [2, 4]).size == 0
    assert np.array_equal(adaptive.kmeans_bits([100], [1.0], [4], [2, 4, 8]), [8])        # one layer: safest width
    # two layers, three widths: each its own cluster, ends of the range
    assert np.array_equal(adaptive.kmeans_bits([1000, 10], [1.0, 5.0], [4, 4], [2, 4, 8]), [2, 8])
    # identical points: one cluster, the largest width
    assert np.array_equal(adaptive.kmeans_bits([50] * 6, [2.0] * 6, [4] * 6, [2, 4]), [4] * 6)
    # one candidate: everything gets it
    assert np.array_equal(adaptive.kmeans_bits([5, 50, 500], [1, 2, 3], [4, 0, 4], [3]), [3, 0, 3])


def test_linear_heuristic_sorts_by_norm_over_size():
    sizes = np.array([1000, 10, 100, 10000, 50, 0])
    norms = np.array([1.0, 1.0, 1.0, 1.0, 1.0, 0.0])
    bits = adaptive.linear_bits(sizes, norms, [4, 4, 4, 4, 0, 4], [2, 4, 8])
    # ascending norm/size: 10000, 1000, 100, 10 -> ranks 0..3 of 4 -> floor(r*3/4) = 0,0,1,2
    assert np.array_equal(bits, [2, 8, 4, 2, 0, 0])
    rng = np.random.default_rng(2)
    s, t = rng.integers(1, 10**6, 40), rng.random(40)
    b = adaptive.linear_bits(s, t, np.full(40, 4), [2, 3, 4, 8])
    assert sorted(np.bincount(b)[[2, 3, 4, 8]]) == [10, 10, 10, 10]
    r = t / s
    assert all(b[i] <= b[j] for i in range(40) for j in range(40) if r[i] < r[j])


def test_bucket_sizes_follow_the_widths_linearly():
    """Sec. "Layer-wise Adaptive Quantization": bit-widths and bucket sizes are mapped to the layers
    linearly; fewest bits go with the longest buckets.  Hand-worked cases of the interpolation."""
    from oracle import adaptive as A
    # as many sizes as widths: a one-to-one, order-reversing map
    assert A.buckets_from_bits([2, 3, 4, 8], [8, 4, 3, 2], [128, 512, 1024, 2048]).tolist() == [2048, 1024, 512, 128]
    # 4 widths over 3 sizes: positions 0, 1, 2, 3 -> 0, 2/3, 4/3, 2 -> rounded 0, 1, 1, 2
    assert A.buckets_from_bits([2, 3, 4, 8], [2, 3, 4, 8], [2048, 512, 128]).tolist() == [2048, 512, 512, 128]
    # 2 widths over 5 sizes take the two ends
    assert A.buckets_from_bits([2, 8, 2], [2, 8], [64, 128, 256, 512, 1024]).tolist() == [1024, 64, 1024]
    # half-way positions round up: 3 widths over 2 sizes -> 0, 1/2, 1 -> 0, 1, 1
    assert A.buckets_from_bits([1, 4, 8], [1, 4, 8], [1024, 128]).tolist() == [1024, 128, 128]
    # one width: the longest bucket; uncompressed layers get a valid size too
    assert A.buckets_from_bits([4, 0, 4], [4], [128, 512]).tolist() == [512, 512, 512]
    # monotone: more bits never means a longer bucket
    rng = np.random.default_rng(0)
    for _ in range(50):
        widths = sorted(rng.choice(np.arange(1, 9), int(rng.integers(1, 8)), replace=False).tolist())
        sizes = rng.choice([32, 64, 128, 256, 512, 1024, 2048, 4096], int(rng.integers(1, 8)), replace=False).tolist()
        got = A.buckets_from_bits(widths, widths, sizes)
        assert all(a >= b for a, b in zip(got[:-1], got[1:]))
        assert got[0] == max(sizes) and (len(widths) == 1 or got[-1] == min(sizes))
