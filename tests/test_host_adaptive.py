"""Host-side parts of the layer-wise adaptive scheme through the C ABI (no GPU needed): the
bit-width assigners against the CPU oracle (integer results: exact), their argument checks,
and the workspace sizes of the per-layer statistics."""
import ctypes

import numpy as np
import pytest

from oracle import adaptive
from paper_2111_08617_amd import binding as cgx
from paper_2111_08617_amd import workloads as wl


@pytest.fixture(scope="module")
def lib():
    import os
    if not os.path.exists(cgx.LIB_PATH):
        from paper_2111_08617_amd import build
        build.build()
    return cgx.lib()


def offsets_of(sizes):
    return np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)


def random_case(rng, L):
    sizes = np.exp(rng.uniform(2, 17, L)).astype(np.int64)
    sizes[rng.random(L) < 0.05] = 0
    norms = np.exp(rng.normal(0, 2, L)) * np.sqrt(np.maximum(sizes, 1)) * 1e-3
    bits_in = np.where((sizes < 2048) | (rng.random(L) < 0.1), 0, 4).astype(np.uint8)
    return sizes, norms, bits_in


@pytest.mark.parametrize("cands", [[2, 4, 8], [1, 2, 3, 4, 8], [4], [8, 2], [2, 3, 4, 5, 6, 7, 8]])
def test_kmeans_assigner_equals_the_oracle(lib, cands):
    rng = np.random.default_rng(len(cands) * 17 + cands[0])
    for L in (1, 2, 3, 7, 40, 161, 292):
        sizes, norms, bits_in = random_case(rng, L)
        got = cgx.cgx_assign_bits_kmeans(offsets_of(sizes), norms, bits_in, cands)
        want = adaptive.kmeans_bits(sizes, norms, bits_in, cands)
        assert np.array_equal(got, want), (L, cands)
        assert set(got[got > 0].tolist()) <= set(cands) and (got[(bits_in == 0) | (sizes == 0)] == 0).all()
        # a small iteration limit is honoured the same way
        assert np.array_equal(cgx.cgx_assign_bits_kmeans(offsets_of(sizes), norms, bits_in, cands, max_iter=2),
                              adaptive.kmeans_bits(sizes, norms, bits_in, cands, max_iter=2))


@pytest.mark.parametrize("cands", [[2, 4, 8], [1, 2, 3, 4, 8], [4], [8, 2]])
def test_linear_assigner_equals_the_oracle(lib, cands):
    rng = np.random.default_rng(len(cands) + 100)
    for L in (1, 2, 5, 33, 199):
        sizes, norms, bits_in = random_case(rng, L)
        got = cgx.cgx_assign_bits_linear(offsets_of(sizes), norms, bits_in, cands)
        assert np.array_equal(got, adaptive.linear_bits(sizes, norms, bits_in, cands))


def test_assigners_on_the_model_shaped_workloads(lib):
    """Layer tables of the benchmark configurations with synthetic norms: big quiet layers get
    the fewest bits, and the bandwidth objective sum(b_l * size_l) drops below all-4-bit."""
    for name in ("resnet50", "bert_base", "gpt2_medium"):
        w = wl.WORKLOADS[name]()
        sizes = np.diff(w.offsets)
        rng = np.random.default_rng(5)
        norms = np.sqrt(sizes) * 0.01 * np.exp(rng.normal(0, 0.3, w.L)) / (1 + sizes / 1e6)
        bits_in = np.where(w.bits == 0, 0, 4).astype(np.uint8)
        for fn, ref in ((cgx.cgx_assign_bits_kmeans, adaptive.kmeans_bits),
                        (cgx.cgx_assign_bits_linear, adaptive.linear_bits)):
            got = fn(w.offsets, norms, bits_in, [2, 3, 4])
            assert np.array_equal(got, ref(sizes, norms, bits_in, [2, 3, 4]))
            assert (got[w.bits == 0] == 0).all()
            assert (got * sizes).sum() < (bits_in * sizes).sum()
            assert got[np.argmax(np.where(bits_in > 0, sizes, 0))] == 2
            cgx.cgx_sizes(cgx.Plan(w.offsets, got, w.bucket, w.dt))     # a valid plan for the library


def test_assigner_argument_errors(lib):
    c = ctypes
    off = np.array([0, 10, 30], np.int64)
    norms = np.array([1.0, 2.0])
    bits = np.array([4, 4], np.uint8)
    cand = np.array([2, 4], np.uint8)
    out = np.zeros(2, np.uint8)
    km, lin = lib.cgx_assign_bits_kmeans, lib.cgx_assign_bits_linear
    a = (off.ctypes.data, norms.ctypes.data, bits.ctypes.data, cand.ctypes.data)
    assert km(2, *a, 2, 10, out.ctypes.data) == 0
    assert km(-1, *a, 2, 10, out.ctypes.data) == -2
    assert km(2, *a, 0, 10, out.ctypes.data) == -2
    assert km(2, *a, 65, 10, out.ctypes.data) == -2
    assert km(2, *a, 2, 0, out.ctypes.data) == -2
    assert km(2, None, a[1], a[2], a[3], 2, 10, out.ctypes.data) == -1
    assert km(2, a[0], None, a[2], a[3], 2, 10, out.ctypes.data) == -1
    assert km(2, a[0], a[1], None, a[3], 2, 10, out.ctypes.data) == -1
    assert km(2, a[0], a[1], a[2], None, 2, 10, out.ctypes.data) == -1
    assert km(2, *a, 2, 10, None) == -1
    assert km(2, np.array([1, 10, 30], np.int64).ctypes.data, a[1], a[2], a[3], 2, 10, out.ctypes.data) == -3
    assert km(2, np.array([0, 40, 30], np.int64).ctypes.data, a[1], a[2], a[3], 2, 10, out.ctypes.data) == -3
    assert km(2, a[0], a[1], np.array([9, 4], np.uint8).ctypes.data, a[3], 2, 10, out.ctypes.data) == -4
    assert km(2, a[0], a[1], a[2], np.array([0, 4], np.uint8).ctypes.data, 2, 10, out.ctypes.data) == -4
    assert km(2, a[0], a[1], a[2], np.array([9, 4], np.uint8).ctypes.data, 2, 10, out.ctypes.data) == -4
    assert lin(2, *a, 2, out.ctypes.data) == 0
    assert lin(2, *a, 0, out.ctypes.data) == -2
    assert lin(2, *a, 2, None) == -1
    assert km(0, None, None, None, a[3], 2, 10, None) == 0 and lin(0, None, None, None, a[3], 2, None) == 0


def test_statistics_workspace_and_argument_errors(lib):
    c = ctypes
    w = wl.tiny_mixed()
    plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
    assert cgx.cgx_layer_stats_workspace(plan) == 8 * cgx.cgx_plan_tiles(plan).size
    zero = cgx.Plan(w.offsets, np.zeros(w.L, np.uint8), 32, w.dt)
    assert cgx.cgx_layer_stats_workspace(plan, for_sqnorms=True) == 8 * cgx.cgx_plan_tiles(zero).size
    big = wl.resnet50()
    ws = cgx.cgx_layer_stats_workspace(cgx.Plan(big.offsets, big.bits, big.bucket, big.dt), for_sqnorms=True)
    assert big.n / 8192 * 8 <= ws <= (big.n / 8192 + big.L) * 8
    o, b = w.offsets.ctypes.data, w.bits.ctypes.data
    buf = 0x1000                                                      # never dereferenced
    nb = c.c_size_t()
    assert lib.cgx_layer_stats_workspace(w.n, w.L, o, b, w.bucket, w.dt, None) == -1
    assert lib.cgx_layer_stats_workspace(w.n + 1, w.L, o, b, w.bucket, w.dt, c.byref(nb)) == -2
    assert lib.cgx_layer_stats_workspace(w.n, w.L, o, b, 100, w.dt, c.byref(nb)) == -5
    sq = lib.cgx_layer_sqnorms
    assert sq(None, w.n, w.L, o, w.dt, buf, buf, 1 << 20, None) == -1
    assert sq(buf, w.n, w.L, o, w.dt, None, buf, 1 << 20, None) == -1
    assert sq(buf, w.n, w.L, o, w.dt, buf, None, 1 << 20, None) == -1
    assert sq(buf + 4, w.n, w.L, o, w.dt, buf, buf, 1 << 20, None) == -9
    assert sq(buf, w.n, w.L, o, w.dt, buf + 4, buf, 1 << 20, None) == -9
    assert sq(buf, w.n, w.L, o, 7, buf, buf, 1 << 20, None) == -7
    assert sq(buf, w.n - 1, w.L, o, w.dt, buf, buf, 1 << 20, None) == -2
    for fn in (lib.cgx_layer_sqerrors, lib.cgx_qsgd_layer_sqerrors):
        assert fn(None, buf, buf, w.n, w.L, o, b, w.bucket, w.dt, buf, buf, 1 << 20, None) == (-1 if fn is lib.cgx_layer_sqerrors else -4)
        assert fn(buf, buf, buf, w.n, w.L, o, b, 48, w.dt, buf, buf, 1 << 20, None) == -5
    two = np.where(w.bits == 1, 2, w.bits).astype(np.uint8).ctypes.data
    assert lib.cgx_qsgd_layer_sqerrors(buf, None, buf, w.n, w.L, o, two, w.bucket, w.dt, buf, buf, 1 << 20, None) == -1
    assert lib.cgx_layer_sqerrors(buf, buf, None, w.n, w.L, o, b, w.bucket, w.dt, buf, buf, 1 << 20, None) == -1
    assert lib.cgx_layer_sqerrors(buf, buf, buf, w.n, w.L, o, b, w.bucket, w.dt, None, buf, 1 << 20, None) == -1
    assert lib.cgx_layer_sqerrors(buf, buf + 8, buf, w.n, w.L, o, b, w.bucket, w.dt, buf, buf, 1 << 20, None) == -9


def test_bucket_sizes_from_widths_equal_the_oracle_and_check_their_arguments(lib):
    rng = np.random.default_rng(11)
    for _ in range(200):
        widths = rng.choice(np.arange(1, 9), int(rng.integers(1, 9)), replace=False).astype(np.uint8)
        sizes = rng.choice(np.arange(1, 257) * 32, int(rng.integers(1, 12)), replace=False).astype(np.int32)
        bits = rng.choice(np.concatenate([[0], widths]), int(rng.integers(0, 40))).astype(np.uint8)
        got = cgx.cgx_assign_buckets_from_bits(bits, widths, sizes)
        assert got.tolist() == adaptive.buckets_from_bits(bits, widths, sizes).tolist()
    c = ctypes
    bits = np.array([2, 0, 4], np.uint8)
    widths = np.array([2, 4], np.uint8)
    sizes = np.array([128, 1024], np.int32)
    out = np.zeros(3, np.int32)

    def call(L=3, b=bits, w=widths, k=2, s=sizes, kb=2, o=out):
        return lib.cgx_assign_buckets_from_bits(L, b.ctypes.data if b is not None else None,
                                                w.ctypes.data if w is not None else None, k,
                                                s.ctypes.data if s is not None else None, kb,
                                                o.ctypes.data if o is not None else None)

    assert call() == 0 and out.tolist() == [1024, 1024, 128]
    assert call(L=-1) == -2 and call(k=0) == -2 and call(kb=65) == -2
    assert call(b=None) == -1 and call(w=None) == -1 and call(s=None) == -1 and call(o=None) == -1
    assert call(w=np.array([2, 9], np.uint8)) == -4
    assert call(b=np.array([2, 3, 4], np.uint8)) == -4          # 3 is not a candidate
    assert call(s=np.array([128, 100], np.int32)) == -5
    assert call(L=0, b=None, o=None) == 0
