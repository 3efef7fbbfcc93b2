"""Pins of the oracle's calls with a bucket size per layer (CGX paper Sec. 4.1: compression
parameters, the bucket size among them, are per layer).

The layered calls are pinned to the single-size ones, which have pins of their own: layers
are compressed independently of each other (Sec. 4.1), so layer l of a layered chunk must be
what the single-size quantizer gives for that layer alone, as a window of the buffer (the
draws are keyed on the position in the whole buffer), with bucket size buckets[l].
"""
import numpy as np
import pytest

import oracle as orc

F32, F16 = 0, 1


@pytest.fixture(scope="module")
def oracle():
    orc.build()
    return orc


def plan(seed):
    rng = np.random.default_rng(seed)
    L = int(rng.integers(1, 9))
    sizes = [int(rng.choice([0, 1, 31, 96, 1000, 2048, 4097, 9000])) for _ in range(L)]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    bits = rng.integers(0, 9, L).astype(np.uint8)
    buckets = rng.choice([32, 64, 96, 128, 512, 1024, 4096, 8192], L).astype(np.int32)
    return off, bits, buckets, rng


@pytest.mark.parametrize("dt", [F32, F16])
@pytest.mark.parametrize("seed", range(8))
def test_every_layer_is_the_single_size_quantizer_on_its_window(oracle, seed, dt):
    off, bits, buckets, rng = plan(seed)
    n = int(off[-1])
    g = (rng.standard_normal(n) * 3).astype(np.float16 if dt == F16 else np.float32)
    packed, meta = oracle.layered_quantize(g, off, bits, buckets, 11, dt)
    assert (packed.size, meta.size * 4) == oracle.layered_sizes(off, bits, buckets, dt)
    pos = mpos = 0
    for l in range(bits.size):
        a, b = int(off[l]), int(off[l + 1])
        if a == b:
            continue
        pl, ml = oracle.quantize(g[a:b], [0, b - a], [bits[l]], int(buckets[l]), 11, dt, index_base=a)
        assert np.array_equal(packed[pos:pos + pl.size], pl), f"layer {l}"
        assert np.array_equal(meta[mpos:mpos + ml.shape[0]].view(np.uint32), ml.view(np.uint32)), f"layer {l}"
        pos += pl.size
        mpos += ml.shape[0]
    assert pos == packed.size and mpos == meta.shape[0]


@pytest.mark.parametrize("seed", range(6))
def test_reduce_is_the_single_size_reduce_layer_by_layer(oracle, seed):
    off, bits, buckets, rng = plan(100 + seed)
    n = int(off[-1])
    W = 3
    chunks = [oracle.layered_quantize((rng.standard_normal(n)).astype(np.float32), off, bits, buckets, 5 + w) for w in range(W)]
    got = oracle.layered_dequant_reduce([c[0] for c in chunks], [c[1] for c in chunks], off, bits, buckets)
    pos = mpos = 0
    for l in range(bits.size):
        a, b = int(off[l]), int(off[l + 1])
        if a == b:
            continue
        pb, mb = oracle.sizes([0, b - a], [bits[l]], int(buckets[l]))
        ref = oracle.dequant_reduce([c[0][pos:pos + pb] for c in chunks],
                                    [c[1].reshape(-1)[mpos:mpos + mb // 4] for c in chunks],
                                    [0, b - a], [bits[l]], int(buckets[l]))
        for key in ("sum32", "sum64", "abs64"):
            assert np.array_equal(got[key][a:b], ref[key]), f"layer {l} {key}"
        pos += pb
        mpos += mb // 4


def test_equal_sizes_give_the_single_size_result_and_bad_sizes_are_rejected(oracle):
    off, bits, _, rng = plan(7)
    n = int(off[-1])
    g = rng.standard_normal(n).astype(np.float32)
    for bucket in (32, 96, 1024):
        same = np.full(bits.size, bucket, np.int32)
        p1, m1 = oracle.layered_quantize(g, off, bits, same, 3)
        p2, m2 = oracle.quantize(g, off, bits, bucket, 3)
        assert np.array_equal(p1, p2) and np.array_equal(m1.view(np.uint32), m2.view(np.uint32))
    for bad in (0, 16, 100, 8224):
        with pytest.raises(ValueError):
            oracle.layered_sizes(off, bits, np.full(bits.size, bad, np.int32))


@pytest.mark.parametrize("seed", range(6))
def test_squared_errors_are_those_of_the_layers_alone(oracle, seed):
    """Per-layer squared compression errors of a layered chunk: each layer's value is what the
    single-size function gives for that layer alone (same codes, same meta, its bucket size)."""
    off, bits, buckets, rng = plan(200 + seed)
    n = int(off[-1])
    g = rng.standard_normal(n).astype(np.float32)
    packed, meta = oracle.layered_quantize(g, off, bits, buckets, 9)
    got = oracle.layered_layer_sqerrors(g, packed, meta, off, bits, buckets)
    pos = mpos = 0
    for l in range(bits.size):
        a, b = int(off[l]), int(off[l + 1])
        if a == b:
            assert got[l] == 0
            continue
        pb, mb = oracle.sizes([0, b - a], [bits[l]], int(buckets[l]))
        ref = oracle.layer_sqerrors(g[a:b], packed[pos:pos + pb], meta.reshape(-1)[mpos:mpos + mb // 4],
                                    [0, b - a], [bits[l]], int(buckets[l]))
        assert got[l] == ref[0], f"layer {l}"
        pos += pb
        mpos += mb // 4


def test_local_addend_comes_first_in_the_layered_reduce(oracle):
    """With a local term the layered reduce is the single-size one layer by layer as well, and with
    W = 1 and no local term it is plain dequantization of the chunk."""
    off, bits, buckets, rng = plan(301)
    n = int(off[-1])
    chunks = [oracle.layered_quantize(rng.standard_normal(n).astype(np.float32), off, bits, buckets, 5 + w) for w in range(2)]
    local = rng.standard_normal(n).astype(np.float16)
    got = oracle.layered_dequant_reduce([c[0] for c in chunks], [c[1] for c in chunks], off, bits, buckets, local=local)
    pos = mpos = 0
    for l in range(bits.size):
        a, b = int(off[l]), int(off[l + 1])
        if a == b:
            continue
        pb, mb = oracle.sizes([0, b - a], [bits[l]], int(buckets[l]))
        ref = oracle.dequant_reduce([c[0][pos:pos + pb] for c in chunks],
                                    [c[1].reshape(-1)[mpos:mpos + mb // 4] for c in chunks],
                                    [0, b - a], [bits[l]], int(buckets[l]), local=local[a:b])
        assert np.array_equal(got["sum32"][a:b], ref["sum32"]) and np.array_equal(got["sum64"][a:b], ref["sum64"])
        pos += pb
        mpos += mb // 4


def qsgd_plan(seed):
    off, bits, buckets, rng = plan(seed)
    return off, np.where(bits == 1, 2, bits).astype(np.uint8), buckets, rng


@pytest.mark.parametrize("dt", [F32, F16])
@pytest.mark.parametrize("seed", range(6))
def test_norm_and_sign_form_layer_by_layer(oracle, seed, dt):
    """The norm-and-sign quantizer with a bucket size per layer: every layer is the single-size
    quantizer on its window, and the reduce is the single-size reduce of the layers' pieces."""
    off, bits, buckets, rng = qsgd_plan(400 + seed)
    n = int(off[-1])
    W = 2
    grads = [(rng.standard_normal(n) * 2).astype(np.float16 if dt == F16 else np.float32) for _ in range(W)]
    chunks = [oracle.qsgd_layered_quantize(g, off, bits, buckets, 7 + w, dt) for w, g in enumerate(grads)]
    assert (chunks[0][0].size, chunks[0][1].size * 4) == oracle.qsgd_layered_sizes(off, bits, buckets, dt)
    got = oracle.qsgd_layered_dequant_reduce([c[0] for c in chunks], [c[1] for c in chunks], off, bits, buckets, dt)
    pos = mpos = 0
    for l in range(bits.size):
        a, b = int(off[l]), int(off[l + 1])
        if a == b:
            continue
        pieces = []
        for w in range(W):
            pl, ml = oracle.qsgd_quantize(grads[w][a:b], [0, b - a], [bits[l]], int(buckets[l]), 7 + w, dt, index_base=a)
            assert np.array_equal(chunks[w][0][pos:pos + pl.size], pl), f"layer {l} peer {w}"
            assert np.array_equal(chunks[w][1][mpos:mpos + ml.size].view(np.uint32), ml.view(np.uint32)), f"layer {l}"
            pieces.append((pl, ml))
        ref = oracle.qsgd_dequant_reduce([p for p, _ in pieces], [m for _, m in pieces], [0, b - a], [bits[l]],
                                         int(buckets[l]), dt)
        for key in ("sum32", "sum64", "abs64"):
            assert np.array_equal(got[key][a:b], ref[key]), f"layer {l} {key}"
        pos += pieces[0][0].size
        mpos += pieces[0][1].size
    assert pos == chunks[0][0].size and mpos == chunks[0][1].size


def test_norm_and_sign_window_equals_the_slice_of_the_whole(oracle):
    """The window form of the norm-and-sign quantizer (used by the pin above): a window of a
    single-layer buffer that starts on a bucket boundary gives the slice of the whole chunk."""
    rng = np.random.default_rng(9)
    n, bucket, b = 4096, 256, 5
    g = rng.standard_normal(n).astype(np.float32)
    p, m = oracle.qsgd_quantize(g, [0, n], [b], bucket, 13)
    a = 1024
    pw, mw = oracle.qsgd_quantize(g[a:], [0, n - a], [b], bucket, 13, index_base=a)
    assert np.array_equal(pw, p[a * b // 8:]) and np.array_equal(mw.view(np.uint32), m[a // bucket:].view(np.uint32))
