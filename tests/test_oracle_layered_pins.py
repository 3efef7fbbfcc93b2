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
