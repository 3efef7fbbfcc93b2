"""Pins of the oracle's norm-and-sign quantizer against the paper's printed formula
(Sec. 2.3, paragraph "Gradient Quantization": Q_s(v_i) = ||v|| sign(v_i) q(|v_i| / ||v||, s), with
q = l/s with probability 1 - p and (l+1)/s otherwise, p = a s - l), applied per bucket
(Sec. 4.3) with the maximum absolute value as the norm."""
from fractions import Fraction

import numpy as np
import pytest

from paper_2111_08617_amd import workloads as wl


def signed_levels(codes, b):
    """b-bit two's complement codes -> signed levels."""
    codes = np.asarray(codes).astype(np.int64)
    return codes - ((codes >> (b - 1)) << b)


def one_layer(n, b):
    return np.array([0, n], np.int64), np.array([b], np.uint8)


@pytest.mark.parametrize("b", [2, 3, 4, 8])
def test_levels_follow_the_printed_rule_exactly_enumerated(oracle, b):
    """All 65536 draws for every element of a bucket: E[level] = |v| / ||v|| * s, levels are the two
    neighbours, the code carries the sign of v, and the largest |v| always gets level s."""
    rng = np.random.default_rng(40 + b)
    B, s, K = 32, (1 << (b - 1)) - 1, 65536
    x = rng.standard_normal(B).astype(np.float32)
    grad = np.tile(x, K)
    offsets = np.arange(K + 1, dtype=np.int64) * B
    bits = np.full(K, b, np.uint8)
    draws = np.repeat(np.arange(K, dtype=np.uint16), B)
    packed, meta = oracle.qsgd_quantize(grad, offsets, bits, B, seed=0, draws=draws)
    codes = oracle.unpack_codes(packed, offsets, bits, B).reshape(K, B).astype(np.int64)
    signed = signed_levels(codes, b)
    level = np.abs(signed)
    assert (codes != 1 << (b - 1)).all()                               # -2^(b-1) is never used
    norm = Fraction(float(np.abs(x).max()))
    tol = Fraction(1, 65536) + Fraction(4 * s, 1 << 24)
    for j in range(B):
        pos = abs(Fraction(float(x[j]))) / norm * s
        seen = np.unique(level[:, j])
        assert seen.max() - seen.min() <= 1
        assert seen.min() >= int(np.floor(pos - tol)) and seen.max() <= int(np.ceil(pos + tol))
        assert abs(Fraction(int(level[:, j].sum()), K) - pos) <= tol
        assert (signed[:, j] * (-1 if x[j] < 0 else 1) >= 0).all()      # never the other sign
    top = level[:, int(np.abs(x).argmax())]
    assert (top >= s - 1).all() and (top == s).sum() >= K - 4
    assert np.allclose(meta, float(norm) / s, rtol=1e-6)


@pytest.mark.parametrize("b", [2, 3, 4, 8])
def test_levels_are_exact_draw_by_draw(oracle, b):
    """The 16-bit reading of the rule, every element and every draw: with T = trunc(|v| * inv16) and
    inv16 = (s * 65536) / ||v|| in binary32 arithmetic (each operation rounded to nearest even, redone
    here in exact rational arithmetic), level(u) = min(floor((T + u) / 65536), s): exactly the
    T mod 65536 largest draws go up.  The code is the signed level as a b-bit two's complement number."""
    from test_oracle_pins import to_binary32
    rng = np.random.default_rng(300 + b)
    B, s, K = 32, (1 << (b - 1)) - 1, 65536
    x = (rng.standard_normal(B) * 10.0 ** rng.uniform(-3, 2)).astype(np.float32)
    x[4] = -x[11]
    grad = np.tile(x, K)
    offsets = np.arange(K + 1, dtype=np.int64) * B
    bits = np.full(K, b, np.uint8)
    draws = np.repeat(np.arange(K, dtype=np.uint16), B)
    packed, meta = oracle.qsgd_quantize(grad, offsets, bits, B, seed=0, draws=draws)
    codes = oracle.unpack_codes(packed, offsets, bits, B).reshape(K, B).astype(np.int64)
    norm = Fraction(float(np.abs(x).max()))
    inv16 = to_binary32(Fraction(s * 65536) / norm)
    assert Fraction(float(np.asarray(meta).reshape(-1)[0])) == to_binary32(norm / s)
    u = np.arange(K, dtype=np.int64)
    for j in range(B):
        S = to_binary32(abs(Fraction(float(x[j]))) * inv16)
        T = S.numerator // S.denominator
        level = np.minimum((T + u) >> 16, s)
        signed = -level if x[j] < 0 else level
        assert np.array_equal(codes[:, j], signed & ((1 << b) - 1)), (j, T)
        assert np.array_equal(signed_levels(codes[:, j], b), signed)


def test_unbiased_and_within_one_step(oracle):
    rng = np.random.default_rng(2)
    n, B, b, N = 1024, 128, 4, 2000
    x = rng.standard_normal(n).astype(np.float32)
    off, bits = one_layer(n, b)
    acc = np.zeros(n)
    for seed in range(N):
        p, m = oracle.qsgd_quantize(x, off, bits, B, seed=seed * 31 + 5)
        d = oracle.qsgd_dequant_reduce([p], [m], off, bits, B)["sum64"]
        unit = np.repeat(m.astype(np.float64), B)
        assert (np.abs(d - x) <= unit * (1 + 1e-3)).all()
        assert (np.sign(d) * np.sign(x) >= 0).all()            # the sign never flips
        acc += d
    unit = np.repeat(m.astype(np.float64), B)
    assert np.abs(acc / N - x).max() < 5 * unit.max() * 0.5 / np.sqrt(N)


def test_exact_on_symmetric_power_of_two_grids(oracle):
    rng = np.random.default_rng(9)
    for b in (2, 3, 5, 8):
        s, B, n = (1 << (b - 1)) - 1, 64, 64 * 5 + 9
        lv = rng.integers(-s, s + 1, n)
        lv[::B] = s
        lv[-1] = -s
        x = (lv * 2.0 ** -9).astype(np.float32)
        off, bits = one_layer(n, b)
        for seed in (0, 99):
            p, m = oracle.qsgd_quantize(x, off, bits, B, seed=seed)
            assert (m == np.float32(2.0 ** -9)).all()
            codes = oracle.unpack_codes(p, off, bits, B)
            assert np.array_equal(signed_levels(codes, b), lv)
            d = oracle.qsgd_dequant_reduce([p], [m], off, bits, B)
            assert np.array_equal(d["sum32"], x) and np.array_equal(d["sum64"], x.astype(np.float64))


def test_zero_bucket_sizes_and_rejection_of_one_bit(oracle):
    n, B = 256, 128
    x = np.zeros(n, np.float32)
    x[130] = -0.0
    off, bits = one_layer(n, 4)
    p, m = oracle.qsgd_quantize(x, off, bits, B, seed=1)
    assert not m.any()
    assert not oracle.unpack_codes(p, off, bits, B).any()      # sign(0) * 0 has the one code 0
    d = oracle.qsgd_dequant_reduce([p], [m], off, bits, B)["sum32"]
    assert np.array_equal(d, x) and not np.signbit(d).any()
    y = np.full(n, -1e-30, np.float32)                          # negative values that round to level 0
    y[::B] = 1.0
    p, m = oracle.qsgd_quantize(y, off, bits, B, seed=2)
    codes = oracle.unpack_codes(p, off, bits, B)
    assert (codes[::B] == 7).all() and codes.sum() == 7 * (n // B)
    d = oracle.qsgd_dequant_reduce([p], [m], off, bits, B)["sum32"]
    assert (d[1:B] == 0).all() and not np.signbit(d[1:B]).any()
    pb, mb = oracle.qsgd_sizes(off, bits, B)
    pb2, mb2 = oracle.sizes(off, bits, B)
    assert pb == pb2 and 2 * mb == mb2                          # one float of meta per bucket
    with pytest.raises(ValueError):
        oracle.qsgd_sizes(off, np.array([1], np.uint8), B)


def test_reduce_is_exact_on_integer_grids_and_layout_is_shared(oracle):
    rng = np.random.default_rng(8)
    W, n, B, b = 5, 64 * 7 + 5, 64, 4
    off, bits = one_layer(n, b)
    total = np.zeros(n, np.int64)
    chunks, metas = [], []
    for w in range(W):
        lv = rng.integers(-7, 8, n)
        lv[::B] = 7
        lv[-1] = 7
        total += lv * (w + 1)
        p, m = oracle.qsgd_quantize((lv * (w + 1)).astype(np.float32), off, bits, B, seed=w)
        # the stream is the same LSB-first layout: code j in bits [4j, 4j+4)
        codes = lv & 15                                          # two's complement nibbles
        big = 0
        for j, c in enumerate(codes.tolist()):
            big |= c << (4 * j)
        assert p[:(n * 4 + 7) // 8].tobytes() == big.to_bytes((n * 4 + 7) // 8, "little")
        chunks.append(p)
        metas.append(m)
    d = oracle.qsgd_dequant_reduce(chunks, metas, off, bits, B)
    assert np.array_equal(d["sum32"], total.astype(np.float32))
    w = wl.tiny_mixed(seed=3)
    w.bits = np.where(w.bits == 1, 2, w.bits).astype(np.uint8)
    g = w.gradient()
    p, m = oracle.qsgd_quantize(g, w.offsets, w.bits, w.bucket, seed=4)
    s = oracle.qsgd_dequant_reduce([p, p], [m, m], w.offsets, w.bits, w.bucket)
    for l in np.nonzero(w.bits == 0)[0]:
        x = g[w.offsets[l]:w.offsets[l + 1]]
        assert np.array_equal(s["sum32"][w.offsets[l]:w.offsets[l + 1]], x + x)
    assert (np.abs(s["sum32"].astype(np.float64) - s["sum64"]) <= 1e-6 * s["abs64"] + 1e-45).all()
