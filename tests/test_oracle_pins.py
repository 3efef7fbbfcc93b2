"""Pins of the CPU oracle against what the paper and the mathematics fix.

Nothing here touches the GPU library.  Each test names the passage it pins:
  - rounding rule: Sec. 2.3 "Communication Compression Methods", paragraph
    "Gradient Quantization", definition of q(v_i, s)
    (level l+1 with probability p = a*s - l, else l);
  - bucketing with per-bucket meta-data: Sec. 4.3 "Efficient Quantization";
  - per-layer compression and uncompressed small layers: Sec. 4.1 "The Native
    CGX Framework";
  - dequantize first, then sum: Sec. 4 (non-associativity) and Sec. 4.1
    "Choosing a Reduction Scheme" (Scatter-Reduce-Allgather);
  - "~8x" compression at 4 bits: the table "Compression approaches" (the paper's third).
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2111_08617_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def one_layer(n, b):
    return np.array([0, n], np.int64), np.array([b], np.uint8)


# ------------------------------------------------------------------ rounding rule

@pytest.mark.parametrize("b", [1, 2, 3, 4, 5, 8])
def test_rounding_probability_brute_force(oracle, b):
    """Enumerate all 65536 draws for every element of one 32-element bucket and
    compare the level frequencies with the paper's rule evaluated in exact
    rational arithmetic on the same binary32 inputs."""
    rng = np.random.default_rng(100 + b)
    B, Lv = 32, (1 << b) - 1
    x = rng.standard_normal(B).astype(np.float32)
    x[5] = x[6]                      # a repeated value
    K = 65536
    grad = np.tile(x, K)
    offsets = np.arange(K + 1, dtype=np.int64) * B      # K layers, each the same bucket
    bits = np.full(K, b, np.uint8)
    draws = np.repeat(np.arange(K, dtype=np.uint16), B)  # copy k sees draw k for all its elements
    packed, meta = oracle.quantize(grad, offsets, bits, B, seed=0, draws=draws)
    codes = oracle.unpack_codes(packed, offsets, bits, B).reshape(K, B).astype(np.int64)

    mn, mx = Fraction(float(x.min())), Fraction(float(x.max()))
    tol = Fraction(1, 65536) + Fraction(4 * Lv, 1 << 24)   # 16-bit p + binary32 rounding of (x-mn)*inv
    for j in range(B):
        pos = (Fraction(float(x[j])) - mn) / (mx - mn) * Lv    # a * s in the paper's notation
        seen = np.unique(codes[:, j])
        assert seen.min() >= int(np.floor(pos - tol)) and seen.max() <= int(np.ceil(pos + tol)), (j, seen, float(pos))
        assert seen.max() - seen.min() <= 1
        mean = Fraction(int(codes[:, j].sum()), K)          # l + P(up)
        assert abs(mean - pos) <= tol, (j, float(mean), float(pos))
    # the minimum gets code 0 for every draw; the maximum gets code Lv for all but at
    # most a few of the 65536 draws (binary32 rounding of range * inv16 may land just
    # below Lv * 65536) and never leaves the top interval
    assert (codes[:, int(x.argmin())] == 0).all()
    top = codes[:, int(x.argmax())]
    assert (top >= Lv - 1).all() and (top == Lv).sum() >= K - 4


def to_binary32(v: Fraction) -> Fraction:
    """v rounded to the nearest IEEE binary32 number, ties to even, in exact integer arithmetic
    (written out here so that the pins below do not lean on any library's float32)."""
    if v == 0:
        return Fraction(0)
    sign, a = (-1 if v < 0 else 1), abs(v)
    e = a.numerator.bit_length() - a.denominator.bit_length()          # 2^(e-1) < a < 2^(e+1)
    if Fraction(2) ** e > a:
        e -= 1                                                          # now 2^e <= a < 2^(e+1)
    q = max(e - 23, -149)                                               # weight of the last mantissa bit
    scaled = a / Fraction(2) ** q
    m = scaled.numerator // scaled.denominator
    rest = scaled - m
    if rest > Fraction(1, 2) or (rest == Fraction(1, 2) and m % 2 == 1):
        m += 1
    assert m < 2 ** 24 + 1 and e < 128
    return sign * m * Fraction(2) ** q


def test_binary32_rounding_helper():
    rng = np.random.default_rng(0)
    for v in np.concatenate([rng.standard_normal(200) * 10.0 ** rng.integers(-30, 30, 200), [1e-45, 3e-39, 2.0 ** -126]]):
        assert to_binary32(Fraction(float(v))) == Fraction(float(np.float32(v)))
    assert to_binary32(Fraction(2 ** 24 + 1)) == 2 ** 24 and to_binary32(Fraction(2 ** 24 + 3)) == 2 ** 24 + 4


@pytest.mark.parametrize("b", [1, 2, 3, 4, 5, 8])
def test_rounding_rule_is_exact_draw_by_draw(oracle, b):
    """Sec. 2.3 "Gradient Quantization": level l goes up with probability p = a s - l.  The reading
    in force resolves p to 16 bits: with T = trunc((x - mn) * inv16) in binary32 arithmetic, exactly
    the T mod 65536 largest of the 65536 possible draws round up.  Every element, every draw:
    code(u) = min(floor((T + u) / 65536), Lv), with T recomputed here in exact rational arithmetic
    with an explicit round-to-nearest-even after each of the three binary32 operations and after the
    division that gives inv16.  (Fails for a rounded instead of truncated T, for <= in place of <
    in the carry, for a fused multiply, for one rounding left out.)"""
    rng = np.random.default_rng(200 + b)
    B, Lv, K = 32, (1 << b) - 1, 65536
    x = (rng.standard_normal(B) * 10.0 ** rng.uniform(-3, 2)).astype(np.float32)
    x[3] = x[9]
    grad = np.tile(x, K)
    offsets = np.arange(K + 1, dtype=np.int64) * B
    bits = np.full(K, b, np.uint8)
    draws = np.repeat(np.arange(K, dtype=np.uint16), B)
    packed, meta = oracle.quantize(grad, offsets, bits, B, seed=0, draws=draws)
    codes = oracle.unpack_codes(packed, offsets, bits, B).reshape(K, B).astype(np.int64)
    mn, mx = Fraction(float(x.min())), Fraction(float(x.max()))
    rng_ = to_binary32(mx - mn)
    inv16 = to_binary32(Fraction(Lv * 65536) / rng_)
    unit = to_binary32(rng_ / Lv)
    assert Fraction(float(meta[0, 0])) == unit and Fraction(float(meta[0, 1])) == mn
    u = np.arange(K, dtype=np.int64)
    up_total = 0
    for j in range(B):
        S = to_binary32(to_binary32(Fraction(float(x[j])) - mn) * inv16)
        T = S.numerator // S.denominator                                # truncation (S >= 0)
        expect = np.minimum((T + u) >> 16, Lv)
        assert np.array_equal(codes[:, j], expect), (j, T)
        if (T >> 16) < Lv:
            assert int(codes[:, j].sum()) == 65536 * (T >> 16) + (T & 0xffff)
            up_total += T & 0xffff
        # and the same T from numpy's binary32, step by step
        d32 = np.float32(x[j]) - np.float32(x.min())
        S32 = np.float32(d32) * np.float32(float(inv16))
        assert int(S32) == T
    assert up_total > 0
    # the probability of going up is p truncated to 16 bits: never above p, less than 2^-16 below it
    for j in range(B):
        pos = (Fraction(float(x[j])) - mn) / (mx - mn) * Lv
        mean = Fraction(int(codes[:, j].sum()), K)
        if 0 < pos < Lv:
            assert mean - pos <= Fraction(4 * Lv, 1 << 24)               # binary32 rounding of (x - mn) * inv16 only
            assert pos - mean < Fraction(1, 65536) + Fraction(4 * Lv, 1 << 24)


def test_real_draws_even_elements_take_the_low_half(oracle):
    """With the generator in place of mock draws: element i uses the low half of the word of its pair
    i >> 1 when i is even and the high half when it is odd (the words are taken from oracle.rng32,
    whose stream is pinned statistically further down; what is pinned here is which half goes where,
    and that the buffer index, not the position in the bucket or layer, selects the draw)."""
    rng = np.random.default_rng(9)
    B, b, n, seed = 64, 4, 64 * 5, 2 ** 40 + 17
    x = rng.standard_normal(n).astype(np.float32)
    offsets, bits = np.array([0, 3 * B, n], np.int64), np.array([b, b], np.uint8)
    for base in (0, 2 ** 33 - 2 * B, 7):
        packed, meta = oracle.quantize(x, offsets, bits, B, seed=seed, index_base=base)
        codes = oracle.unpack_codes(packed, offsets, bits, B).astype(np.int64)
        words = [oracle.rng32(seed, (base + i) >> 1) for i in range(n)]
        u = np.array([(w >> 16) if (base + i) & 1 else (w & 0xffff) for i, w in enumerate(words)], np.int64)
        assert len(set(words[::2])) > n // 2 - 2
        for k in range(n // B):
            xb = x[k * B:(k + 1) * B]
            r32 = np.float32(xb.max()) - np.float32(xb.min())
            inv16 = np.float32(15 * 65536) / r32
            T = ((xb - xb.min()) * inv16).astype(np.int64)
            assert np.array_equal(codes[k * B:(k + 1) * B], np.minimum((T + u[k * B:(k + 1) * B]) >> 16, 15))


def test_unbiased_over_seeds(oracle):
    """E[dequantized] = x (the property QSGD-style rounding is chosen for):
    per-element mean over many seeds, z-scored with the rule's own variance."""
    rng = np.random.default_rng(5)
    n, B, b, N = 1024, 128, 4, 3000
    x = (rng.standard_normal(n) * 0.01).astype(np.float32)
    offsets, bits = one_layer(n, b)
    acc = np.zeros(n)
    acc2 = np.zeros(n)
    for seed in range(N):
        p, m = oracle.quantize(x, offsets, bits, B, seed=seed * 7919 + 1)
        d = oracle.dequant_reduce([p], [m], offsets, bits, B)["sum64"]
        acc += d
        acc2 += d * d
    mean = acc / N
    var = acc2 / N - mean ** 2
    unit = np.repeat(m[:, 0].astype(np.float64), B)
    # expected variance unit^2 p(1-p) <= unit^2/4
    assert (var <= unit ** 2 / 4 * 1.2 + 1e-30).all()
    sigma = np.sqrt(np.maximum(var, (unit * 1e-3) ** 2) / N)
    z = (mean - x.astype(np.float64)) / sigma
    inner = var > (unit * 0.05) ** 2
    assert np.abs(z[inner]).max() < 5.0
    assert abs(z[inner].mean()) < 5.0 / np.sqrt(inner.sum())
    # elements with (almost) no variance sit on the grid: their mean must be x itself
    assert np.abs(mean[~inner] - x[~inner]).max() <= unit.max() * 0.06


@pytest.mark.parametrize("b", [1, 2, 3, 4, 6, 8])
@pytest.mark.parametrize("dt", [wl.F32, wl.F16])
def test_error_at_most_one_step(oracle, b, dt):
    """Every element lands on one of the two grid points around it."""
    rng = np.random.default_rng(b)
    n, B = 5000, 256
    x = (rng.standard_normal(n) * 3).astype(np.float16 if dt else np.float32)
    offsets, bits = one_layer(n, b)
    p, m = oracle.quantize(x, offsets, bits, B, seed=11, dt=dt)
    d = oracle.dequant_reduce([p], [m], offsets, bits, B, dt=dt)["sum32"]
    unit = np.repeat(m[:, 0], B)[:n].astype(np.float64)
    err = np.abs(d.astype(np.float64) - x.astype(np.float64))
    assert (err <= unit * (1 + 1e-3) + 1e-6).all()
    assert (m[:, 0] > 0).all()
    # meta is (unit, min): min is exact, unit = (max - min) / Lv
    xb = np.pad(x.astype(np.float32), (0, -n % B), constant_values=np.nan).reshape(-1, B)
    assert np.array_equal(m[:, 1], np.nanmin(xb, axis=1))
    rng_ = (np.nanmax(xb, axis=1).astype(np.float64) - np.nanmin(xb, axis=1)) / ((1 << b) - 1)
    assert np.allclose(m[:, 0], rng_, rtol=1e-6)


@pytest.mark.parametrize("b", [1, 2, 3, 4, 7, 8])
def test_grid_points_round_trip_exactly(oracle, b):
    """Values already on a power-of-two grid have p = 0: exact for every seed."""
    rng = np.random.default_rng(b)
    Lv, B, n = (1 << b) - 1, 64, 64 * 9 + 17
    codes = rng.integers(0, Lv + 1, n)
    nb = -(-n // B)
    for k in range(nb):                         # every bucket spans the whole grid
        codes[k * B] = 0
        codes[min(k * B + 1, n - 1)] = Lv
    codes[-2:] = [0, Lv]
    x = (np.float32(-3.25) + codes.astype(np.float32) * np.float32(2.0 ** -7)).astype(np.float32)
    offsets, bits = one_layer(n, b)
    for seed in (0, 1, 2**63 + 5):
        p, m = oracle.quantize(x, offsets, bits, B, seed=seed)
        assert np.array_equal(oracle.unpack_codes(p, offsets, bits, B), codes.astype(np.uint8))
        d = oracle.dequant_reduce([p], [m], offsets, bits, B)["sum32"]
        assert np.array_equal(d, x)
        assert (m[:, 0] == np.float32(2.0 ** -7)).all() and (m[:, 1] == np.float32(-3.25)).all()


def test_constant_and_zero_buckets(oracle):
    n, B = 3 * 128, 128
    x = np.empty(n, np.float32)
    x[:128] = 0.37                      # constant
    x[128:256] = 0.0
    x[128] = -0.0                       # signed zeros only
    x[256:] = 1e-42                     # constant subnormal
    offsets, bits = one_layer(n, 4)
    p, m = oracle.quantize(x, offsets, bits, B, seed=3)
    assert not p.any()
    assert np.array_equal(m[:, 0], np.zeros(3, np.float32))
    assert m[0, 1] == np.float32(0.37) and m[2, 1] == np.float32(1e-42)
    assert m[1, 1] == 0 and not np.signbit(m[1, 1])            # a zero minimum is stored as +0
    d = oracle.dequant_reduce([p], [m], offsets, bits, B)["sum32"]
    assert np.array_equal(d, np.abs(x))                         # abs only drops the sign of -0


def test_negative_zero_minimum_is_canonical(oracle):
    x = np.linspace(0, 1, 64).astype(np.float32)
    y = x.copy()
    y[0] = -0.0
    offsets, bits = one_layer(64, 4)
    pa, ma = oracle.quantize(x, offsets, bits, 64, seed=9)
    pb, mb = oracle.quantize(y, offsets, bits, 64, seed=9)
    assert np.array_equal(pa, pb) and ma.tobytes() == mb.tobytes()


# ------------------------------------------------------------------ packing and sizes

def read_golden():
    rows = []
    with open(os.path.join(GOLDEN, "packing_layout.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            b, codes, data = line.split("|")
            rows.append((int(b), [int(c) for c in codes.split()], bytes(int(h, 16) for h in data.split())))
    return rows


@pytest.mark.parametrize("row", read_golden(), ids=lambda r: f"b{r[0]}n{len(r[1])}")
def test_packing_matches_hand_worked_bytes(oracle, row):
    b, codes, expect = row
    x = np.array(codes, np.float32)             # unit = 1, min = 0: the code of x is x
    offsets, bits = one_layer(len(codes), b)
    p, m = oracle.quantize(x, offsets, bits, 32, seed=123)
    assert p.tobytes() == expect
    assert m.tolist() == [[1.0, 0.0]]


@pytest.mark.parametrize("b", [1, 2, 3, 4, 5, 6, 7, 8])
def test_packing_is_little_endian_big_integer(oracle, b):
    """The layer's stream read as one little-endian integer is sum code_j << (j*b)."""
    rng = np.random.default_rng(b)
    Lv, n, B = (1 << b) - 1, 1000 + b, 96
    codes = rng.integers(0, Lv + 1, n)
    codes[::B] = 0
    codes[1::B] = Lv
    codes[-2:] = [0, Lv]
    x = codes.astype(np.float32) * np.float32(0.5)
    offsets, bits = one_layer(n, b)
    p, _ = oracle.quantize(x, offsets, bits, B, seed=1)
    big = 0
    for j, c in enumerate(codes.tolist()):
        big |= c << (j * b)
    nbytes = (n * b + 7) // 8
    assert p[:nbytes].tobytes() == big.to_bytes(nbytes, "little")
    assert p.size == (nbytes + 15) // 16 * 16 and not p[nbytes:].any()


def test_sizes_closed_form_and_compression_ratio(oracle):
    n = 1 << 20
    off, bits = one_layer(n, 4)
    pb, mb = oracle.sizes(off, bits, 128)
    assert (pb, mb) == (n // 2, 8 * n // 128)
    assert abs(4 * n / (pb + mb) - 7.11) < 0.01        # "~8x" at 4 bits, bucket 128
    pb, mb = oracle.sizes(off, bits, 1024)
    assert abs(4 * n / (pb + mb) - 7.88) < 0.01        # bucket 1024
    # ragged: 3-bit layer of 1001 elements, pass-through of 7 binary16 values, empty layer
    off = np.array([0, 1001, 1008, 1008], np.int64)
    bits = np.array([3, 0, 5], np.uint8)
    pb, mb = oracle.sizes(off, bits, 64, wl.F16)
    assert pb == 384 + 16 and mb == 8 * 16             # ceil(3003/8)=376 -> 384; 14 -> 16; 16 buckets


def test_plan_validation(oracle):
    off, bits = one_layer(100, 4)
    for bad_bucket in (0, 16, 48, 8224, -32):
        with pytest.raises(ValueError):
            oracle.sizes(off, bits, bad_bucket)
    with pytest.raises(ValueError):
        oracle.sizes(off, np.array([9], np.uint8), 32)
    with pytest.raises(ValueError):
        oracle.sizes(np.array([0, 10, 5], np.int64), np.array([4, 4], np.uint8), 32)
    with pytest.raises(ValueError):
        oracle.sizes(np.array([1, 10], np.int64), np.array([4], np.uint8), 32)


# ------------------------------------------------------------------ locality

def test_bucket_and_layer_independence(oracle):
    """Changing one element changes only its own bucket's meta and payload."""
    w = wl.tiny_mixed(seed=21)
    g = w.gradient()
    p0, m0 = oracle.quantize(g, w.offsets, w.bits, w.bucket, seed=4)
    layer = 4                                     # 8-bit layer with a ragged tail
    j = 1000
    g2 = g.copy()
    g2[w.offsets[layer] + j] = 50.0
    p1, m1 = oracle.quantize(g2, w.offsets, w.bits, w.bucket, seed=4)
    seg = 0
    bucket0 = 0
    for l in range(layer):
        ln = int(w.offsets[l + 1] - w.offsets[l])
        if ln == 0:
            continue
        if w.bits[l]:
            seg += (-(-ln * int(w.bits[l]) // 8) + 15) // 16 * 16
            bucket0 += -(-ln // w.bucket)
        else:
            seg += (ln * 4 + 15) // 16 * 16
    k = j // w.bucket
    lo = seg + k * w.bucket * 8 // 8
    hi = lo + w.bucket
    changed = np.nonzero(p0 != p1)[0]
    assert changed.size and changed.min() >= lo and changed.max() < hi
    mchg = np.nonzero((m0 != m1).any(axis=1))[0]
    assert mchg.tolist() == [bucket0 + k]


def test_pass_through_layers_are_verbatim(oracle):
    for dt in (wl.F32, wl.F16):
        w = wl.tiny_mixed(seed=3, dt=dt)
        g = w.gradient()
        p, m = oracle.quantize(g, w.offsets, w.bits, w.bucket, seed=8, dt=dt)
        codes = oracle.unpack_codes(p, w.offsets, w.bits, w.bucket, dt)
        seg = 0
        es = 2 if dt else 4
        for l in range(w.L):
            ln = int(w.offsets[l + 1] - w.offsets[l])
            b = int(w.bits[l])
            if ln == 0:
                continue
            if b == 0:
                raw = g[w.offsets[l]:w.offsets[l + 1]].tobytes()
                assert p[seg:seg + len(raw)].tobytes() == raw
                assert (codes[w.offsets[l]:w.offsets[l + 1]] == 0xff).all()
                seg += (ln * es + 15) // 16 * 16
            else:
                assert (codes[w.offsets[l]:w.offsets[l + 1]] <= (1 << b) - 1).all()
                seg += (-(-ln * b // 8) + 15) // 16 * 16
        assert seg == p.size
        s = oracle.dequant_reduce([p, p, p], [m, m, m], w.offsets, w.bits, w.bucket, dt)
        for l in np.nonzero(w.bits == 0)[0]:
            x = g[w.offsets[l]:w.offsets[l + 1]].astype(np.float32)
            assert np.array_equal(s["sum32"][w.offsets[l]:w.offsets[l + 1]], (x + x) + x)


def test_binary16_storage_equals_widened_input(oracle):
    """Binary16 storage only changes how elements are read: quantizing the
    widened values in binary32 storage gives the same codes and meta."""
    rng = np.random.default_rng(0)
    h = (rng.standard_normal(4096) * 1e-3).astype(np.float16)
    h[:40] = np.array([6e-8 * k for k in range(40)], np.float16)      # binary16 subnormals
    offsets, bits = one_layer(h.size, 4)
    ph, mh = oracle.quantize(h, offsets, bits, 128, seed=2, dt=wl.F16)
    pf, mf = oracle.quantize(h.astype(np.float32), offsets, bits, 128, seed=2, dt=wl.F32)
    assert np.array_equal(ph, pf) and mh.tobytes() == mf.tobytes()


# ------------------------------------------------------------------ dequantize and reduce

def nearest_f32(fr: Fraction) -> np.float32:
    """Correctly rounded binary32 of an exact rational."""
    c = np.float32(float(fr))
    best = None
    for cand in (np.nextafter(c, np.float32(-np.inf)), c, np.nextafter(c, np.float32(np.inf))):
        err = abs(Fraction(float(cand)) - fr)
        even = (np.float32(cand).view(np.uint32) & 1) == 0
        key = (err, 0 if even else 1)
        if best is None or key < best[0]:
            best = (key, cand)
    return np.float32(best[1])


def test_single_chunk_is_affine_dequantization(oracle):
    """W = 1 reduces to q * unit + min with a single rounding."""
    rng = np.random.default_rng(3)
    n, B, b = 2048, 128, 4
    x = rng.standard_normal(n).astype(np.float32)
    offsets, bits = one_layer(n, b)
    p, m = oracle.quantize(x, offsets, bits, B, seed=5)
    codes = oracle.unpack_codes(p, offsets, bits, B)
    d = oracle.dequant_reduce([p], [m], offsets, bits, B)
    for j in rng.integers(0, n, 300):
        unit, mn = m[j // B]
        exact = Fraction(int(codes[j])) * Fraction(float(unit)) + Fraction(float(mn))
        assert d["sum32"][j] == nearest_f32(exact)
        assert d["sum64"][j] == float(exact)            # exact in binary64 here
        assert d["abs64"][j] == abs(float(exact))


def test_reduce_is_exact_on_integer_grids(oracle):
    """With power-of-two steps and small integers every sum is exact, so the
    result equals integer arithmetic."""
    rng = np.random.default_rng(8)
    W, n, B, b = 5, 64 * 7 + 5, 64, 4
    offsets, bits = one_layer(n, b)
    total = np.zeros(n, np.int64)
    chunks, metas = [], []
    for w in range(W):
        codes = rng.integers(0, 16, n)
        codes[::B] = 0
        codes[1::B] = 15
        codes[-2:] = [0, 15]
        shift = int(rng.integers(-20, 20))
        x = (codes + shift).astype(np.float32)
        total += codes + shift
        p, m = oracle.quantize(x, offsets, bits, B, seed=w)
        chunks.append(p)
        metas.append(m)
    d = oracle.dequant_reduce(chunks, metas, offsets, bits, B)
    assert np.array_equal(d["sum32"], total.astype(np.float32))
    assert np.array_equal(d["sum64"], total.astype(np.float64))


def test_reduce_binary32_stays_within_bound_of_binary64(oracle):
    w = wl.tiny_mixed(seed=5)
    chunks, metas = [], []
    for peer in range(8):
        p, m = oracle.quantize(w.gradient(peer), w.offsets, w.bits, w.bucket, seed=w.quant_seed(peer))
        chunks.append(p)
        metas.append(m)
    d = oracle.dequant_reduce(chunks, metas, w.offsets, w.bits, w.bucket)
    err = np.abs(d["sum32"].astype(np.float64) - d["sum64"])
    assert (err <= 1e-6 * d["abs64"] + 1e-45).all()
    # and the sum of W unbiased estimates estimates the true sum: error ~ sqrt(W) steps at most
    true = sum(w.gradient(peer).astype(np.float64) for peer in range(8))
    q = w.bits > 0
    for l in np.nonzero(q)[0]:
        a, b_ = int(w.offsets[l]), int(w.offsets[l + 1])
        if b_ > a:
            unit_max = max(float(m[:, 0].max()) for m in metas)
            assert np.abs(d["sum64"][a:b_] - true[a:b_]).max() <= 8 * unit_max * 1.001


def test_mean_of_sums_converges(oracle):
    """E[sum_w deq_w] = sum_w x_w, and the spread of the mean over W peers of the
    same vector shrinks like 1/sqrt(W)."""
    rng = np.random.default_rng(2)
    n, B, b = 4096, 128, 2
    x = rng.standard_normal(n).astype(np.float32)
    offsets, bits = one_layer(n, b)
    spread = {}
    for W in (1, 16):
        chunks, metas = zip(*[oracle.quantize(x, offsets, bits, B, seed=1000 * W + w) for w in range(W)])
        mean = oracle.dequant_reduce(list(chunks), list(metas), offsets, bits, B)["sum64"] / W
        spread[W] = np.sqrt(np.mean((mean - x) ** 2))
    assert 3.0 < spread[1] / spread[16] < 5.5           # sqrt(16) = 4


def test_half_conversion_matches_ieee_rounding(oracle):
    """binary32 -> binary16 with ties to even: numpy's conversion is the reference routine."""
    rng = np.random.default_rng(0)
    x = np.concatenate([
        rng.standard_normal(200000).astype(np.float32) * np.float32(10.0) ** rng.integers(-9, 5, 200000).astype(np.float32),
        np.arange(0, 70000, 0.25, dtype=np.float32),                       # around the overflow threshold
        np.float32(2.0 ** -24) * np.arange(0, 4096, 0.125, dtype=np.float32),   # subnormal halves and their ties
        np.array([0.0, -0.0, np.inf, -np.inf, 65504.0, 65519.99, 65520.0, 1e-10, -1e-10], np.float32),
        np.arange(2048, 4096, 0.5, dtype=np.float32),                      # exact ties in the normal range
    ])
    x = np.concatenate([x, -x])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(oracle.float_to_half(x), want)
    assert oracle.float_to_half(np.array([np.nan], np.float32))[0] & 0x7c00 == 0x7c00


def test_local_addend_comes_first(oracle):
    """sum = local + deq_0 + deq_1 ...: equals the plain reduce when local is -0, and
    equals numpy's ordered binary32 sum of the separately dequantized terms."""
    w = wl.tiny_mixed(seed=12)
    chunks, metas = zip(*[oracle.quantize(w.gradient(p), w.offsets, w.bits, w.bucket, p) for p in range(3)])
    plain = oracle.dequant_reduce(list(chunks), list(metas), w.offsets, w.bits, w.bucket)
    zero = np.full(w.n, -0.0, np.float32)
    same = oracle.dequant_reduce(list(chunks), list(metas), w.offsets, w.bits, w.bucket, local=zero)
    assert np.array_equal(plain["sum32"].view(np.uint32), same["sum32"].view(np.uint32))
    for local in (w.gradient(7), w.gradient(7).astype(np.float16)):
        got = oracle.dequant_reduce(list(chunks), list(metas), w.offsets, w.bits, w.bucket, local=local)
        terms = [oracle.dequantize(c, m, w.offsets, w.bits, w.bucket) for c, m in zip(chunks, metas)]
        acc = local.astype(np.float32)
        acc64 = local.astype(np.float64)
        for t in terms:
            acc = acc + t
        assert np.array_equal(got["sum32"], acc)
        approx = acc64 + sum(t.astype(np.float64) for t in terms)          # terms rounded to binary32 once
        assert (np.abs(got["sum64"] - approx) <= 1e-6 * got["abs64"] + 1e-30).all()


def test_window_of_a_buffer_equals_the_slice_of_the_whole(oracle):
    """Quantizing elements [a, b) of a layer as a window (bucket aligned) gives the bytes the
    whole buffer gives for that range."""
    rng = np.random.default_rng(3)
    n, B, b = 64 * 40, 64, 3
    x = rng.standard_normal(n).astype(np.float32)
    off, bits = one_layer(n, b)
    p, m = oracle.quantize(x, off, bits, B, seed=17)
    a, e = 64 * 7, 64 * 23
    pw, mw = oracle.quantize(x[a:e], *one_layer(e - a, b), B, seed=17, index_base=a)
    assert np.array_equal(pw[:(e - a) * b // 8], p[a * b // 8:e * b // 8])
    assert mw.tobytes() == m[a // B:e // B].tobytes()


def test_oracle_is_deterministic_and_thread_independent(oracle):
    w = wl.tiny_mixed(seed=1)
    g = w.gradient()
    oracle.set_threads(1)
    a = oracle.quantize(g, w.offsets, w.bits, w.bucket, seed=77)
    oracle.set_threads(4)
    b = oracle.quantize(g, w.offsets, w.bits, w.bucket, seed=77)
    c = oracle.quantize(g, w.offsets, w.bits, w.bucket, seed=78)
    assert np.array_equal(a[0], b[0]) and a[1].tobytes() == b[1].tobytes()
    assert not np.array_equal(a[0], c[0]) and a[1].tobytes() == c[1].tobytes()   # seed moves codes, not meta


# ------------------------------------------------------------------ generator quality

def chi2_uniform(counts):
    e = counts.sum() / counts.size
    return ((counts - e) ** 2 / e).sum()


@pytest.mark.parametrize("seed", [0, 1, 2**40 + 12345])
def test_draws_are_uniform_and_uncorrelated(oracle, seed):
    n = 1 << 21
    u = oracle.draws(seed, 0, n).astype(np.int64)
    assert u.min() >= 0 and u.max() <= 65535
    for part in (u >> 8, u & 0xff):                          # 255 d.o.f.: mean 255, sd 22.6
        assert chi2_uniform(np.bincount(part, minlength=256)) < 255 + 6 * 22.6
    assert chi2_uniform(np.bincount(u, minlength=65536)) < 65535 + 6 * 362     # sd = sqrt(2*65535)
    v = u / 65536.0 - 0.5
    for lag in (1, 2, 3, 7, 64, 128, 1024):
        r = np.mean(v[:-lag] * v[lag:]) * 12
        assert abs(r) < 5 / np.sqrt(n)
    assert abs(np.mean(v[0::2] * v[1::2]) * 12) < 5 / np.sqrt(n / 2)   # two halves of one word
    other = oracle.draws(seed + 1, 0, n).astype(np.int64) / 65536.0 - 0.5
    assert abs(np.mean(v * other) * 12) < 5 / np.sqrt(n)
    # joint law of neighbouring draws, 16 x 16 cells
    cells = np.bincount((u[0::2] >> 12) * 16 + (u[1::2] >> 12), minlength=256)
    assert chi2_uniform(cells) < 255 + 6 * 22.6


def test_draws_depend_on_the_element_index_only(oracle):
    a = oracle.draws(5, 0, 4096)
    b = oracle.draws(5, 1001, 1000)
    assert np.array_equal(a[1001:2001], b)
    hi = oracle.draws(5, (1 << 33) - 50, 100)              # across the 2^32-pair boundary
    assert len(set(hi.tolist())) > 90
    assert not np.array_equal(hi[:50], oracle.draws(5, (1 << 34) - 50, 50))


def test_generator_avalanche(oracle):
    rng = np.random.default_rng(1)
    flips = []
    for _ in range(300):
        seed = int(rng.integers(0, 2**63))
        pair = int(rng.integers(0, 2**40))
        base = oracle.rng32(seed, pair)
        for bit in range(40):
            flips.append(bin(base ^ oracle.rng32(seed, pair ^ (1 << bit))).count("1"))
        for bit in range(64):
            flips.append(bin(base ^ oracle.rng32(seed ^ (1 << bit), pair)).count("1"))
    flips = np.array(flips)
    assert 15.5 < flips.mean() < 16.5
    assert flips.min() >= 3


def test_generator_equals_its_written_specification(oracle):
    """The generator restated in Python from its specification: one 32-bit word per element pair,
    r = mix(pair_lo ^ key), key = mix(seed_lo ^ mix(seed_hi ^ 0x9e3779b9 ^ pair_hi)), mix = xor-shift 16,
    times 0x7feb352d, xor-shift 15, times 0x846ca68b, xor-shift 16; even elements take the low half."""
    M = 0xffffffff

    def mix(x):
        x ^= x >> 16
        x = (x * 0x7feb352d) & M
        x ^= x >> 15
        x = (x * 0x846ca68b) & M
        return x ^ (x >> 16)

    def word(seed, pair):
        key = mix((seed & M) ^ mix(((seed >> 32) & M) ^ 0x9e3779b9 ^ ((pair >> 32) & M)))
        return mix((pair & M) ^ key)

    rng = np.random.default_rng(77)
    seeds = [0, 1, 2**32 - 1, 2**32, 2**64 - 1] + [int(s) for s in rng.integers(0, 2**63, 20)]
    idx = [0, 1, 2, 3, 2**32 - 1, 2**32, 2**33 - 2, 2**33 - 1, 2**33, 2**33 + 1, 2**40 + 5, 2**63 + 1] + \
          [int(i) for i in rng.integers(0, 2**62, 50)]
    for s in seeds:
        for i in idx:
            r = word(s, i >> 1)
            assert oracle.rng32(s, i >> 1) == r
            assert oracle.u16(s, i) == ((r >> 16) if i & 1 else (r & 0xffff))
    d = oracle.draws(12345, 2**33 - 8, 16)                       # a run across a key-block boundary
    assert [int(v) for v in d] == [oracle.u16(12345, 2**33 - 8 + k) for k in range(16)]
