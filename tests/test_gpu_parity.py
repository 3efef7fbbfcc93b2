"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element.

Bar: packed stream and meta bit-exact; reduced sums bit-exact against the
oracle's ordered binary32 sum and within 1e-6 * sum_w |deq_w| of its binary64
sum.  Inputs are seeded and synthetic (paper_2111_08617_amd.workloads); inputs of
the reduce step come from the oracle's quantizer, never from the GPU.
"""
import numpy as np
import pytest

from paper_2111_08617_amd import binding as cgx
from paper_2111_08617_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "these tests need the MI355X"
    cgx.lib()                       # fails loudly if libcgx.so has not been built
    return t


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_quantize(torch, grad, offsets, bits, bucket, seed, dt, requant=False):
    plan = cgx.Plan(offsets, bits, bucket, dt)
    pb, mb = cgx.cgx_sizes(plan)
    # canaries after the buffers catch writes past the sizes cgx_sizes reports
    packed = torch.full((pb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    meta = torch.full((mb // 4 + 16,), -7.0, dtype=torch.float32, device="cuda")
    g = grad if isinstance(grad, torch.Tensor) else dev(torch, grad)
    if requant:
        cgx.cgx_requantize(g, plan, seed, packed, meta)
    else:
        cgx.cgx_quantize(g, plan, seed, packed, meta)
    torch.cuda.synchronize()
    p, m = packed.cpu().numpy(), meta.cpu().numpy()
    assert (p[pb:] == 0xA5).all() and (m[mb // 4:] == -7.0).all(), "wrote past the reported sizes"
    return p[:pb], m[:mb // 4].reshape(-1, 2)


def gpu_reduce(torch, chunks, metas, offsets, bits, bucket, dt):
    plan = cgx.Plan(offsets, bits, bucket, dt)
    dp = [dev(torch, c) for c in chunks]
    dm = [dev(torch, m.reshape(-1)) if m.size else torch.zeros(4, device="cuda") for m in metas]
    total = torch.full((plan.n + 16,), 123.0, dtype=torch.float32, device="cuda")
    cgx.cgx_dequant_reduce(dp, dm, plan, total)
    torch.cuda.synchronize()
    out = total.cpu().numpy()
    assert (out[plan.n:] == 123.0).all(), "wrote past the end of the sum"
    return out[:plan.n], total


def gpu_fused(torch, chunks, metas, offsets, bits, bucket, dt, seed):
    """cgx_dequant_reduce_requantize on host-made chunks; returns (packed, meta) of the requantized sum."""
    plan = cgx.Plan(offsets, bits, bucket, dt)
    pb, mb = cgx.cgx_sizes(cgx.Plan(offsets, bits, bucket, wl.F32))
    dp = [dev(torch, c) for c in chunks]
    dm = [dev(torch, m.reshape(-1)) if m.size else torch.zeros(4, device="cuda") for m in metas]
    packed = torch.full((pb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    meta = torch.full((mb // 4 + 16,), -7.0, dtype=torch.float32, device="cuda")
    cgx.cgx_dequant_reduce_requantize(dp, dm, plan, seed, packed, meta)
    torch.cuda.synchronize()
    p, m = packed.cpu().numpy(), meta.cpu().numpy()
    assert (p[pb:] == 0xA5).all() and (m[mb // 4:] == -7.0).all(), "wrote past the reported sizes"
    return p[:pb], m[:mb // 4].reshape(-1, 2)


def assert_same_chunk(gp, gm, op, om, what=""):
    assert gm.tobytes() == om.tobytes(), f"{what}: meta differs in {int((gm.view(np.uint32) != om.view(np.uint32)).sum())} words"
    if not np.array_equal(gp, op):
        bad = np.nonzero(gp != op)[0]
        raise AssertionError(f"{what}: packed differs in {bad.size} bytes, first at {bad[:5]}")


def assert_sum_parity(got, ref, what=""):
    g, r = got.view(np.uint32), ref["sum32"].view(np.uint32)
    assert np.array_equal(g, r), f"{what}: {int((g != r).sum())} sums differ from the ordered binary32 sum"
    err = np.abs(got.astype(np.float64) - ref["sum64"])
    assert (err <= 1e-6 * ref["abs64"] + 1e-45).all(), f"{what}: worst relative error {np.max(err / (ref['abs64'] + 1e-300))}"


def full_cycle(torch, oracle, w, W, seed_shift=0, what=""):
    """quantize, reduce over W oracle-made chunks, requantize of the GPU's own sum."""
    chunks, metas = [], []
    for peer in range(W):
        g = w.gradient(peer)
        seed = w.quant_seed(peer) + seed_shift
        op, om = oracle.quantize(g, w.offsets, w.bits, w.bucket, seed, w.dt)
        if peer < 2:
            gp, gm = gpu_quantize(torch, g, w.offsets, w.bits, w.bucket, seed, w.dt)
            assert_same_chunk(gp, gm, op, om, f"{what} quantize peer {peer}")
        chunks.append(op)
        metas.append(om)
    ref = oracle.dequant_reduce(chunks, metas, w.offsets, w.bits, w.bucket, w.dt)
    got, total = gpu_reduce(torch, chunks, metas, w.offsets, w.bits, w.bucket, w.dt)
    assert_sum_parity(got, ref, f"{what} reduce")
    # decompression of one chunk into either storage type (canaries behind the output)
    plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
    dp0, dm0 = dev(torch, chunks[0]), (dev(torch, metas[0].reshape(-1)) if metas[0].size else torch.zeros(4, device="cuda"))
    for out_dt, tdt in ((wl.F32, torch.float32), (wl.F16, torch.float16)):
        out = torch.full((w.n + 16,), 9.0, dtype=tdt, device="cuda")
        cgx.cgx_dequantize(dp0, dm0, plan, out_dt, out)
        torch.cuda.synchronize()
        o = out.cpu().numpy()
        assert (o[w.n:] == 9.0).all(), f"{what}: dequantize wrote past the end"
        want = oracle.dequantize(chunks[0], metas[0], w.offsets, w.bits, w.bucket, w.dt, out_dt)
        assert o[:w.n].tobytes() == want.tobytes(), f"{what}: dequantize to {'f16' if out_dt else 'f32'}"
    # requantize: the definition is quantize(sum) on binary32 input, so compare on the GPU's own sum
    rp, rm = gpu_quantize(torch, total[:w.n], w.offsets, w.bits, w.bucket, 99 + seed_shift, wl.F32, requant=True)
    op, om = oracle.quantize(got, w.offsets, w.bits, w.bucket, 99 + seed_shift, wl.F32)
    assert_same_chunk(rp, rm, op, om, f"{what} requantize")
    # fused reduce + requantize: expected value from the oracle alone (its ordered binary32 sum, quantized)
    if W <= cgx.MAX_FUSED_PEERS:
        fp, fm = gpu_fused(torch, chunks, metas, w.offsets, w.bits, w.bucket, w.dt, 99 + seed_shift)
        op, om = oracle.quantize(ref["sum32"], w.offsets, w.bits, w.bucket, 99 + seed_shift, wl.F32)
        assert_same_chunk(fp, fm, op, om, f"{what} fused reduce+requantize")


@pytest.mark.parametrize("dt", [wl.F32, wl.F16], ids=["f32", "f16"])
@pytest.mark.parametrize("bucket", [32, 64, 96, 128, 512, 2048, 4096, 8192])
def test_edge_case_plan(torch, oracle, bucket, dt):
    """All bit widths, pass-through, empty, tiny and ragged layers, odd offsets."""
    w = wl.tiny_mixed(seed=bucket + dt, dt=dt, bucket=bucket)
    full_cycle(torch, oracle, w, W=3, what=f"tiny_mixed B={bucket}")


@pytest.mark.parametrize("dt", [wl.F32, wl.F16], ids=["f32", "f16"])
@pytest.mark.parametrize("bucket", [32, 64, 128, 256, 512, 1024, 2048])
def test_vectorised_path_all_bit_widths(torch, oracle, bucket, dt):
    """Aligned layers of whole chunks (the fast tiles) plus ragged tails, every bit width."""
    sizes = [2048 * 3, 2048 * 2 + 40, 8, 2048, 2048 * 5 + 1000, 2048 * 4, 16384, 2048 + bucket, 6144, 8192 * 2 + 24]
    bits = [1, 2, 0, 3, 4, 5, 0, 6, 7, 8]
    w = wl.Workload("chunks", [(s,) for s in sizes], np.array(bits, np.uint8), bucket, dt, 4, 1000 + bucket,
                    wl._normal, np.linspace(0.01, 2.0, len(sizes)))
    plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
    kinds = (cgx.cgx_plan_tiles(plan)["info"] >> 4) & 15
    assert (kinds == 1).sum() >= 20 and (kinds == 3).any() and (kinds == 5).any()
    full_cycle(torch, oracle, w, W=4, what=f"chunks B={bucket}")


@pytest.mark.parametrize("dt", [wl.F32, wl.F16], ids=["f32", "f16"])
@pytest.mark.parametrize("bucket", [96, 160, 224, 672, 992, 1056, 2016, 2080])
def test_bucket_sizes_that_are_no_power_of_two(torch, oracle, bucket, dt):
    """Multiples of 32 that are no power of two: whole buckets stream row by row (tile kind 6), only the ragged
    end of a layer and sizes above the chunk stay on the generic path; every bit width, layers of whole
    buckets, ragged layers, layers that start on odd elements, pass-through layers in between; then the same
    chunks through cgx_dequantize (binary16 out) and the reduce with a local addend."""
    sizes = [bucket * 21, bucket * 3 + 40, 8, bucket, bucket * 40 + 1000, bucket * 7 + 1, 500, bucket * 2 + bucket // 2,
             bucket * 64, bucket * 5]
    bits = [1, 2, 0, 3, 4, 5, 0, 6, 7, 8]
    w = wl.Workload("anysize", [(s,) for s in sizes], np.array(bits, np.uint8), bucket, dt, 5, 3000 + bucket,
                    wl._normal, np.linspace(0.01, 2.0, len(sizes)))
    plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
    for chunk in (1024, 2048):
        kinds = (cgx.cgx_plan_tiles(plan, chunk)["info"] >> 4) & 15
        if bucket <= chunk:
            assert (kinds == 6).sum() >= 8 and (kinds == 0).sum() <= 5       # generic: the ragged ends only
        else:
            assert not (kinds == 6).any()
    full_cycle(torch, oracle, w, W=5, what=f"any-size B={bucket}")
    chunks = [oracle.quantize(w.gradient(p), w.offsets, w.bits, bucket, w.quant_seed(p), dt) for p in range(3)]
    dp = [dev(torch, c[0]) for c in chunks]
    dm = [dev(torch, c[1].reshape(-1)) for c in chunks]
    out16 = torch.zeros(w.n, dtype=torch.float16, device="cuda")
    cgx.cgx_dequantize(dp[0], dm[0], plan, wl.F16, out16)
    local = dev(torch, w.gradient(7))
    total = torch.zeros(w.n, device="cuda")
    cgx.cgx_dequant_reduce_add(local, dt, dp, dm, plan, total)
    torch.cuda.synchronize()
    one = oracle.dequant_reduce([chunks[0][0]], [chunks[0][1]], w.offsets, w.bits, bucket, dt)["sum32"]
    assert np.array_equal(out16.cpu().numpy().view(np.uint16), oracle.float_to_half(one))
    ref = oracle.dequant_reduce([c[0] for c in chunks], [c[1] for c in chunks], w.offsets, w.bits, bucket, dt,
                                local=w.gradient(7))
    assert np.array_equal(total.cpu().numpy().view(np.uint32), ref["sum32"].view(np.uint32))


def test_single_tensor_config(torch, oracle):
    """2^20 elements ~ N(0, 0.01^2), 4 bit, bucket 128, seed 0, reduce over W = 2."""
    w = wl.single_tensor(seed=0)
    full_cycle(torch, oracle, w, W=2, what="single_1m")


def test_many_peers_take_several_launches(torch, oracle):
    w = wl.tiny_mixed(seed=77, bucket=128)
    for W in (1, 16, 17, 37, 64):
        chunks, metas = zip(*[oracle.quantize(w.gradient(p), w.offsets, w.bits, w.bucket, p) for p in range(W)])
        ref = oracle.dequant_reduce(list(chunks), list(metas), w.offsets, w.bits, w.bucket)
        got, _ = gpu_reduce(torch, chunks, metas, w.offsets, w.bits, w.bucket, w.dt)
        assert_sum_parity(got, ref, f"W={W}")


def test_fused_peer_counts(torch, oracle):
    """Every chunk count the fused entry point accepts, on the edge-case plan in binary16 storage."""
    w = wl.tiny_mixed(seed=91, dt=wl.F16, bucket=64)
    chunks, metas = zip(*[oracle.quantize(w.gradient(p), w.offsets, w.bits, w.bucket, p, w.dt) for p in range(16)])
    for W in (1, 2, 3, 5, 8, 11, 16):
        ref = oracle.dequant_reduce(list(chunks[:W]), list(metas[:W]), w.offsets, w.bits, w.bucket, w.dt)
        fp, fm = gpu_fused(torch, chunks[:W], metas[:W], w.offsets, w.bits, w.bucket, w.dt, 1000 + W)
        op, om = oracle.quantize(ref["sum32"], w.offsets, w.bits, w.bucket, 1000 + W, wl.F32)
        assert_same_chunk(fp, fm, op, om, f"fused W={W}")
    with pytest.raises(cgx.CgxError):
        gpu_fused(torch, list(chunks) + [chunks[0]], list(metas) + [metas[0]], w.offsets, w.bits, w.bucket, w.dt, 1)


@pytest.mark.parametrize("dt", [wl.F32, wl.F16], ids=["f32", "f16"])
def test_dequantize_and_local_addend(torch, oracle, dt):
    """cgx_dequantize into binary32 / binary16 and cgx_dequant_reduce_add with a binary32 / binary16
    local term, on a plan with vectorised, generic and pass-through tiles."""
    sizes = [2048 * 3, 100, 2048 + 700, 8, 4096, 33, 2048 * 2]
    bits = [4, 0, 3, 0, 8, 2, 1]
    w = wl.Workload("mix", [(s,) for s in sizes], np.array(bits, np.uint8), 128, dt, 4, 321, wl._normal,
                    np.linspace(0.01, 2.0, len(sizes)))
    plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
    chunks, metas = zip(*[oracle.quantize(w.gradient(p), w.offsets, w.bits, w.bucket, 50 + p, w.dt) for p in range(20)])
    dp = [dev(torch, c) for c in chunks]
    dm = [dev(torch, m.reshape(-1)) for m in metas]
    for out_dt, tdt in ((wl.F32, torch.float32), (wl.F16, torch.float16)):
        out = torch.full((w.n + 16,), 9.0, dtype=tdt, device="cuda")
        cgx.cgx_dequantize(dp[0], dm[0], plan, out_dt, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert (got[w.n:] == 9.0).all()
        want = oracle.dequantize(chunks[0], metas[0], w.offsets, w.bits, w.bucket, w.dt, out_dt)
        assert got[:w.n].tobytes() == want.tobytes(), f"dequantize to {'f16' if out_dt else 'f32'}"
    for W in (3, 20):
        for local in (w.gradient(99).astype(np.float32), w.gradient(99).astype(np.float16)):
            total = torch.full((w.n + 16,), 9.0, dtype=torch.float32, device="cuda")
            cgx.cgx_dequant_reduce_add(dev(torch, local), wl.F16 if local.dtype == np.float16 else wl.F32,
                                       dp[:W], dm[:W], plan, total)
            torch.cuda.synchronize()
            got = total.cpu().numpy()
            assert (got[w.n:] == 9.0).all()
            ref = oracle.dequant_reduce(list(chunks[:W]), list(metas[:W]), w.offsets, w.bits, w.bucket, w.dt, local=local)
            assert_sum_parity(got[:w.n], ref, f"local addend W={W} {local.dtype}")


def test_degenerate_values(torch, oracle):
    """Constant, zero, signed-zero, subnormal and huge buckets; exact grids."""
    B, n = 128, 128 * 24
    rng = np.random.default_rng(4)
    x = rng.standard_normal(n).astype(np.float32)
    x[0:128] = 0.37
    x[128:256] = 0.0
    x[130] = -0.0
    x[256:384] = -0.0
    x[384:512] = 1e-42
    x[512:640] = np.float32(1e-42) * rng.integers(0, 50, 128).astype(np.float32)     # subnormal range
    x[640:768] = rng.standard_normal(128).astype(np.float32) * np.float32(1e37)      # near the top of the range
    x[768:896] = np.float32(-3.25) + rng.integers(0, 16, 128).astype(np.float32) * np.float32(2.0 ** -7)
    x[768], x[769] = np.float32(-3.25), np.float32(-3.25) + np.float32(15 * 2.0 ** -7)
    x[896:1024] = np.abs(x[896:1024])
    x[896] = -0.0                                            # minimum is -0 with positive values
    x[1024:1152] = np.float32(1e-30) * rng.standard_normal(128).astype(np.float32)
    x[1152:1280] = np.float32(1.0) + np.float32(2.0 ** -23) * rng.integers(0, 3, 128).astype(np.float32)
    for b in (1, 2, 3, 4, 8):
        off, bits = np.array([0, n], np.int64), np.array([b], np.uint8)
        for seed in (0, 2**64 - 1, 2**32, 12345678901234567):
            gp, gm = gpu_quantize(torch, x, off, bits, B, seed, wl.F32)
            op, om = oracle.quantize(x, off, bits, B, seed, wl.F32)
            assert_same_chunk(gp, gm, op, om, f"degenerate b={b} seed={seed}")
        got, _ = gpu_reduce(torch, [op, op], [om, om], off, bits, B, wl.F32)
        assert_sum_parity(got, oracle.dequant_reduce([op, op], [om, om], off, bits, B), f"degenerate b={b}")
    # binary16 storage with subnormal halves
    h = (rng.standard_normal(4096) * 1e-3).astype(np.float16)
    h[:64] = np.arange(64, dtype=np.float32) * np.float32(6e-8)
    h[2048:2048 + 128] = 0
    off, bits = np.array([0, 4096], np.int64), np.array([4], np.uint8)
    gp, gm = gpu_quantize(torch, h, off, bits, 128, 5, wl.F16)
    op, om = oracle.quantize(h, off, bits, 128, 5, wl.F16)
    assert_same_chunk(gp, gm, op, om, "binary16 subnormals")


@pytest.mark.parametrize("b", [2, 4, 8])
def test_units_at_both_ends_of_the_exponent_range(torch, oracle, b):
    """Chunks whose buckets' units are huge (on both sides of 2^118, where the fused kernel's scaled unit
    starts to overflow and it falls back to the plain conversion), tiny (subnormal units) or ordinary, in
    different peers: the reduce and the fused call, whole chunks and a short end."""
    B, n, W = 256, 2048 * 4 + 1200, 5
    off, bits = np.array([0, n], np.int64), np.array([b], np.uint8)
    rng = np.random.default_rng(100 + b)
    top = float(2 ** b - 1)
    chunks, metas = [], []
    for peer in range(W):
        x = rng.standard_normal(n).astype(np.float32)
        scale = np.ones(n // B + 1, np.float32)
        kinds = rng.integers(0, 6, scale.size)
        scale[kinds == 0] = np.float32(2.0 ** 114 * top)        # units around 2^117 ...
        scale[kinds == 1] = np.float32(2.0 ** 116 * top)        # ... and around 2^119
        scale[kinds == 2] = np.float32(2.0 ** 100)
        scale[kinds == 3] = np.float32(2.0 ** -140)             # subnormal unit
        x *= np.repeat(scale, B)[:n]
        if peer == 3:
            x = rng.standard_normal(n).astype(np.float32)      # one peer with ordinary values everywhere
        op, om = oracle.quantize(x, off, bits, B, 7 + peer, wl.F32)
        chunks.append(op)
        metas.append(om)
    units = np.concatenate([m[:, 0] for m in metas])
    assert (units >= 2.0 ** 118).any() and ((units > 2.0 ** 110) & (units < 2.0 ** 118)).any()
    assert (units < 2.0 ** -126).any() and ((units > 1e-3) & (units < 10)).any()
    ref = oracle.dequant_reduce(chunks, metas, off, bits, B, wl.F32)
    got, _ = gpu_reduce(torch, chunks, metas, off, bits, B, wl.F32)
    assert np.array_equal(got.view(np.uint32), ref["sum32"].view(np.uint32)), "reduce"
    fp, fm = gpu_fused(torch, chunks, metas, off, bits, B, wl.F32, 31)
    op, om = oracle.quantize(ref["sum32"], off, bits, B, 31, wl.F32)
    assert_same_chunk(fp, fm, op, om, "fused")


def test_repeatable_and_seed_sensitive(torch, oracle):
    w = wl.tiny_mixed(seed=5, bucket=256)
    g = w.gradient()
    a = gpu_quantize(torch, g, w.offsets, w.bits, w.bucket, 42, w.dt)
    b = gpu_quantize(torch, g, w.offsets, w.bits, w.bucket, 42, w.dt)
    c = gpu_quantize(torch, g, w.offsets, w.bits, w.bucket, 43, w.dt)
    assert np.array_equal(a[0], b[0]) and a[1].tobytes() == b[1].tobytes()
    assert not np.array_equal(a[0], c[0]) and a[1].tobytes() == c[1].tobytes()


def test_non_default_stream(torch, oracle):
    w = wl.tiny_mixed(seed=6, bucket=128)
    g = w.gradient()
    plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
    pb, mb = cgx.cgx_sizes(plan)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        dg = dev(torch, g)
        packed = torch.empty(pb, dtype=torch.uint8, device="cuda")
        meta = torch.empty(mb // 4, dtype=torch.float32, device="cuda")
        cgx.cgx_quantize(dg, plan, 3, packed, meta, stream=s)
    s.synchronize()
    op, om = oracle.quantize(g, w.offsets, w.bits, w.bucket, 3)
    assert_same_chunk(packed.cpu().numpy(), meta.cpu().numpy().reshape(-1, 2), op, om, "side stream")


def test_resnet50_config_full_size(torch, oracle):
    """161 tensors, 25.6M elements, 4 bit, bucket 1024, small tensors pass-through, W = 8."""
    w = wl.resnet50()
    full_cycle(torch, oracle, w, W=8, what="resnet50")


def test_bert_base_config_full_size(torch, oracle):
    """199 tensors, 109M elements, bits in {2,3,4,8}, bucket 512; reduce over W = 8 on a 1/8 share."""
    w = wl.bert_base()
    g = w.gradient(0)
    gp, gm = gpu_quantize(torch, g, w.offsets, w.bits, w.bucket, w.quant_seed(0), w.dt)
    op, om = oracle.quantize(g, w.offsets, w.bits, w.bucket, w.quant_seed(0), w.dt)
    assert_same_chunk(gp, gm, op, om, "bert_base quantize")
    del g, gp, op
    share_cycle(torch, oracle, w, rank=3, what="bert_base")


def share_cycle(torch, oracle, w, rank, what):
    """Reduce and requantize on one rank's share of a W-way scatter-reduce."""
    first, sub_off, sub_bits = wl.share_subplan(w.offsets, w.bits, w.bucket, w.W, rank)
    m = int(sub_off[-1])
    chunks, metas = [], []
    for peer in range(w.W):
        g = w.gradient(peer, first, first + m)
        op, om = oracle.quantize(g, sub_off, sub_bits, w.bucket, w.quant_seed(peer), w.dt)
        chunks.append(op)
        metas.append(om)
    ref = oracle.dequant_reduce(chunks, metas, sub_off, sub_bits, w.bucket, w.dt)
    got, total = gpu_reduce(torch, chunks, metas, sub_off, sub_bits, w.bucket, w.dt)
    assert_sum_parity(got, ref, f"{what} share reduce")
    rp, rm = gpu_quantize(torch, total[:m], sub_off, sub_bits, w.bucket, 7, wl.F32, requant=True)
    op, om = oracle.quantize(got, sub_off, sub_bits, w.bucket, 7, wl.F32)
    assert_same_chunk(rp, rm, op, om, f"{what} share requantize")
    del rp, got, total
    fp, fm = gpu_fused(torch, chunks, metas, sub_off, sub_bits, w.bucket, w.dt, 7)
    op, om = oracle.quantize(ref["sum32"], sub_off, sub_bits, w.bucket, 7, wl.F32)
    assert_same_chunk(fp, fm, op, om, f"{what} share fused reduce+requantize")


def test_gpt2_medium_config_full_size(torch, oracle):
    """292 tensors, 355M elements in binary16 storage, 20% exact zeros, 4 bit, bucket 128:
    quantize the full buffer; reduce over W = 8 and requantize on one rank's 1/8 share."""
    w = wl.gpt2_medium()
    g = w.gradient(0, threads=16)
    gp, gm = gpu_quantize(torch, g, w.offsets, w.bits, w.bucket, w.quant_seed(0), w.dt)
    op, om = oracle.quantize(g, w.offsets, w.bits, w.bucket, w.quant_seed(0), w.dt)
    assert_same_chunk(gp, gm, op, om, "gpt2_medium quantize")
    del g, gp, op
    share_cycle(torch, oracle, w, rank=5, what="gpt2_medium")


@pytest.mark.parametrize("bucket", [64, 128, 1024, 4096])
def test_binary16_buffers_that_take_tiles_of_two_chunks(torch, oracle, bucket):
    """cgx_quantize joins chunks into longer tiles on binary16 gradients of 2^24 elements or
    more: layers of an odd number of chunks, with short ends, an odd start, a pass-through
    layer and all widths in one buffer give the same bytes as the oracle; the reduce and the
    fused step of the same plan (tiles of one chunk) agree too."""
    shapes = [(2048 * 3001 + 77,), (1,), (2048 * 2000,), (999,), (2048 * 1501 + 1024,), (2048 * 1700 + 5,)]
    bits = np.array([4, 0, 3, 0, 2, 8], np.uint8)
    w = wl.Workload("f16long", shapes, bits, bucket, wl.F16, 2, 11, wl._normal, np.array([1.0, 1.0, 0.01, 1.0, 3.0, 1e-3]))
    assert w.n >= 1 << 24
    full_cycle(torch, oracle, w, W=2, what="f16long")


@pytest.mark.parametrize("seed", range(24))
def test_random_plans(torch, oracle, seed):
    """Seeded random plans through the whole cycle (quantize, reduce, requantize, fused)."""
    w = wl.random_plan(seed)
    if w.n == 0:
        pytest.skip("empty plan (covered by the edge cases)")
    full_cycle(torch, oracle, w, W=w.W, what=f"random plan {seed} (bucket {w.bucket}, bits {w.bits.tolist()})")


@pytest.mark.parametrize("seed", range(48))
def test_random_plans_with_any_legal_bucket_size(torch, oracle, seed):
    """The same random plans with the bucket size drawn from all multiples of 32 up to 2176 (whole-bucket
    tiles that are no power of two, sizes just above a chunk) and now and then from the rest up to 8192."""
    w = wl.random_plan(500 + seed)
    if w.n == 0:
        pytest.skip("empty plan (covered by the edge cases)")
    rng = np.random.default_rng(900 + seed)
    w.bucket = int(32 * rng.integers(1, 69)) if seed % 6 else int(32 * rng.integers(69, 257))
    full_cycle(torch, oracle, w, W=min(w.W, 5), what=f"random plan {500 + seed} (bucket {w.bucket}, bits {w.bits.tolist()})")


@pytest.mark.parametrize("bucket,dt", [(96, wl.F32), (992, wl.F16), (2016, wl.F32)], ids=["96-f32", "992-f16", "2016-f32"])
def test_long_buffers_with_bucket_sizes_that_are_no_power_of_two(torch, oracle, bucket, dt):
    """Tens of thousands of streamed tiles per launch: layers of millions of elements, every width."""
    rng = np.random.default_rng(bucket)
    sizes = [int(rng.integers(1 << 20, 1 << 22)) for _ in range(5)] + [(1 << 23) + 12345]
    bits = np.array([4, 2, 8, 3, 0, 5], np.uint8)
    w = wl.Workload("long", [(s,) for s in sizes], bits, bucket, dt, 3, 40 + bucket, wl._normal,
                    10.0 ** rng.uniform(-3, 0, len(sizes)))
    plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
    kinds = (cgx.cgx_plan_tiles(plan)["info"] >> 4) & 15
    assert (kinds == 6).sum() > 5000
    full_cycle(torch, oracle, w, W=w.W, what=f"long B={bucket}")


def test_decoder_1p3b_config_full_size(torch, oracle):
    """292 tensors, 1.316G elements, Laplace values with outliers, bits in {2,4,8}, bucket 1024:
    quantize the full buffer (the launch bench.py times); reduce over W = 8 and requantize on
    one rank's 1/8 share."""
    w = wl.decoder_1p3b()
    g = w.gradient(0, threads=16)
    gp, gm = gpu_quantize(torch, g, w.offsets, w.bits, w.bucket, w.quant_seed(0), w.dt)
    op, om = oracle.quantize(g, w.offsets, w.bits, w.bucket, w.quant_seed(0), w.dt)
    assert_same_chunk(gp, gm, op, om, "decoder_1p3b quantize")
    del g, gp, op
    share_cycle(torch, oracle, w, rank=4, what="decoder_1p3b")


def test_indices_beyond_2_to_33(torch, oracle):
    """Maximum sizes: a binary16 buffer of 2^33 + 3 M elements.  Element indices need more than
    32 bits, the generator's key changes at element 2^33, and one tile straddles that point
    (it takes the generic path).  Windows at the start, around 2^33 and at the ragged end are
    compared with the oracle run on the same slices."""
    B, b, seed = 1024, 2, 2**40 + 7
    head = 1024                                   # shifts the big layer so that 2^33 falls inside a chunk
    n = (1 << 33) + 3 * (1 << 20) + 1000
    offsets = np.array([0, head, n], np.int64)
    bits = np.array([4, b], np.uint8)
    plan = cgx.Plan(offsets, bits, B, wl.F16)
    tiles = cgx.cgx_plan_tiles(plan)
    straddle = tiles[(tiles["elem0"] < (1 << 33)) & (tiles["elem0"] + tiles["count"].astype(np.int64) > (1 << 33))]
    assert straddle.size == 1 and (int(straddle["info"][0]) >> 4) & 15 == 0
    grad = torch.empty(n, dtype=torch.float16, device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(5)
    step = 1 << 28
    for a in range(0, n, step):
        e = min(a + step, n)
        grad[a:e] = torch.randn(e - a, device="cuda", generator=gen, dtype=torch.float32).to(torch.float16)
    pb, mb = cgx.cgx_sizes(plan)
    packed = torch.empty(pb, dtype=torch.uint8, device="cuda")
    meta = torch.empty(mb // 4, dtype=torch.float32, device="cuda")
    cgx.cgx_quantize(grad, plan, seed, packed, meta)
    torch.cuda.synchronize()
    seg1 = head * 4 // 8                          # first layer: 512 bytes, already a multiple of 16
    windows = [(head, head + (1 << 20)), ((1 << 33) - (1 << 20) + head, (1 << 33) + (1 << 20) + head),
               (n - ((n - head) % B) - 512 * B, n)]
    for a, e in windows:
        assert (a - head) % B == 0
        x = grad[a:e].cpu().numpy()
        op, om = oracle.quantize(x, np.array([0, e - a], np.int64), np.array([b], np.uint8), B, seed, wl.F16,
                                 index_base=a)
        nbytes = -(-(e - a) * b // 8)
        lo = seg1 + (a - head) * b // 8
        gp = packed[lo:lo + nbytes].cpu().numpy()
        g0 = 1 + (a - head) // B                  # one bucket in the first layer
        gm = meta[2 * g0:2 * (g0 + om.shape[0])].cpu().numpy().reshape(-1, 2)
        assert_same_chunk(gp, gm, op[:nbytes], om, f"window [{a}, {e})")
    # the reduce side reads the same positions: dequantize the last window's chunk region and compare
    del grad
    out = torch.empty(n, dtype=torch.float16, device="cuda")
    cgx.cgx_dequantize(packed, meta, plan, wl.F16, out)
    torch.cuda.synchronize()
    a, e = windows[1]
    x_codes = packed[seg1 + (a - head) * b // 8: seg1 + (e - head) * b // 8].cpu().numpy()
    m_win = meta[2 * (1 + (a - head) // B):2 * (1 + (e - head) // B)].cpu().numpy().reshape(-1, 2)
    want = oracle.dequantize(np.concatenate([x_codes, np.zeros((-x_codes.size) % 16, np.uint8)]), m_win,
                             np.array([0, e - a], np.int64), np.array([b], np.uint8), B, wl.F16, wl.F16)
    assert out[a:e].cpu().numpy().tobytes() == want.tobytes()


def test_non_finite_inputs_do_not_disturb_other_buckets(torch, oracle):
    """NaN and infinities violate the precondition: their own buckets are unspecified, but
    nothing is written out of bounds and every other bucket still matches the oracle."""
    rng = np.random.default_rng(11)
    B, n = 128, 128 * 64 + 77
    x = rng.standard_normal(n).astype(np.float32)
    bad = {3: np.nan, 10: np.inf, 20: -np.inf, 33: np.nan, 64: np.inf}
    for k, v in bad.items():
        x[k * B + 5] = v
    x[33 * B + 6] = np.inf
    for b in (2, 4, 8):
        off, bits = np.array([0, n], np.int64), np.array([b], np.uint8)
        gp, gm = gpu_quantize(torch, x, off, bits, B, 9, wl.F32)         # checks the canaries
        op, om = oracle.quantize(x, off, bits, B, 9, wl.F32)
        good = np.array([k not in bad for k in range(om.shape[0])])
        assert gm[good].tobytes() == om[good].tobytes()
        per = B * b // 8
        nb_full = n // B
        gpb, opb = gp[:nb_full * per].reshape(nb_full, per), op[:nb_full * per].reshape(nb_full, per)
        assert np.array_equal(gpb[good[:nb_full]], opb[good[:nb_full]])
        assert np.array_equal(gp[nb_full * per:], op[nb_full * per:])


def test_result_does_not_depend_on_launch_geometry(torch, oracle):
    """Counter-based draws: tiles of several chunks, a small persistent grid, either chunk size and either
    store policy give the same bytes (quantize, reduce, the fused reduce + requantize, decompression)."""
    import hashlib
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = (
        "import sys, hashlib, numpy as np, torch; sys.path.insert(0, %r)\n"
        "from paper_2111_08617_amd import binding as cgx, workloads as wl\n"
        "w = wl.Workload('g', [(2048 * 37 + 300,), (500,), (2048 * 64,)], np.array([4, 0, 2], np.uint8), 256, wl.F32, 2, 5,\n"
        "                wl._normal, np.array([1.0, 1.0, 0.1]))\n"
        "plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt); pb, mb = cgx.cgx_sizes(plan)\n"
        "p = torch.zeros(pb, dtype=torch.uint8, device='cuda'); m = torch.zeros(mb // 4, device='cuda')\n"
        "cgx.cgx_quantize(torch.from_numpy(w.gradient()).cuda(), plan, 77, p, m); torch.cuda.synchronize()\n"
        "s = torch.zeros(w.n, device='cuda'); cgx.cgx_dequant_reduce([p, p], [m, m], plan, s); torch.cuda.synchronize()\n"
        "fp = torch.zeros(pb, dtype=torch.uint8, device='cuda'); fm = torch.zeros(mb // 4, device='cuda')\n"
        "cgx.cgx_dequant_reduce_requantize([p, p], [m, m], plan, 78, fp, fm); torch.cuda.synchronize()\n"
        "d32 = torch.zeros(w.n, device='cuda'); cgx.cgx_dequantize(p, m, plan, wl.F32, d32)\n"
        "d16 = torch.zeros(w.n, dtype=torch.float16, device='cuda'); cgx.cgx_dequantize(p, m, plan, wl.F16, d16)\n"
        "torch.cuda.synchronize()\n"
        "print(hashlib.sha256(b''.join(t.cpu().numpy().tobytes() for t in (p, m, s, fp, fm, d32, d16))).hexdigest())\n"
    ) % root
    digests = set()
    for env in ({}, {"CGX_CHUNKS_PER_TILE": "3"}, {"CGX_CHUNKS_PER_TILE": "8", "CGX_MAX_BLOCKS": "5"},
                {"CGX_QUANTIZE_GROUPS": "4", "CGX_KEEP_SUMS_MB": "0"}, {"CGX_QUANTIZE_GROUPS": "2", "CGX_VIA_LDS": "0"},
                {"CGX_REDUCE_GROUPS": "2"}, {"CGX_REDUCE_GROUPS": "4", "CGX_DEQUANTIZE_THROUGH": "0"},
                {"CGX_QUANTIZE_TILES_PER_WAVE_X4": "4"}, {"CGX_QUANTIZE_TILES_PER_WAVE_X4": "11"}):
        out = subprocess.run([sys.executable, "-c", code], env={**os.environ, **env}, capture_output=True, text=True,
                             timeout=300)
        assert out.returncode == 0, out.stderr[-2000:]
        digests.add(out.stdout.strip().splitlines()[-1])
    assert len(digests) == 1


def test_plan_cache_keeps_working_beyond_its_capacity(torch, oracle):
    """More distinct plans than the library caches (64): the least recently used tables are
    dropped and rebuilt on demand, results stay exact."""
    rng = np.random.default_rng(21)
    x = rng.standard_normal(8192 + 300).astype(np.float32)
    plans = []
    for k in range(70):
        cut = 2048 + 8 * k
        plans.append((np.array([0, cut, x.size], np.int64), np.array([4, 2 + k % 7], np.uint8)))
    for rnd in range(2):                                  # the second round finds the early plans evicted
        for k, (off, bits) in enumerate(plans):
            gp, gm = gpu_quantize(torch, x, off, bits, 128, 3 + k, wl.F32)
            if k % 9 == 0 or rnd == 1 and k < 8:
                op, om = oracle.quantize(x, off, bits, 128, 3 + k, wl.F32)
                assert_same_chunk(gp, gm, op, om, f"plan {k} round {rnd}")


@pytest.mark.parametrize("dt", [wl.F32, wl.F16], ids=["f32", "f16"])
@pytest.mark.parametrize("bucket", [4096, 8192])
def test_buckets_longer_than_a_chunk(torch, oracle, bucket, dt):
    """Whole buckets of 4096 / 8192 elements take the two-pass vectorised tiles; tails and
    unaligned layers the generic ones; every bit width."""
    sizes = [bucket * 3, bucket + 40, 8, bucket * 2, bucket * 2 + 1000, 4, bucket, 16384, bucket * 4 + 24, 100, bucket * 2]
    bits = [1, 2, 0, 3, 4, 5, 0, 6, 7, 8, 4]
    w = wl.Workload("wide", [(s,) for s in sizes], np.array(bits, np.uint8), bucket, dt, 3, 500 + bucket,
                    wl._normal, np.linspace(0.01, 2.0, len(sizes)))
    plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
    kinds = (cgx.cgx_plan_tiles(plan)["info"] >> 4) & 15
    assert (kinds == 4).sum() >= 10 and (kinds == 0).any() and not (kinds == 1).any()
    full_cycle(torch, oracle, w, W=3, what=f"wide B={bucket}")


@pytest.mark.parametrize("dt", [wl.F32, wl.F16], ids=["f32", "f16"])
@pytest.mark.parametrize("bucket", [64, 128, 1024, 4096])
def test_layers_that_start_anywhere(torch, oracle, bucket, dt):
    """Odd-length tensors shift every later layer off the 8-element grid, onto odd element indices
    and back: the vectorised tiles (quantized and pass-through) must take them as they come."""
    sizes = [2048 * 3 + 1, 2048 * 2, 7, 8192 + 3, 2048 * 4 + 2, 1, 8192 * 2, 4096 + 5, 2048 * 5, 3, 8192 + 4096]
    bits = [4, 1, 0, 3, 8, 0, 0, 5, 2, 0, 7]
    w = wl.Workload("shifted", [(s,) for s in sizes], np.array(bits, np.uint8), bucket, dt, 3, 700 + bucket,
                    wl._normal, np.linspace(0.01, 2.0, len(sizes)))
    plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
    tiles = cgx.cgx_plan_tiles(plan)
    vec = np.isin((tiles["info"] >> 4) & 15, (1, 4))
    assert (tiles["elem0"][vec] % 2 == 1).sum() >= 5 and (tiles["elem0"][vec] % 8 == 0).sum() >= 1
    assert np.isin(tiles["elem0"][vec] % 8, (2, 4, 6)).any()
    full_cycle(torch, oracle, w, W=3, what=f"shifted B={bucket}")


def test_step_can_be_captured_in_a_graph_and_replayed(torch, oracle):
    """Once a plan's tables exist the entry points only queue kernels, so a step can be captured;
    every replay (with eager work and synchronisations in between) gives the eager result."""
    w = wl.tiny_mixed(seed=12, bucket=128)
    W = 3
    plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
    plan32 = cgx.Plan(w.offsets, w.bits, w.bucket, wl.F32)
    pb, mb = cgx.cgx_sizes(plan)
    g = dev(torch, w.gradient(0))
    chunks = [oracle.quantize(w.gradient(p), w.offsets, w.bits, w.bucket, w.quant_seed(p), w.dt) for p in range(W)]
    dp = [dev(torch, c[0]) for c in chunks]
    dm = [dev(torch, c[1].reshape(-1)) for c in chunks]

    def buffers():
        return (torch.zeros(pb, dtype=torch.uint8, device="cuda"), torch.zeros(max(mb // 4, 4), device="cuda"),
                torch.zeros(w.n, device="cuda"), torch.zeros(pb, dtype=torch.uint8, device="cuda"),
                torch.zeros(max(mb // 4, 4), device="cuda"))

    def step(out):
        cgx.cgx_quantize(g, plan, 5, out[0], out[1])
        cgx.cgx_dequant_reduce(dp, dm, plan, out[2])
        cgx.cgx_requantize(out[2], plan32, 6, out[3], out[4])

    eager = buffers()
    step(eager)                                   # also builds the plans' tables
    torch.cuda.synchronize()
    want = [t.cpu().numpy().copy() for t in eager]
    op, om = oracle.quantize(w.gradient(0), w.offsets, w.bits, w.bucket, 5, w.dt)
    assert np.array_equal(want[0], op) and want[1][:mb // 4].tobytes() == om.tobytes()

    captured = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(captured)
    torch.cuda.synchronize()
    for replay in range(3):
        for t in captured:
            t.fill_(7 if t.dtype == torch.uint8 else 7.0)      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(captured, want):
            assert got.cpu().numpy().tobytes() == ref.tobytes(), f"replay {replay}"


def test_captured_graph_survives_any_number_of_later_plans(torch, oracle):
    """A table read by a captured graph is pinned: 70 further plans (more than the cache holds) do not free
    it, and the graph still replays to the eager result.  A call whose plan has no table yet is refused
    during a capture (CGX_ERR_CAPTURE) and records nothing; the capture goes on."""
    rng = np.random.default_rng(33)
    x = rng.standard_normal(2048 * 5 + 77).astype(np.float32)
    off, bits = np.array([0, 4096, x.size], np.int64), np.array([4, 3], np.uint8)
    plan = cgx.Plan(off, bits, 256)
    never_seen = cgx.Plan(np.array([0, 4104, x.size], np.int64), bits, 256)
    pb, mb = cgx.cgx_sizes(plan)
    g = dev(torch, x)
    out = (torch.zeros(pb, dtype=torch.uint8, device="cuda"), torch.zeros(mb // 4, device="cuda"))
    spare = (torch.zeros(pb + 64, dtype=torch.uint8, device="cuda"), torch.zeros(mb // 4 + 16, device="cuda"))
    cgx.cgx_quantize(g, plan, 5, out[0], out[1])              # builds the table
    torch.cuda.synchronize()
    op, om = oracle.quantize(x, off, bits, 256, 5, wl.F32)
    assert_same_chunk(out[0].cpu().numpy(), out[1].cpu().numpy(), op, om, "eager")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        with pytest.raises(cgx.CgxError) as refused:
            cgx.cgx_quantize(g, never_seen, 5, spare[0], spare[1])
        cgx.cgx_quantize(g, plan, 5, out[0], out[1])
    assert refused.value.status == -11 and "capture" in str(refused.value)
    torch.cuda.synchronize()
    for k in range(70):                                       # evicts every table that is not pinned
        cut = 2048 + 8 * k
        gpu_quantize(torch, x, np.array([0, cut, x.size], np.int64), np.array([2, 4], np.uint8), 128, k, wl.F32)
    for replay in range(2):
        out[0].fill_(9)
        out[1].fill_(9.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert_same_chunk(out[0].cpu().numpy(), out[1].cpu().numpy(), op, om, f"replay {replay}")
    assert (spare[0] == 0).all() and (spare[1] == 0).all()    # the refused call wrote nothing, then or on replay
    cgx.cgx_quantize(g, never_seen, 5, spare[0], spare[1])    # and works outside a capture
    torch.cuda.synchronize()
    sp, sm = oracle.quantize(x, never_seen.offsets, bits, 256, 5, wl.F32)
    assert np.array_equal(spare[0].cpu().numpy()[:sp.size], sp)


def test_calls_from_several_host_threads_and_streams(torch, oracle):
    """The plan cache is shared by host threads; concurrent calls on separate streams with
    separate outputs give the same bytes as a single call."""
    import threading
    w = wl.tiny_mixed(seed=14, bucket=512)
    plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
    pb, mb = cgx.cgx_sizes(plan)
    g = dev(torch, w.gradient(0))
    op, om = oracle.quantize(w.gradient(0), w.offsets, w.bits, w.bucket, 9, w.dt)
    torch.cuda.synchronize()
    results, errors = {}, []

    def worker(k):
        try:
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.default_stream())
            for rep in range(5):
                # a plan of its own (new tables) and the shared one, alternately
                own = cgx.Plan(np.array([0, 4096 + 8 * k, w.n], np.int64), np.array([4, 2], np.uint8), 128, w.dt)
                opb, omb = cgx.cgx_sizes(own)
                a = torch.empty(opb, dtype=torch.uint8, device="cuda")
                b = torch.empty(max(omb // 4, 4), device="cuda")
                packed = torch.empty(pb, dtype=torch.uint8, device="cuda")
                meta = torch.empty(max(mb // 4, 4), device="cuda")
                cgx.cgx_quantize(g, own, k, a, b, stream=s)
                cgx.cgx_quantize(g, plan, 9, packed, meta, stream=s)
                s.synchronize()
                results[(k, rep)] = (packed.cpu().numpy(), meta.cpu().numpy()[:mb // 4])
        except Exception as e:                      # noqa: BLE001 - reported below
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(6)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    assert len(results) == 30
    for p, m in results.values():
        assert np.array_equal(p, op) and m.tobytes() == om.tobytes()


@pytest.mark.parametrize("dt", [wl.F32, wl.F16], ids=["f32", "f16"])
def test_thousands_of_small_layers(torch, oracle, dt):
    """A layer table of 4000 short tensors of random length, width and alignment."""
    rng = np.random.default_rng(31 + dt)
    sizes = rng.integers(0, 3000, 4000)
    sizes[rng.random(4000) < 0.02] = 0
    sizes[::97] = rng.integers(5000, 40000, sizes[::97].size)
    bits = rng.integers(0, 9, 4000).astype(np.uint8)
    w = wl.Workload("small_layers", [(int(s),) for s in sizes], bits, 256, dt, 2, 4242, wl._normal,
                    np.exp(rng.normal(-3, 1, 4000)))
    full_cycle(torch, oracle, w, W=2, what="4000 layers")
