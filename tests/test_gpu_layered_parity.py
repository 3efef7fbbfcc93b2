"""Parity of the cgx_layered_* calls (a bucket size per layer) with the CPU oracle.

Same bar as the single-size calls: packed stream and meta bit-exact, sums bit-exact against the
oracle's ordered binary32 sum and within 1e-6 * sum |deq| of its binary64 sum.  Inputs of the
reduce come from the oracle's quantizer.
"""
import numpy as np
import pytest

from paper_2111_08617_amd import binding as cgx
from paper_2111_08617_amd import workloads as wl

pytestmark = pytest.mark.gpu

BUCKETS = [32, 64, 96, 128, 256, 512, 1024, 2048, 4096, 8192]


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "these tests need the MI355X"
    cgx.lib()
    return t


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_quantize(torch, grad, plan, seed, requant=False):
    pb, mb = cgx.cgx_layered_sizes(cgx.LayeredPlan(plan.offsets, plan.bits, plan.buckets, wl.F32 if requant else plan.dt))
    packed = torch.full((pb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    meta = torch.full((mb // 4 + 16,), -7.0, dtype=torch.float32, device="cuda")
    g = grad if isinstance(grad, torch.Tensor) else dev(torch, grad)
    if requant:
        cgx.cgx_layered_requantize(g, plan, seed, packed, meta)
    else:
        cgx.cgx_layered_quantize(g, plan, seed, packed, meta)
    torch.cuda.synchronize()
    p, m = packed.cpu().numpy(), meta.cpu().numpy()
    assert (p[pb:] == 0xA5).all() and (m[mb // 4:] == -7.0).all(), "wrote past the reported sizes"
    return p[:pb], m[:mb // 4].reshape(-1, 2)


def same_chunk(gp, gm, op, om, what):
    assert gm.tobytes() == om.tobytes(), f"{what}: meta differs"
    assert np.array_equal(gp, op), f"{what}: packed differs in {int((gp != op).sum())} bytes"


def cycle(torch, oracle, w, buckets, what):
    plan = cgx.LayeredPlan(w.offsets, w.bits, buckets, w.dt)
    chunks, metas = [], []
    for peer in range(w.W):
        g = w.gradient(peer)
        op, om = oracle.layered_quantize(g, w.offsets, w.bits, buckets, w.quant_seed(peer), w.dt)
        if peer < 2:
            gp, gm = gpu_quantize(torch, g, plan, w.quant_seed(peer))
            same_chunk(gp, gm, op, om, f"{what} quantize peer {peer}")
        chunks.append(op)
        metas.append(om)
    ref = oracle.layered_dequant_reduce(chunks, metas, w.offsets, w.bits, buckets, w.dt)
    dp = [dev(torch, c) for c in chunks]
    dm = [dev(torch, m.reshape(-1)) if m.size else torch.zeros(4, device="cuda") for m in metas]
    total = torch.full((w.n + 16,), 123.0, dtype=torch.float32, device="cuda")
    cgx.cgx_layered_dequant_reduce(dp, dm, plan, total)
    torch.cuda.synchronize()
    got = total.cpu().numpy()
    assert (got[w.n:] == 123.0).all(), "wrote past the end of the sum"
    got = got[:w.n]
    assert np.array_equal(got.view(np.uint32), ref["sum32"].view(np.uint32)), f"{what}: sums differ"
    assert (np.abs(got.astype(np.float64) - ref["sum64"]) <= 1e-6 * ref["abs64"] + 1e-45).all(), what
    rp, rm = gpu_quantize(torch, total[:w.n], plan, 99, requant=True)
    op, om = oracle.layered_quantize(got, w.offsets, w.bits, buckets, 99, wl.F32)
    same_chunk(rp, rm, op, om, f"{what} requantize")
    if w.W <= cgx.MAX_FUSED_PEERS:
        pb, mb = cgx.cgx_layered_sizes(cgx.LayeredPlan(w.offsets, w.bits, buckets, wl.F32))
        fp = torch.full((pb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        fm = torch.full((mb // 4 + 16,), -7.0, dtype=torch.float32, device="cuda")
        cgx.cgx_layered_dequant_reduce_requantize(dp, dm, plan, 99, fp, fm)
        torch.cuda.synchronize()
        p, m = fp.cpu().numpy(), fm.cpu().numpy()
        assert (p[pb:] == 0xA5).all() and (m[mb // 4:] == -7.0).all(), "wrote past the reported sizes"
        op, om = oracle.layered_quantize(ref["sum32"], w.offsets, w.bits, buckets, 99, wl.F32)
        same_chunk(p[:pb], m[:mb // 4].reshape(-1, 2), op, om, f"{what} fused reduce+requantize")


@pytest.mark.parametrize("seed", range(24))
def test_random_plans_with_a_bucket_size_per_layer(torch, oracle, seed):
    w = wl.random_plan(seed)
    if w.n == 0:
        pytest.skip("empty plan")
    buckets = np.random.default_rng(seed).choice(BUCKETS, w.L).astype(np.int32)
    cycle(torch, oracle, w, buckets, f"random plan {seed} (buckets {buckets.tolist()}, bits {w.bits.tolist()})")


def test_equal_sizes_give_the_single_size_bytes(torch, oracle):
    w = wl.tiny_mixed(seed=5, dt=wl.F32, bucket=256)
    g = w.gradient()
    gp, gm = gpu_quantize(torch, g, cgx.LayeredPlan(w.offsets, w.bits, np.full(w.L, 256, np.int32), w.dt), 21)
    op, om = oracle.quantize(g, w.offsets, w.bits, 256, 21, w.dt)
    same_chunk(gp, gm, op, om, "equal sizes")


def test_resnet50_with_bucket_sizes_by_layer_size(torch, oracle):
    """The ResNet-50 plan at full size: small layers 128, medium 512, large 2048 (three launches)."""
    w = wl.resnet50()
    sizes = np.diff(w.offsets)
    buckets = np.where(sizes < 100_000, 128, np.where(sizes < 1_000_000, 512, 2048)).astype(np.int32)
    cycle(torch, oracle, w, buckets, "resnet50 layered")


def test_adaptive_round_with_widths_and_bucket_sizes(torch, oracle):
    """One round of the layer-wise scheme ending in a layered plan: norms of an accumulated gradient
    on the device -> k-means widths -> bucket sizes from the widths -> the layered cycle."""
    from oracle import adaptive
    w = wl.bert_base()
    L = 40                                                       # embeddings + 2 blocks
    off = (w.offsets[:L + 1] - w.offsets[0]).astype(np.int64)
    n = int(off[-1])
    acc = sum(w.gradient(p, 0, n) for p in range(3))
    bits_in = np.where(w.bits[:L] == 0, 0, 4).astype(np.uint8)
    plan0 = cgx.Plan(off, np.zeros(L, np.uint8), 32, w.dt)
    ws = torch.empty(max(cgx.cgx_layer_stats_workspace(plan0, for_sqnorms=True), 16), dtype=torch.uint8, device="cuda")
    sq = torch.zeros(L, dtype=torch.float64, device="cuda")
    cgx.cgx_layer_sqnorms(dev(torch, acc), plan0, sq, ws)
    torch.cuda.synchronize()
    norms = np.sqrt(sq.cpu().numpy())
    bits = cgx.cgx_assign_bits_kmeans(off, norms, bits_in, [2, 3, 4])
    buckets = cgx.cgx_assign_buckets_from_bits(bits, [2, 3, 4], [128, 512, 2048])
    sizes = np.diff(off)
    assert bits.tolist() == adaptive.kmeans_bits(sizes, norms, bits_in, [2, 3, 4]).tolist()
    assert buckets.tolist() == adaptive.buckets_from_bits(bits, [2, 3, 4], [128, 512, 2048]).tolist()
    assert len(set(buckets[bits != 0].tolist())) > 1, "the round should mix bucket sizes"
    sub = wl.Workload("bert_head", [tuple(s) for s in w.shapes[:L]], bits, 512, w.dt, 3, w.seed, w.draw, w.scales[:L])
    cycle(torch, oracle, sub, buckets, "adaptive round, layered")


def gpu_layered_sqerrors(torch, grad, packed, meta, plan):
    need = cgx.cgx_layered_stats_workspace(plan)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    out = torch.full((plan.L + 2,), -1.0, dtype=torch.float64, device="cuda")
    m = dev(torch, meta.reshape(-1)) if meta.size else torch.zeros(4, device="cuda")
    cgx.cgx_layered_layer_sqerrors(dev(torch, grad), dev(torch, packed), m, plan, out, ws)
    torch.cuda.synchronize()
    res = out.cpu().numpy()
    assert (res[plan.L:] == -1.0).all(), "wrote past the L outputs"
    return res[:plan.L], need


@pytest.mark.parametrize("seed", range(0, 24, 2))
def test_squared_errors_of_layered_chunks(torch, oracle, seed):
    """Per-layer squared compression errors of chunks with a bucket size per layer: within
    1e-12 relative of the oracle (binary64 sums in a fixed order), zeros exactly."""
    w = wl.random_plan(seed)
    if w.n == 0:
        pytest.skip("empty plan")
    buckets = np.random.default_rng(100 + seed).choice(BUCKETS, w.L).astype(np.int32)
    plan = cgx.LayeredPlan(w.offsets, w.bits, buckets, w.dt)
    g = w.gradient()
    p, m = oracle.layered_quantize(g, w.offsets, w.bits, buckets, 4, w.dt)
    ref = oracle.layered_layer_sqerrors(g, p, m, w.offsets, w.bits, buckets, w.dt)
    got, need = gpu_layered_sqerrors(torch, g, p, m, plan)
    assert np.isfinite(got).all()
    assert (np.abs(got - ref) <= 1e-12 * ref).all(), f"layers {np.nonzero(np.abs(got - ref) > 1e-12 * ref)[0][:5]}"
    assert (got[ref == 0] == 0).all()
    if need >= 16:                      # (an empty tensor has a null pointer: another error)
        small = torch.empty(need - 8, dtype=torch.uint8, device="cuda")
        out = torch.zeros(plan.L, dtype=torch.float64, device="cuda")
        mm = dev(torch, m.reshape(-1)) if m.size else torch.zeros(4, device="cuda")
        with pytest.raises(cgx.CgxError) as e:
            cgx.cgx_layered_layer_sqerrors(dev(torch, g), dev(torch, p), mm, plan, out, small)
        assert e.value.status == -2


@pytest.mark.parametrize("dt", [wl.F32, wl.F16], ids=["f32", "f16"])
def test_layered_dequantize_and_local_addend(torch, oracle, dt):
    """cgx_layered_dequantize into binary32 / binary16 and cgx_layered_dequant_reduce_add with a
    binary32 / binary16 local term, on a plan that mixes all three size classes."""
    sizes = [2048 * 3, 100, 2048 + 700, 8, 8192 + 4096, 33, 2048 * 2, 640]
    bits = np.array([4, 0, 3, 0, 8, 2, 1, 5], np.uint8)
    buckets = np.array([128, 32, 64, 512, 4096, 96, 2048, 32], np.int32)
    w = wl.Workload("mix", [(s,) for s in sizes], bits, 128, dt, 4, 321, wl._normal, np.linspace(0.01, 2.0, len(sizes)))
    plan = cgx.LayeredPlan(w.offsets, w.bits, buckets, w.dt)
    chunks, metas = zip(*[oracle.layered_quantize(w.gradient(p), w.offsets, w.bits, buckets, 50 + p, w.dt) for p in range(20)])
    dp = [dev(torch, c) for c in chunks]
    dm = [dev(torch, m.reshape(-1)) for m in metas]
    one = oracle.layered_dequant_reduce([chunks[0]], [metas[0]], w.offsets, w.bits, buckets, w.dt)["sum32"]
    for out_dt, tdt in ((wl.F32, torch.float32), (wl.F16, torch.float16)):
        out = torch.full((w.n + 16,), 9.0, dtype=tdt, device="cuda")
        cgx.cgx_layered_dequantize(dp[0], dm[0], plan, out_dt, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert (got[w.n:] == 9.0).all()
        want = one if out_dt == wl.F32 else oracle.float_to_half(one).view(np.float16)
        assert got[:w.n].tobytes() == want.tobytes(), f"dequantize to {'f16' if out_dt else 'f32'}"
    for W in (3, 20):
        for local in (w.gradient(99).astype(np.float32), w.gradient(99).astype(np.float16)):
            total = torch.full((w.n + 16,), 9.0, dtype=torch.float32, device="cuda")
            cgx.cgx_layered_dequant_reduce_add(dev(torch, local), wl.F16 if local.dtype == np.float16 else wl.F32,
                                               dp[:W], dm[:W], plan, total)
            torch.cuda.synchronize()
            got = total.cpu().numpy()
            assert (got[w.n:] == 9.0).all()
            ref = oracle.layered_dequant_reduce(list(chunks[:W]), list(metas[:W]), w.offsets, w.bits, buckets, w.dt,
                                                local=local)
            assert np.array_equal(got[:w.n].view(np.uint32), ref["sum32"].view(np.uint32)), f"W={W} {local.dtype}"


def qsgd_cycle(torch, oracle, w, buckets, what):
    """The norm-and-sign calls with a bucket size per layer: quantize, reduce, requantize, fused."""
    plan = cgx.LayeredPlan(w.offsets, w.bits, buckets, w.dt)
    out_plan = cgx.LayeredPlan(w.offsets, w.bits, buckets, wl.F32)

    def quantize(grad, p, seed):
        pb, mb = cgx.cgx_qsgd_layered_sizes(p)
        packed = torch.full((pb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        meta = torch.full((mb // 4 + 16,), -7.0, dtype=torch.float32, device="cuda")
        cgx.cgx_qsgd_layered_quantize(grad if isinstance(grad, torch.Tensor) else dev(torch, grad), p, seed, packed, meta)
        torch.cuda.synchronize()
        a, b = packed.cpu().numpy(), meta.cpu().numpy()
        assert (a[pb:] == 0xA5).all() and (b[mb // 4:] == -7.0).all(), "wrote past the reported sizes"
        return a[:pb], b[:mb // 4]

    chunks, metas = [], []
    for peer in range(w.W):
        g = w.gradient(peer)
        op, om = oracle.qsgd_layered_quantize(g, w.offsets, w.bits, buckets, w.quant_seed(peer), w.dt)
        if peer < 2:
            gp, gm = quantize(g, plan, w.quant_seed(peer))
            same_chunk(gp, gm, op, om, f"{what} quantize peer {peer}")
        chunks.append(op)
        metas.append(om)
    ref = oracle.qsgd_layered_dequant_reduce(chunks, metas, w.offsets, w.bits, buckets, w.dt)
    dp = [dev(torch, c) for c in chunks]
    dm = [dev(torch, m) if m.size else torch.zeros(4, device="cuda") for m in metas]
    total = torch.full((w.n + 16,), 123.0, dtype=torch.float32, device="cuda")
    cgx.cgx_qsgd_layered_dequant_reduce(dp, dm, plan, total)
    torch.cuda.synchronize()
    got = total.cpu().numpy()
    assert (got[w.n:] == 123.0).all()
    got = got[:w.n]
    assert np.array_equal(got.view(np.uint32), ref["sum32"].view(np.uint32)), f"{what}: sums differ"
    rp, rm = quantize(total[:w.n], out_plan, 99)
    op, om = oracle.qsgd_layered_quantize(got, w.offsets, w.bits, buckets, 99, wl.F32)
    same_chunk(rp, rm, op, om, f"{what} requantize")
    if w.W <= cgx.MAX_FUSED_PEERS:
        pb, mb = cgx.cgx_qsgd_layered_sizes(out_plan)
        fp = torch.full((pb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        fm = torch.full((mb // 4 + 16,), -7.0, dtype=torch.float32, device="cuda")
        cgx.cgx_qsgd_layered_dequant_reduce_requantize(dp, dm, plan, 99, fp, fm)
        torch.cuda.synchronize()
        a, b = fp.cpu().numpy(), fm.cpu().numpy()
        assert (a[pb:] == 0xA5).all() and (b[mb // 4:] == -7.0).all()
        op, om = oracle.qsgd_layered_quantize(ref["sum32"], w.offsets, w.bits, buckets, 99, wl.F32)
        same_chunk(a[:pb], b[:mb // 4], op, om, f"{what} fused reduce+requantize")


@pytest.mark.parametrize("seed", range(16))
def test_norm_and_sign_random_plans_with_a_bucket_size_per_layer(torch, oracle, seed):
    w = wl.random_plan(seed)
    if w.n == 0:
        pytest.skip("empty plan")
    w.bits = np.where(w.bits == 1, 2, w.bits).astype(np.uint8)
    buckets = np.random.default_rng(50 + seed).choice(BUCKETS, w.L).astype(np.int32)
    qsgd_cycle(torch, oracle, w, buckets, f"norm-sign random plan {seed} (buckets {buckets.tolist()}, bits {w.bits.tolist()})")


ANY_BUCKETS = [96, 160, 224, 672, 992, 1056, 2016, 2080, 128, 1024, 2048]


@pytest.mark.parametrize("seed", range(10))
def test_layered_plans_that_mix_sizes_that_are_no_power_of_two(torch, oracle, seed):
    """One launch whose tiles are of every kind: buckets of 96 ... 2080 elements next to powers of two."""
    w = wl.random_plan(100 + seed)
    if w.n == 0:
        pytest.skip("empty plan")
    buckets = np.random.default_rng(200 + seed).choice(ANY_BUCKETS, w.L).astype(np.int32)
    what = f"mixed sizes, plan {100 + seed} (buckets {buckets.tolist()}, bits {w.bits.tolist()})"
    cycle(torch, oracle, w, buckets, what)
    if seed < 5:
        w.bits = np.where(w.bits == 1, 2, w.bits).astype(np.uint8)
        qsgd_cycle(torch, oracle, w, buckets, "norm-sign " + what)
