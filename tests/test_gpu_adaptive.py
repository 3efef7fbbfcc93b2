"""Per-layer statistics of the layer-wise adaptive scheme (cgx_layer_sqnorms, cgx_layer_sqerrors,
cgx_qsgd_layer_sqerrors through the C ABI) against the CPU oracle.

Bar: binary64 sums within 1e-12 relative of the oracle's (long double) sums -- the kernels'
own bound is (140 + tiles/64) * 2^-53 < 1e-13 for every layer here -- exact zeros where the
definition gives zero, and bit-for-bit reproducibility.  Chunks whose error is measured come
from the oracle's quantizer.
"""
import numpy as np
import pytest

from paper_2111_08617_amd import binding as cgx
from paper_2111_08617_amd import workloads as wl

pytestmark = pytest.mark.gpu
RTOL = 1e-12


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "these tests need the MI355X"
    cgx.lib()
    return t


def dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_sqnorms(torch, buf, offsets, dt):
    plan = cgx.Plan(offsets, np.zeros(len(offsets) - 1, np.uint8), 32, dt)
    ws = torch.empty(max(cgx.cgx_layer_stats_workspace(plan, for_sqnorms=True), 16), dtype=torch.uint8, device="cuda")
    out = torch.full((plan.L + 2,), -1.0, dtype=torch.float64, device="cuda")
    b = buf if isinstance(buf, torch.Tensor) else dev(torch, buf)
    cgx.cgx_layer_sqnorms(b, plan, out, ws)
    torch.cuda.synchronize()
    res = out.cpu().numpy()
    assert (res[plan.L:] == -1.0).all(), "wrote past the L outputs"
    return res[:plan.L]


def gpu_sqerrors(torch, grad, packed, meta, offsets, bits, bucket, dt, qsgd=False):
    plan = cgx.Plan(offsets, bits, bucket, dt)
    ws = torch.empty(max(cgx.cgx_layer_stats_workspace(plan), 16), dtype=torch.uint8, device="cuda")
    out = torch.full((plan.L + 2,), -1.0, dtype=torch.float64, device="cuda")
    m = dev(torch, meta.reshape(-1)) if meta.size else torch.zeros(4, device="cuda")
    cgx.cgx_layer_sqerrors(dev(torch, grad), dev(torch, packed), m, plan, out, ws, qsgd=qsgd)
    torch.cuda.synchronize()
    res = out.cpu().numpy()
    assert (res[plan.L:] == -1.0).all(), "wrote past the L outputs"
    return res[:plan.L]


def assert_close(got, ref, what):
    assert np.isfinite(got).all(), what
    bad = np.abs(got - ref) > RTOL * ref
    assert not bad.any(), f"{what}: layers {np.nonzero(bad)[0][:5]} off by {np.max(np.abs(got - ref) / (ref + 1e-300))}"
    assert (got[ref == 0] == 0).all(), what


@pytest.mark.parametrize("dt", [wl.F32, wl.F16], ids=["f32", "f16"])
def test_sqnorms_on_edge_case_layers(torch, oracle, dt):
    """Empty, tiny, ragged and unaligned layers; layers longer than one work item."""
    w = wl.tiny_mixed(seed=3, dt=dt)
    g = w.gradient()
    assert_close(gpu_sqnorms(torch, g, w.offsets, dt), oracle.layer_sqnorms(g, w.offsets, dt), "tiny_mixed")
    sizes = [8192 * 3, 5, 8192 + 7, 0, 40000, 3, 8192 * 2, 100001]
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    rng = np.random.default_rng(9)
    x = (rng.standard_normal(off[-1]) * np.repeat(np.logspace(-3, 2, len(sizes)), sizes)).astype(
        np.float16 if dt == wl.F16 else np.float32)
    got = gpu_sqnorms(torch, x, off, dt)
    assert_close(got, oracle.layer_sqnorms(x, off, dt), "ragged layers")
    assert np.array_equal(got, gpu_sqnorms(torch, x, off, dt)), "not reproducible"
    assert gpu_sqnorms(torch, np.zeros(0, x.dtype), np.zeros(4, np.int64), dt).tolist() == [0.0, 0.0, 0.0]


@pytest.mark.parametrize("name", ["resnet50", "gpt2_medium", "decoder_1p3b"])
def test_sqnorms_full_size(torch, oracle, name):
    w = wl.WORKLOADS[name]()
    g = w.gradient(0, threads=16)
    assert_close(gpu_sqnorms(torch, g, w.offsets, w.dt), oracle.layer_sqnorms(g, w.offsets, w.dt), name)


@pytest.mark.parametrize("qsgd", [False, True], ids=["minmax", "normsign"])
@pytest.mark.parametrize("dt", [wl.F32, wl.F16], ids=["f32", "f16"])
@pytest.mark.parametrize("bucket", [32, 96, 128, 1024, 4096])
def test_sqerrors_on_edge_case_plans(torch, oracle, bucket, dt, qsgd):
    w = wl.tiny_mixed(seed=bucket + dt, dt=dt, bucket=bucket)
    if qsgd:
        w.bits = np.where(w.bits == 1, 2, w.bits).astype(np.uint8)
    g = w.gradient()
    p, m = (oracle.qsgd_quantize if qsgd else oracle.quantize)(g, w.offsets, w.bits, bucket, 3, dt)
    ref = oracle.layer_sqerrors(g, p, m, w.offsets, w.bits, bucket, dt, scheme=int(qsgd))
    assert_close(gpu_sqerrors(torch, g, p, m, w.offsets, w.bits, bucket, dt, qsgd), ref, f"tiny_mixed B={bucket}")


@pytest.mark.parametrize("seed", range(0, 24, 2))
def test_statistics_of_random_plans(torch, oracle, seed):
    """Seeded random plans: squared norms, and squared errors of both quantizers."""
    w = wl.random_plan(seed)
    if w.n == 0:
        pytest.skip("empty plan (covered by the edge cases)")
    g = w.gradient()
    assert_close(gpu_sqnorms(torch, g, w.offsets, w.dt), oracle.layer_sqnorms(g, w.offsets, w.dt), f"random plan {seed}")
    for qsgd in (False, True):
        bits = np.where(w.bits == 1, 2, w.bits).astype(np.uint8) if qsgd else w.bits
        p, m = (oracle.qsgd_quantize if qsgd else oracle.quantize)(g, w.offsets, bits, w.bucket, 5, w.dt)
        ref = oracle.layer_sqerrors(g, p, m, w.offsets, bits, w.bucket, w.dt, scheme=int(qsgd))
        assert_close(gpu_sqerrors(torch, g, p, m, w.offsets, bits, w.bucket, w.dt, qsgd), ref,
                     f"random plan {seed} (bucket {w.bucket}, bits {bits.tolist()}, {'norm-sign' if qsgd else 'min/max'})")


@pytest.mark.parametrize("qsgd", [False, True], ids=["minmax", "normsign"])
@pytest.mark.parametrize("dt", [wl.F32, wl.F16], ids=["f32", "f16"])
@pytest.mark.parametrize("bucket", [64, 512, 2048, 4096])
def test_sqerrors_vectorised_path_all_bit_widths(torch, oracle, bucket, dt, qsgd):
    sizes = [2048 * 4, 2048 * 2 + 40, 8, 4096, 2048 * 5 + 1000, 2048 * 4, 16384, 2048 + bucket, 8192, 8192 * 2 + 24]
    bits = [2 if qsgd else 1, 2, 0, 3, 4, 5, 0, 6, 7, 8]
    w = wl.Workload("chunks", [(s,) for s in sizes], np.array(bits, np.uint8), bucket, dt, 1, 3000 + bucket,
                    wl._normal, np.linspace(0.01, 2.0, len(sizes)))
    g = w.gradient()
    p, m = (oracle.qsgd_quantize if qsgd else oracle.quantize)(g, w.offsets, w.bits, bucket, 8, dt)
    ref = oracle.layer_sqerrors(g, p, m, w.offsets, w.bits, bucket, dt, scheme=int(qsgd))
    got = gpu_sqerrors(torch, g, p, m, w.offsets, w.bits, bucket, dt, qsgd)
    assert_close(got, ref, f"chunks B={bucket}")
    assert got[2] == 0 and got[6] == 0 and (got[[0, 1, 3, 4, 5, 7, 8, 9]] > 0).all()


def test_sqerrors_resnet50_full_size_and_workspace_check(torch, oracle):
    w = wl.resnet50()
    g = w.gradient(0)
    p, m = oracle.quantize(g, w.offsets, w.bits, w.bucket, 1, w.dt)
    ref = oracle.layer_sqerrors(g, p, m, w.offsets, w.bits, w.bucket, w.dt)
    assert_close(gpu_sqerrors(torch, g, p, m, w.offsets, w.bits, w.bucket, w.dt), ref, "resnet50")
    plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
    need = cgx.cgx_layer_stats_workspace(plan)
    small = torch.empty(need - 8, dtype=torch.uint8, device="cuda")
    out = torch.zeros(w.L, dtype=torch.float64, device="cuda")
    with pytest.raises(cgx.CgxError) as e:
        cgx.cgx_layer_sqerrors(dev(torch, g), dev(torch, p), dev(torch, m.reshape(-1)), plan, out, small)
    assert e.value.status == -2


def test_adaptive_round_on_the_device(torch, oracle):
    """One round of the scheme: norms of an accumulated gradient -> k-means widths -> quantize with
    them -> error per layer, next to the all-4-bit error E_4 (problem definition of the section)."""
    w = wl.bert_base()
    sub = slice(0, 40)                                           # the first 40 tensors: embeddings + 2 blocks
    off = (w.offsets[:41] - w.offsets[0]).astype(np.int64)
    n = int(off[-1])
    acc = sum(w.gradient(p, 0, n) for p in range(3))             # stand-in for an accumulated gradient
    bits_in = np.where(w.bits[sub] == 0, 0, 4).astype(np.uint8)
    sq = gpu_sqnorms(torch, acc, off, w.dt)
    assert_close(sq, oracle.layer_sqnorms(acc, off, w.dt), "accumulated gradient")
    bits = cgx.cgx_assign_bits_kmeans(off, np.sqrt(sq), bits_in, [2, 3, 4])
    g = w.gradient(0, 0, n)
    plan = cgx.Plan(off, bits, w.bucket, w.dt)
    pb, mb = cgx.cgx_sizes(plan)
    packed = torch.empty(pb, dtype=torch.uint8, device="cuda")
    meta = torch.empty(max(mb // 4, 4), dtype=torch.float32, device="cuda")
    dg = dev(torch, g)
    cgx.cgx_quantize(dg, plan, 5, packed, meta)
    ws = torch.empty(max(cgx.cgx_layer_stats_workspace(plan), 16), dtype=torch.uint8, device="cuda")
    err = torch.zeros(plan.L, dtype=torch.float64, device="cuda")
    cgx.cgx_layer_sqerrors(dg, packed, meta, plan, err, ws)
    torch.cuda.synchronize()
    op, om = oracle.quantize(g, off, bits, w.bucket, 5, w.dt)
    assert np.array_equal(packed.cpu().numpy(), op)
    assert_close(err.cpu().numpy(), oracle.layer_sqerrors(g, op, om, off, bits, w.bucket, w.dt), "assigned widths")
    p4, m4 = oracle.quantize(g, off, bits_in, w.bucket, 5, w.dt)
    e4 = oracle.layer_sqerrors(g, p4, m4, off, bits_in, w.bucket, w.dt)
    size = np.diff(off)
    assert (bits * size).sum() < (bits_in * size).sum()          # fewer bits on the wire ...
    assert err.cpu().numpy().sum() > e4.sum()                    # ... paid with a larger error than E_4


@pytest.mark.parametrize("dt", [wl.F32, wl.F16], ids=["f32", "f16"])
def test_statistics_of_layers_that_start_anywhere(torch, oracle, dt):
    sizes = [2048 * 3 + 1, 2048 * 2, 7, 8192 + 3, 2048 * 4 + 2, 1, 8192 * 2, 4096 + 5, 2048 * 5]
    bits = [4, 1, 0, 3, 8, 0, 0, 5, 2]
    w = wl.Workload("shifted", [(s,) for s in sizes], np.array(bits, np.uint8), 256, dt, 1, 900, wl._normal,
                    np.linspace(0.01, 2.0, len(sizes)))
    g = w.gradient()
    assert_close(gpu_sqnorms(torch, g, w.offsets, dt), oracle.layer_sqnorms(g, w.offsets, dt), "shifted sqnorms")
    p, m = oracle.quantize(g, w.offsets, w.bits, w.bucket, 2, dt)
    assert_close(gpu_sqerrors(torch, g, p, m, w.offsets, w.bits, w.bucket, dt),
                 oracle.layer_sqerrors(g, p, m, w.offsets, w.bits, w.bucket, dt), "shifted sqerrors")


def test_measurement_aids_run_and_stay_in_bounds(torch):
    """The streaming probe (every load and store policy, both block numberings, a persistent grid, odd sizes)
    and the issue-rate probe (every instruction form) run, and write nothing past the bytes they were given."""
    src = torch.arange(0, 3 * 8192 + 48, dtype=torch.int32, device="cuda").view(torch.uint8)
    rb = src.numel() // 16 * 16
    for wb in (0, 1600, rb // 2 // 16 * 16, rb):
        for loads in cgx.LOAD_POLICIES:
            for stores in cgx.STORE_POLICIES:
                dst = torch.full((wb + 64,), 0xA5, dtype=torch.uint8, device="cuda")
                for slice_bytes, block, xcd, max_blocks in ((8192, 256, False, 0), (2048, 1024, True, 0), (4096, 64, True, 3)):
                    cgx.cgx_stream_probe_shaped(src, rb, dst, wb, slice_bytes, block, loads, stores, xcd, max_blocks)
                torch.cuda.synchronize()
                assert (dst[wb:] == 0xA5).all(), (wb, loads, stores)
    cgx.cgx_stream_probe(src, rb, torch.empty(rb, dtype=torch.uint8, device="cuda"), rb)
    forms = cgx.cgx_issue_probe_forms()
    out = torch.full((8 * 256 + 16,), -1, dtype=torch.int32, device="cuda")
    for form in range(len(forms)):
        cgx.cgx_issue_probe(form, 8, 3, out)
    torch.cuda.synchronize()
    assert (out[8 * 256:] == -1).all()
