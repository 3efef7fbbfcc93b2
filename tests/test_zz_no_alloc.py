"""cgx_layer_sqnorms_noalloc (the entry point for callers that cannot allocate device memory)
against cgx_layer_sqnorms, through the C ABI: same sums bit for bit, on two calls in a row, the
second on a smaller input, so that whatever the first call left in the library's fixed device
array must not leak into the second.  Collected last (file name), so that a failure here hides no
other test; passes alone in a fresh process and after the other GPU tests.
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
    cgx.lib()
    return t


def both(torch, x, offsets, dt):
    """(allocating call, no-allocation call) on the same device buffer, outputs guarded past L."""
    plan = cgx.Plan(offsets, np.zeros(len(offsets) - 1, np.uint8), 32, dt)
    buf = torch.from_numpy(np.ascontiguousarray(x)).cuda() if x.size else torch.zeros(8, device="cuda").view(
        torch.float16 if dt == wl.F16 else torch.float32)
    ws = torch.empty(max(cgx.cgx_layer_stats_workspace(plan, for_sqnorms=True), 16), dtype=torch.uint8, device="cuda")
    ref = torch.full((plan.L + 2,), -1.0, dtype=torch.float64, device="cuda")
    got = torch.full((plan.L + 2,), -2.0, dtype=torch.float64, device="cuda")
    cgx.cgx_layer_sqnorms(buf, plan, ref, ws)
    cgx.cgx_layer_sqnorms_noalloc(buf, plan, got)
    torch.cuda.synchronize()
    ref, got = ref.cpu().numpy(), got.cpu().numpy()
    assert (ref[plan.L:] == -1.0).all() and (got[plan.L:] == -2.0).all(), "wrote past the L outputs"
    return ref[:plan.L], got[:plan.L]


def layers(seed, sizes, dt):
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    rng = np.random.default_rng(seed)
    scale = np.repeat(np.logspace(-3, 2, len(sizes)), sizes)
    x = (rng.standard_normal(int(off[-1])) * scale).astype(np.float16 if dt == wl.F16 else np.float32)
    return x, off


@pytest.mark.parametrize("dt", [wl.F32, wl.F16], ids=["f32", "f16"])
def test_two_calls_in_a_row_second_one_smaller(torch, dt):
    # first: 300 layers (two slices of the layer table), several tiles per layer, ragged and empty layers
    rng = np.random.default_rng(5)
    sizes = [int(s) for s in rng.integers(0, 60000, 300)]
    sizes[7] = 0
    sizes[11] = 8192 * 5
    sizes[200] = 1
    x, off = layers(1, sizes, dt)
    ref, got = both(torch, x, off, dt)
    assert np.array_equal(ref.view(np.uint64), got.view(np.uint64)), "first call differs from cgx_layer_sqnorms"
    assert (ref[np.array(sizes) > 0] > 0).all()
    # second: fewer, shorter layers; nothing of the first call's tables may show
    x2, off2 = layers(2, [100001, 3, 0, 8192, 8193, 40], dt)
    ref2, got2 = both(torch, x2, off2, dt)
    assert np.array_equal(ref2.view(np.uint64), got2.view(np.uint64)), "second call differs from cgx_layer_sqnorms"
    # and again the larger one
    ref3, got3 = both(torch, x, off, dt)
    assert np.array_equal(ref3.view(np.uint64), got3.view(np.uint64)) and np.array_equal(ref3, ref)


def test_back_to_back_on_one_stream_without_synchronizing(torch):
    """Calls queued on one stream are ordered: each sees its own tables."""
    cases = [layers(10 + k, sizes, wl.F32) for k, sizes in enumerate([[50000, 20000, 7], [9000], [0, 0, 5, 123456]])]
    bufs = [torch.from_numpy(x).cuda() for x, _ in cases]
    plans = [cgx.Plan(off, np.zeros(len(off) - 1, np.uint8), 32, wl.F32) for _, off in cases]
    outs = [torch.empty(p.L, dtype=torch.float64, device="cuda") for p in plans]
    for _ in range(3):
        for b, p, o in zip(bufs, plans, outs):
            cgx.cgx_layer_sqnorms_noalloc(b, p, o)
    torch.cuda.synchronize()
    for (x, off), o in zip(cases, outs):
        ref, _ = both(torch, x, off, wl.F32)
        assert np.array_equal(ref, o.cpu().numpy())


def test_model_shaped_layer_table(torch):
    w = wl.WORKLOADS["resnet50"]()
    g = w.gradient(0, threads=16)
    ref, got = both(torch, g, w.offsets, w.dt)
    assert np.array_equal(ref.view(np.uint64), got.view(np.uint64))
    exact = np.array([float(np.sum(g[a:b].astype(np.float64) ** 2)) for a, b in zip(w.offsets[:-1], w.offsets[1:])])
    assert np.allclose(got, exact, rtol=1e-12, atol=0)


def test_empty_plans(torch):
    ref, got = both(torch, np.zeros(0, np.float32), np.zeros(4, np.int64), wl.F32)
    assert got.tolist() == [0.0, 0.0, 0.0] and ref.tolist() == got.tolist()
    out = torch.full((2,), 7.0, dtype=torch.float64, device="cuda")
    nothing = torch.zeros(8, device="cuda")
    cgx.cgx_layer_sqnorms_noalloc(nothing, cgx.Plan(np.zeros(1, np.int64), np.zeros(0, np.uint8), 32), out)   # L = 0
    torch.cuda.synchronize()
    assert out.tolist() == [7.0, 7.0]
