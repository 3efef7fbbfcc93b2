"""Host-side tests of libcgx.so: no kernel is launched, no GPU is needed.

They cover the exported symbols, the argument checks of every entry point, the
sizes of the packed stream / meta array (against the oracle's layout rules) and
the tile table the kernels walk (paper Sec. 4.1: per-layer compression from the
layer offsets of the fused buffer; Sec. 4.3: whole buckets).
"""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2111_08617_amd import binding as cgx
from paper_2111_08617_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CHUNK = 2048            # elements a wavefront takes per pass of the vectorised path


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(cgx.LIB_PATH):
        from paper_2111_08617_amd import build
        build.build()
    return cgx.lib()


def test_library_exports_every_declared_symbol(lib):
    header = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("cgx.h", "cgx_diag.h"))
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(cgx_[a-z_0-9]+)\s*\(", header))
    assert declared == set(cgx.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings(lib):
    seen = {cgx.status_string(s) for s in range(0, -11, -1)}
    assert len(seen) == 11 and "unknown status" not in seen
    assert cgx.status_string(-99) == "unknown status"


@pytest.mark.parametrize("name", ["single_1m", "resnet50", "bert_base", "gpt2_medium", "decoder_1p3b"])
def test_sizes_match_the_oracle_layout(lib, oracle, name):
    w = wl.WORKLOADS[name]()
    plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
    assert cgx.cgx_sizes(plan) == oracle.sizes(w.offsets, w.bits, w.bucket, w.dt)


def test_sizes_of_edge_plans(lib, oracle):
    for dt in (wl.F32, wl.F16):
        for bucket in (32, 64, 96, 1024, 8192):
            w = wl.tiny_mixed(dt=dt, bucket=bucket)
            plan = cgx.Plan(w.offsets, w.bits, bucket, dt)
            assert cgx.cgx_sizes(plan) == oracle.sizes(w.offsets, w.bits, bucket, dt)
    empty = cgx.Plan(np.zeros(1, np.int64), np.zeros(0, np.uint8), 128)
    assert cgx.cgx_sizes(empty) == (0, 0)
    only_empty_layers = cgx.Plan(np.zeros(4, np.int64), np.array([4, 0, 8], np.uint8), 128)
    assert cgx.cgx_sizes(only_empty_layers) == (0, 0)


def _status(fn, *args):
    return fn(*args)


def test_argument_errors_are_found_on_the_host(lib):
    c = ctypes
    off = np.array([0, 100, 300], np.int64)
    bits = np.array([4, 0], np.uint8)
    pb, mb = c.c_size_t(), c.c_size_t()

    def sizes(n, L, o, b, bucket, dt=0):
        return lib.cgx_sizes(n, L, o.ctypes.data if o is not None else None,
                             b.ctypes.data if b is not None else None, bucket, dt, c.byref(pb), c.byref(mb))

    assert sizes(300, 2, off, bits, 128) == 0
    assert sizes(-1, 2, off, bits, 128) == -2
    assert sizes(300, -1, off, bits, 128) == -2
    assert sizes(301, 2, off, bits, 128) == -2                       # n != offsets[L]
    assert sizes(300, 2, None, bits, 128) == -1
    assert sizes(300, 2, off, None, 128) == -1
    assert sizes(300, 2, np.array([1, 100, 300], np.int64), bits, 128) == -3
    assert sizes(300, 2, np.array([0, 400, 300], np.int64), bits, 128) == -3
    assert sizes(300, 2, off, np.array([9, 0], np.uint8), 128) == -4
    for bad in (0, 16, 33, 100, 8192 + 32, -128):
        assert sizes(300, 2, off, bits, bad) == -5
    assert sizes(300, 2, off, bits, 128, 2) == -7
    assert sizes(5, 0, off, bits, 128) == -2                         # no layers but n > 0

    # the compute entry points reject bad arguments before touching the device
    o, b = off.ctypes.data, bits.ctypes.data
    buf = 0x1000                                                      # never dereferenced
    assert lib.cgx_quantize(buf, 300, 2, o, b, 100, 0, 0, buf, buf, None) == -5
    assert lib.cgx_quantize(None, 300, 2, o, b, 128, 0, 0, buf, buf, None) == -1
    assert lib.cgx_quantize(buf, 300, 2, o, b, 128, 0, 0, None, buf, None) == -1
    assert lib.cgx_quantize(buf, 300, 2, o, b, 128, 0, 0, buf, None, None) == -1
    assert lib.cgx_quantize(buf + 4, 300, 2, o, b, 128, 0, 0, buf, buf, None) == -9
    assert lib.cgx_quantize(buf, 300, 2, o, b, 128, 0, 0, buf + 8, buf, None) == -9
    assert lib.cgx_quantize(buf, 300, 2, o, b, 128, 0, 3, buf, buf, None) == -7
    assert lib.cgx_requantize(None, 300, 2, o, b, 128, 0, buf, buf, None) == -1
    assert lib.cgx_requantize(buf, 299, 2, o, b, 128, 0, buf, buf, None) == -2
    ptrs = (c.c_void_p * 2)(buf, buf)
    nulls = (c.c_void_p * 2)(buf, None)
    assert lib.cgx_dequant_reduce(ptrs, ptrs, 0, 300, 2, o, b, 128, 0, buf, None) == -6
    assert lib.cgx_dequant_reduce(ptrs, ptrs, 65, 300, 2, o, b, 128, 0, buf, None) == -6
    assert lib.cgx_dequant_reduce(None, ptrs, 2, 300, 2, o, b, 128, 0, buf, None) == -1
    assert lib.cgx_dequant_reduce(nulls, ptrs, 2, 300, 2, o, b, 128, 0, buf, None) == -1
    assert lib.cgx_dequant_reduce(ptrs, nulls, 2, 300, 2, o, b, 128, 0, buf, None) == -1
    assert lib.cgx_dequant_reduce(ptrs, ptrs, 2, 300, 2, o, b, 128, 0, None, None) == -1
    assert lib.cgx_dequant_reduce(ptrs, ptrs, 2, 300, 2, o, b, 128, 0, buf + 4, None) == -9
    assert lib.cgx_dequant_reduce(ptrs, ptrs, 2, 300, 2, o, b, 48, 0, buf, None) == -5
    assert lib.cgx_dequant_reduce_add(None, 0, ptrs, ptrs, 2, 300, 2, o, b, 128, 0, buf, None) == -1
    assert lib.cgx_dequant_reduce_add(buf, 2, ptrs, ptrs, 2, 300, 2, o, b, 128, 0, buf, None) == -7
    assert lib.cgx_dequant_reduce_add(buf + 2, 1, ptrs, ptrs, 2, 300, 2, o, b, 128, 0, buf, None) == -9
    assert lib.cgx_dequantize(None, buf, 300, 2, o, b, 128, 0, 0, buf, None) == -1
    assert lib.cgx_dequantize(buf, buf, 300, 2, o, b, 128, 0, 4, buf, None) == -7
    assert lib.cgx_dequantize(buf, buf, 300, 2, o, b, 128, 0, 1, None, None) == -1
    assert lib.cgx_stream_probe(None, 1024, buf, 1024, None) == -1
    assert lib.cgx_stream_probe(buf, 1000, buf, 1024, None) == -2
    assert lib.cgx_stream_probe(buf + 4, 1024, buf, 1024, None) == -9
    shaped = lambda *v: lib.cgx_stream_probe_shaped(buf, 1024, buf, 1024, (c.c_int32 * 9)(*(v + (0,) * (9 - len(v)))), None)
    assert lib.cgx_stream_probe_shaped(buf, 1024, buf, 1024, None, None) == -1
    for bad in ((1000, 256, 1, 1, 0, 0), (512, 256, 1, 1, 0, 0), (1 << 21, 256, 1, 1, 0, 0), (8192, 96, 1, 1, 0, 0),
                (8192, 2048, 1, 1, 0, 0), (8192, 256, 4, 1, 0, 0), (8192, 256, 1, 5, 0, 0), (8192, 256, -1, 1, 0, 0),
                (8192, 256, 1, 1, 2, 0), (8192, 256, 1, 1, 0, -1), (8192, 256, 1, 1, 0, 0, 2),
                (8192, 256, 1, 1, 0, 0, 0, -1), (8192, 256, 1, 1, 0, 0, 0, 0, 65537)):
        assert shaped(*bad) == -2
    forms = cgx.cgx_issue_probe_forms()
    assert len(forms) >= 30 and forms[0].startswith("v_add_f32") and len(set(forms)) == len(forms)
    assert lib.cgx_issue_probe_form(-1) is None and lib.cgx_issue_probe_form(len(forms)) is None
    assert lib.cgx_issue_probe(0, 8, 10, None, 8 * 1024, None) == -1
    for bad in ((-1, 8, 10, 8192), (len(forms), 8, 10, 8192), (0, 0, 10, 8192), (0, 65537, 10, 1 << 27),
                (0, 8, 0, 8192), (0, 8, (1 << 20) + 1, 8192), (0, 8, 10, 8191)):
        assert lib.cgx_issue_probe(bad[0], bad[1], bad[2], buf, bad[3], None) == -2
    assert lib.cgx_issue_probe(0, 8, 10, buf + 4, 8192, None) == -9
    fused = lib.cgx_dequant_reduce_requantize
    assert fused(ptrs, ptrs, 0, 300, 2, o, b, 128, 0, 1, buf, buf, None) == -6
    assert fused(ptrs, ptrs, 17, 300, 2, o, b, 128, 0, 1, buf, buf, None) == -6
    assert fused(ptrs, nulls, 2, 300, 2, o, b, 128, 0, 1, buf, buf, None) == -1
    assert fused(ptrs, ptrs, 2, 300, 2, o, b, 128, 0, 1, None, buf, None) == -1
    assert fused(ptrs, ptrs, 2, 300, 2, o, b, 128, 0, 1, buf, None, None) == -1
    assert fused(ptrs, ptrs, 2, 300, 2, o, b, 128, 0, 1, buf + 8, buf, None) == -9
    assert fused(ptrs, ptrs, 2, 300, 2, o, b, 128, 5, 1, buf, buf, None) == -7
    assert fused(ptrs, ptrs, 2, 300, 2, o, b, 160 + 8, 0, 1, buf, buf, None) == -5
    # empty buffers are accepted and do nothing
    z = np.zeros(1, np.int64)
    assert lib.cgx_quantize(None, 0, 0, z.ctypes.data, None, 128, 0, 0, None, None, None) == 0
    assert lib.cgx_dequant_reduce(ptrs, ptrs, 2, 0, 0, z.ctypes.data, None, 128, 0, None, None) == 0


def test_no_allocation_entry_point_checks_its_arguments_and_limits(lib):
    """cgx_layer_sqnorms_noalloc: the errors of cgx_layer_sqnorms, and CGX_ERR_CAPACITY beyond its fixed tables;
    all found on the host before anything is queued."""
    fn = lib.cgx_layer_sqnorms_noalloc
    buf = 0x1000                                                      # never dereferenced
    off = np.array([0, 100, 300], np.int64)
    o = off.ctypes.data
    assert fn(buf, -1, 2, o, 0, buf, None) == -2
    assert fn(buf, 301, 2, o, 0, buf, None) == -2
    assert fn(buf, 300, 2, None, 0, buf, None) == -1
    assert fn(buf, 300, 2, o, 2, buf, None) == -7
    assert fn(buf, 300, 2, np.array([1, 100, 300], np.int64).ctypes.data, 0, buf, None) == -3
    assert fn(buf, 300, 2, np.array([0, 400, 300], np.int64).ctypes.data, 0, buf, None) == -3
    assert fn(None, 300, 2, o, 0, buf, None) == -1
    assert fn(buf, 300, 2, o, 0, None, None) == -1
    assert fn(buf + 4, 300, 2, o, 0, buf, None) == -9
    assert fn(buf, 300, 2, o, 0, buf + 4, None) == -9
    assert fn(None, 0, 0, o, 0, None, None) == 0                      # no layers: nothing to do
    # one layer too many
    many = np.arange(cgx.NOALLOC_MAX_LAYERS + 2, dtype=np.int64)
    assert fn(buf, int(many[-1]), many.size - 1, many.ctypes.data, 0, buf, None) == -10
    # one work item too many: a work item is a run of 8192 elements of one layer
    big = np.array([0, 8192 * cgx.NOALLOC_MAX_TILES, 8192 * cgx.NOALLOC_MAX_TILES + 1], np.int64)
    assert fn(buf, int(big[-1]), 2, big.ctypes.data, 0, buf, None) == -10
    assert "no-allocation" in cgx.status_string(-10)
    header = open(os.path.join(ROOT, "include", "cgx.h")).read()
    assert "#define CGX_NOALLOC_MAX_LAYERS %d\n" % cgx.NOALLOC_MAX_LAYERS in header
    assert "#define CGX_NOALLOC_MAX_TILES %d\n" % cgx.NOALLOC_MAX_TILES in header


def test_norm_and_sign_entry_points_check_their_arguments(lib, oracle):
    c = ctypes
    off = np.array([0, 100, 300, 1300], np.int64)
    o = off.ctypes.data
    pb, mb = c.c_size_t(), c.c_size_t()
    ok = np.array([4, 0, 2], np.uint8)
    one = np.array([4, 0, 1], np.uint8)
    assert lib.cgx_qsgd_sizes(1300, 3, o, ok.ctypes.data, 128, 0, c.byref(pb), c.byref(mb)) == 0
    assert (pb.value, mb.value) == oracle.qsgd_sizes(off, ok, 128)
    assert mb.value == 4 * (1 + 8)                                    # one float per bucket
    assert lib.cgx_qsgd_sizes(1300, 3, o, one.ctypes.data, 128, 0, c.byref(pb), c.byref(mb)) == -4
    assert lib.cgx_qsgd_sizes(1300, 3, o, ok.ctypes.data, 100, 0, c.byref(pb), c.byref(mb)) == -5
    buf = 0x1000                                                      # never dereferenced
    ptrs = (c.c_void_p * 2)(buf, buf)
    assert lib.cgx_qsgd_quantize(buf, 1300, 3, o, one.ctypes.data, 128, 0, 0, buf, buf, None) == -4
    assert lib.cgx_qsgd_quantize(None, 1300, 3, o, ok.ctypes.data, 128, 0, 0, buf, buf, None) == -1
    assert lib.cgx_qsgd_quantize(buf, 1300, 3, o, ok.ctypes.data, 128, 0, 0, buf + 4, buf, None) == -9
    assert lib.cgx_qsgd_dequant_reduce(ptrs, ptrs, 2, 1300, 3, o, one.ctypes.data, 128, 0, buf, None) == -4
    assert lib.cgx_qsgd_dequant_reduce(ptrs, ptrs, 65, 1300, 3, o, ok.ctypes.data, 128, 0, buf, None) == -6
    assert lib.cgx_qsgd_dequant_reduce(ptrs, ptrs, 2, 1300, 3, o, ok.ctypes.data, 128, 0, None, None) == -1
    fused = lib.cgx_qsgd_dequant_reduce_requantize
    assert fused(ptrs, ptrs, 2, 1300, 3, o, one.ctypes.data, 128, 0, 1, buf, buf, None) == -4
    assert fused(ptrs, ptrs, 17, 1300, 3, o, ok.ctypes.data, 128, 0, 1, buf, buf, None) == -6
    assert fused(ptrs, ptrs, 2, 1300, 3, o, ok.ctypes.data, 128, 0, 1, buf, None, None) == -1
    for name in ("resnet50", "gpt2_medium"):
        w = wl.WORKLOADS[name]()
        plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
        assert cgx.cgx_qsgd_sizes(plan) == oracle.qsgd_sizes(w.offsets, w.bits, w.bucket, w.dt)


def layer_segments(w):
    """(segment start, payload bytes, first bucket) per layer from the layout rules."""
    seg, g, out = 0, 0, []
    es = 2 if w.dt else 4
    for l in range(w.L):
        ln = int(w.offsets[l + 1] - w.offsets[l])
        b = int(w.bits[l])
        payload = ln * es if b == 0 else -(-ln * b // 8)
        out.append((seg, payload, g))
        if ln:
            seg += (payload + 15) // 16 * 16
            g += 0 if b == 0 else -(-ln // w.bucket)
    return out


@pytest.mark.parametrize("make", [
    lambda: wl.tiny_mixed(), lambda: wl.tiny_mixed(dt=wl.F16, bucket=128), lambda: wl.tiny_mixed(bucket=96),
    lambda: wl.tiny_mixed(bucket=4096), wl.resnet50, wl.bert_base, wl.gpt2_medium,
    lambda: wl.Workload("wide", [(4096 * 3 + 100,), (4,), (8192 * 2,), (4096,), (5000,)], np.array([4, 0, 3, 8, 2], np.uint8),
                        4096, wl.F32, 2, 1, wl._normal, np.ones(5)),
    lambda: wl.Workload("wide16", [(8192 * 2 + 8,), (8192,), (100,)], np.array([4, 5, 1], np.uint8),
                        8192, wl.F16, 2, 1, wl._normal, np.ones(3)),
])
@pytest.mark.parametrize("CHUNK", [2048, 1024])
def test_tiles_cover_every_layer_exactly_once(lib, make, CHUNK):
    """Both tile tables: chunks of 2048 elements (reduce, fused and statistics kernels, binary16 quantizer)
    and of 1024 (binary32 quantizer)."""
    w = make()
    plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
    tiles = cgx.cgx_plan_tiles(plan, CHUNK)
    segs = layer_segments(w)
    es = 2 if w.dt else 4
    # generic and pass-through tiles first, then the vectorised ones; buffer order within each class
    vectorised = np.isin((tiles["info"] >> 4) & 15, (1, 4, 6))
    assert not vectorised[:int((~vectorised).sum())].any()
    for cls in (tiles[~vectorised], tiles[vectorised]):
        assert (np.diff(cls["elem0"]) > 0).all()
    counts = tiles["count"].astype(np.int64)
    assert (counts > 0).all()
    covered = np.zeros(w.n, np.int8)
    for t in tiles:
        covered[t["elem0"]:t["elem0"] + t["count"]] += 1
    assert (covered == 1).all()
    layer_of = np.searchsorted(w.offsets, tiles["elem0"], side="right") - 1     # last layer starting at or before
    for t, l in zip(tiles, layer_of):
        a, e = int(w.offsets[l]), int(w.offsets[l + 1])
        assert a <= t["elem0"] and t["elem0"] + t["count"] <= e       # never crosses a layer
        b = int(w.bits[l])
        kind = (int(t["info"]) >> 4) & 15
        assert int(t["info"]) & 15 == b
        seg, payload, g0 = segs[l]
        j = int(t["elem0"]) - a
        last = t["elem0"] + t["count"] == e
        assert int(t["pad"]) == ((-payload) % 16 if last else 0)
        if b == 0:
            assert kind == 3                                          # every copy tile is vectorised
            assert t["packed_off"] == seg + j * es
        else:
            assert kind in (0, 1, 4, 5, 6)
            assert j % w.bucket == 0                                  # tiles start on a bucket
            assert last or t["count"] % w.bucket == 0                 # and hold whole buckets
            assert t["packed_off"] == seg + j * b // 8
            assert t["bucket0"] == g0 + j // w.bucket
            if kind == 1:
                assert t["count"] % CHUNK == 0
                assert w.bucket & (w.bucket - 1) == 0 and w.bucket <= CHUNK
                assert (int(t["info"]) >> 8) & 15 == int(np.log2(w.bucket * 64 // CHUNK))
            if kind == 5:                                             # the short end of a layer, masked chunk
                assert last and t["count"] < CHUNK and j % CHUNK == 0
                assert w.bucket & (w.bucket - 1) == 0 and w.bucket <= CHUNK
                assert (int(t["info"]) >> 8) & 15 == int(np.log2(w.bucket * 64 // CHUNK))
            if kind == 0:                                             # generic: only where nothing else fits
                assert w.bucket & (w.bucket - 1) != 0 or w.bucket > CHUNK
                if w.bucket & (w.bucket - 1) != 0 and w.bucket <= CHUNK:
                    assert last and t["count"] % w.bucket != 0       # only the ragged end of a layer
            if kind == 6:                                             # whole buckets of a size that is no power of two
                assert w.bucket & (w.bucket - 1) != 0 and w.bucket <= CHUNK
                assert t["count"] % w.bucket == 0 and t["count"] <= CHUNK and t["count"] % 32 == 0
            if kind == 4:                                             # one whole bucket of several chunks
                assert t["count"] == w.bucket and w.bucket in (4096, 8192) + ((2048,) if CHUNK == 1024 else ())
                assert (int(t["info"]) >> 8) & 15 == 6
    if w.name.startswith("wide"):
        assert (((tiles["info"] >> 4) & 15) == 4).sum() == (9 if w.name == "wide" else 3)


def test_large_plans_use_the_vectorised_path(lib):
    for make in (wl.resnet50, wl.decoder_1p3b):
        for chunk in (1024, 2048):
            w = make()
            plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
            tiles = cgx.cgx_plan_tiles(plan, chunk)
            kind = (tiles["info"] >> 4) & 15
            fast = tiles["count"][(kind == 1) | (kind == 3)].astype(np.int64).sum()
            assert fast / w.n > 0.999
    plan = cgx.Plan(np.array([0, 5000], np.int64), np.array([4], np.uint8), 128)
    n_tiles = ctypes.c_int64()
    assert lib.cgx_plan_tiles_chunk(*plan.args, plan.dt, 512, None, 0, ctypes.byref(n_tiles)) == -2
    assert lib.cgx_plan_tiles_chunk(*plan.args, plan.dt, 4096, None, 0, ctypes.byref(n_tiles)) == -2


def test_tiles_do_not_straddle_a_generator_key_block(lib):
    """Vectorised tiles lie inside one 2^33-element block (the generator's key is
    uniform there); a tile that would straddle is handed to the generic path."""
    n = (1 << 33) + 8192
    plan = cgx.Plan(np.array([0, n], np.int64), np.array([2], np.uint8), 1024)
    old = os.environ.get("CGX_CHUNKS_PER_TILE")
    tiles = cgx.cgx_plan_tiles(plan)
    lo, hi = tiles["elem0"] >> 33, (tiles["elem0"] + tiles["count"].astype(np.int64) - 1) >> 33
    kind = (tiles["info"] >> 4) & 15
    assert ((lo == hi) | (kind == 0)).all()
    assert tiles["count"].astype(np.int64).sum() == n
    assert old == os.environ.get("CGX_CHUNKS_PER_TILE")


def test_layered_sizes_and_argument_checks(lib, oracle):
    """A bucket size per layer (paper Sec. 4.1: per-layer compression parameters): sizes follow the
    oracle's layout, bad sizes and missing arrays are refused before anything is queued."""
    rng = np.random.default_rng(3)
    for _ in range(20):
        L = int(rng.integers(1, 10))
        sizes = rng.choice([0, 1, 31, 96, 1000, 2048, 4097, 9000], L)
        off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
        bits = rng.integers(0, 9, L).astype(np.uint8)
        buckets = rng.choice([32, 64, 96, 128, 512, 1024, 4096, 8192], L).astype(np.int32)
        for dt in (wl.F32, wl.F16):
            assert cgx.cgx_layered_sizes(cgx.LayeredPlan(off, bits, buckets, dt)) == \
                oracle.layered_sizes(off, bits, buckets, dt)
        same = np.full(L, 512, np.int32)
        assert cgx.cgx_layered_sizes(cgx.LayeredPlan(off, bits, same)) == cgx.cgx_sizes(cgx.Plan(off, bits, 512))
    off = np.array([0, 100, 300], np.int64)
    bits = np.array([4, 0], np.uint8)
    pb, mb = ctypes.c_size_t(), ctypes.c_size_t()
    for bad in ([16, 32], [32, 100], [8224, 32], [32, 0]):      # also the entry of the pass-through layer
        bk = np.array(bad, np.int32)
        assert lib.cgx_layered_sizes(300, 2, off.ctypes.data, bits.ctypes.data, bk.ctypes.data, 0,
                                     ctypes.byref(pb), ctypes.byref(mb)) == -5
        assert lib.cgx_layered_quantize(16, 300, 2, off.ctypes.data, bits.ctypes.data, bk.ctypes.data, 1, 0, 16, 16,
                                        None) == -5
    ok = np.array([64, 32], np.int32)
    assert lib.cgx_layered_sizes(300, 2, off.ctypes.data, bits.ctypes.data, None, 0, ctypes.byref(pb),
                                 ctypes.byref(mb)) == -1
    assert lib.cgx_layered_quantize(None, 300, 2, off.ctypes.data, bits.ctypes.data, ok.ctypes.data, 1, 0, 16, 16,
                                    None) == -1
    assert lib.cgx_layered_quantize(24, 300, 2, off.ctypes.data, bits.ctypes.data, ok.ctypes.data, 1, 0, 16, 16,
                                    None) == -9
    ptrs = (ctypes.c_void_p * 1)(16)
    assert lib.cgx_layered_dequant_reduce(ptrs, ptrs, 0, 300, 2, off.ctypes.data, bits.ctypes.data, ok.ctypes.data, 0,
                                          16, None) == -6
    assert lib.cgx_layered_dequant_reduce_requantize(ptrs, ptrs, 17, 300, 2, off.ctypes.data, bits.ctypes.data,
                                                     ok.ctypes.data, 0, 1, 16, 16, None) == -6
    assert lib.cgx_layered_requantize(16, 299, 2, off.ctypes.data, bits.ctypes.data, ok.ctypes.data, 1, 16, 16,
                                      None) == -2


def test_tiles_carry_their_bucket_size(lib):
    """Quantized tiles name their bucket size (info bits 12..20 = bucket / 32); pass-through tiles carry 0."""
    for bucket in (32, 96, 512, 2048, 8192):
        w = wl.tiny_mixed(seed=1, dt=wl.F32, bucket=bucket)
        tiles = cgx.cgx_plan_tiles(cgx.Plan(w.offsets, w.bits, bucket, w.dt))
        kind = (tiles["info"] >> 4) & 15
        size = ((tiles["info"] >> 12) & 0x1ff) * 32
        quantized = (kind != 2) & (kind != 3)
        assert (size[quantized] == bucket).all() and (size[~quantized] == 0).all()


def test_norm_and_sign_layered_sizes_and_checks(lib, oracle):
    rng = np.random.default_rng(4)
    for _ in range(10):
        L = int(rng.integers(1, 10))
        off = np.concatenate([[0], np.cumsum(rng.choice([0, 1, 31, 96, 1000, 2048, 4097], L))]).astype(np.int64)
        bits = rng.choice([0, 2, 3, 4, 8], L).astype(np.uint8)
        buckets = rng.choice([32, 64, 96, 128, 512, 1024, 4096, 8192], L).astype(np.int32)
        assert cgx.cgx_qsgd_layered_sizes(cgx.LayeredPlan(off, bits, buckets)) == oracle.qsgd_layered_sizes(off, bits, buckets)
    off = np.array([0, 100, 300], np.int64)
    one_bit = np.array([1, 4], np.uint8)
    ok = np.array([64, 32], np.int32)
    pb, mb = ctypes.c_size_t(), ctypes.c_size_t()
    assert lib.cgx_qsgd_layered_sizes(300, 2, off.ctypes.data, one_bit.ctypes.data, ok.ctypes.data, 0, ctypes.byref(pb),
                                      ctypes.byref(mb)) == -4
    bits = np.array([2, 4], np.uint8)
    assert lib.cgx_qsgd_layered_quantize(16, 300, 2, off.ctypes.data, bits.ctypes.data, None, 1, 0, 16, 16, None) == -1
    bad = np.array([64, 48], np.int32)
    assert lib.cgx_qsgd_layered_quantize(16, 300, 2, off.ctypes.data, bits.ctypes.data, bad.ctypes.data, 1, 0, 16, 16,
                                         None) == -5


def test_binding_refuses_buffers_the_kernels_would_overrun(lib, monkeypatch):
    """The C ABI sees no sizes, so the binding checks them: device, contiguity, element type and length of
    every tensor against the plan, before the call.  Stand-ins with a tensor's attributes and no memory take
    the place of device tensors here; the compute entry points are replaced by a stub that reports that a
    call got past the checks."""
    import torch

    class Stub:
        def __getattr__(self, name):
            if name.endswith("sizes") or "workspace" in name or name == "cgx_status_string":
                return getattr(lib, name)

            def reached(*args):
                raise AssertionError("the call went through to the library")
            return reached

    monkeypatch.setattr(cgx, "lib", lambda: Stub())

    class Fake:
        """A stand-in with the attributes the checks read (no memory behind it: never passed to the library)."""
        def __init__(self, n, dtype=torch.float32, cuda=True, contiguous=True):
            self.n, self.dtype, self.is_cuda, self._c, self.device = n, dtype, cuda, contiguous, "cuda:0" if cuda else "cpu"
        def numel(self): return self.n
        def element_size(self): return torch.empty(0, dtype=self.dtype).element_size()
        def is_contiguous(self): return self._c
        def data_ptr(self): return 0x1000

    off = np.array([0, 4096, 5000], np.int64)
    plan = cgx.Plan(off, np.array([4, 0], np.uint8), 128)
    pb, mb = cgx.cgx_sizes(plan)
    good = dict(grad=Fake(5000), packed=Fake(pb, torch.uint8), meta=Fake(mb // 4))

    def quantize(**kw):
        a = {**good, **kw}
        cgx.cgx_quantize(a["grad"], plan, 1, a["packed"], a["meta"], stream=0)

    for bad in (dict(grad=Fake(4999)), dict(grad=Fake(5000, torch.float16)), dict(grad=Fake(5000, cuda=False)),
                dict(grad=Fake(5000, contiguous=False)), dict(packed=Fake(pb - 1, torch.uint8)),
                dict(meta=Fake(mb // 4 - 1)), dict(meta=Fake(mb // 4, torch.float64)), dict(grad=np.zeros(5000, np.float32)),
                dict(grad=torch.zeros(5000))):
        with pytest.raises(ValueError):
            quantize(**bad)
    with pytest.raises(AssertionError, match="went through"):
        quantize()                                                   # the good set passes every check
    half = cgx.Plan(off, np.array([4, 0], np.uint8), 128, wl.F16)
    with pytest.raises(ValueError, match="float16"):
        cgx.cgx_quantize(Fake(5000), half, 1, good["packed"], good["meta"], stream=0)
    chunks, metas = [Fake(pb, torch.uint8)] * 3, [Fake(mb // 4)] * 3
    with pytest.raises(ValueError, match="sum"):
        cgx.cgx_dequant_reduce(chunks, metas, plan, Fake(4999), stream=0)
    with pytest.raises(ValueError, match="chunk 2"):
        cgx.cgx_dequant_reduce(chunks[:2] + [Fake(pb - 16, torch.uint8)], metas, plan, Fake(5000), stream=0)
    with pytest.raises(ValueError, match="as many"):
        cgx.cgx_dequant_reduce(chunks, metas[:2], plan, Fake(5000), stream=0)
    with pytest.raises(ValueError, match="local"):
        cgx.cgx_dequant_reduce_add(Fake(5000, torch.float16), wl.F32, chunks, metas, plan, Fake(5000), stream=0)
    with pytest.raises(ValueError, match="output"):
        cgx.cgx_dequantize(chunks[0], metas[0], plan, wl.F16, Fake(5000), stream=0)      # float32 where binary16 is due
    with pytest.raises(ValueError, match="output"):
        cgx.cgx_dequant_reduce_requantize(chunks, metas, plan, 3, Fake(pb - 1, torch.uint8), metas[0], stream=0)
    with pytest.raises(ValueError):
        cgx.cgx_requantize(Fake(5000, torch.float16), plan, 1, good["packed"], good["meta"], stream=0)
    with pytest.raises(ValueError, match="workspace"):
        cgx.cgx_layer_sqnorms(Fake(5000), plan, Fake(2, torch.float64), Fake(1 << 20, torch.uint8, cuda=False), stream=0)
    with pytest.raises(ValueError, match="sqnorm"):
        cgx.cgx_layer_sqnorms_noalloc(Fake(5000), plan, Fake(1, torch.float64), stream=0)
    qp, qm = cgx.cgx_qsgd_sizes(plan)
    assert qm == mb // 2
    with pytest.raises(AssertionError, match="went through"):
        cgx.cgx_qsgd_quantize(Fake(5000), plan, 1, Fake(qp, torch.uint8), Fake(qm // 4), stream=0)
    with pytest.raises(ValueError, match="meta"):
        cgx.cgx_qsgd_quantize(Fake(5000), plan, 1, Fake(qp, torch.uint8), Fake(qm // 4 - 1), stream=0)


def test_group_to_bucket_lookup_by_multiply_and_shift_is_exact():
    """The kernels that stream buckets of a size that is no power of two find the bucket of group G of a tile
    as (G * ceil(2^16 / gb)) >> 16, gb = groups of 8 elements per bucket: equal to G // gb for every group of a
    chunk (G < 256) and every bucket size up to the chunk (gb <= 256)."""
    G = np.arange(256, dtype=np.uint64)
    for gb in range(1, 257):
        inv = (65536 + gb - 1) // gb
        assert np.array_equal((G * np.uint64(inv)) >> np.uint64(16), G // np.uint64(gb)), gb
