#!/usr/bin/env python3
"""Benchmark of the CGX hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch: cgx_quantize of
a fused gradient buffer, cgx_dequant_reduce over W compressed chunks, and
cgx_requantize of the sum.  Inputs are resident in HBM before the timed region.

The headline workload is the 1.3 B-parameter decoder (the larger of the two
target configurations); the 25.6 M-parameter ResNet-50 plan is measured in the
same run and reported as a second block of the same JSON line.
Prints ONE JSON line (see --help for the knobs).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak
NAMES = ["quantize", "dequant_reduce", "requantize"]


class TimingEvent:
    """A HIP event that is only a time stamp on a stream: created with hipEventDisableSystemFence, so that
    recording it does not write back and invalidate the caches (the default event, torch.cuda.Event, does, and
    the launch behind it then starts from a flushed cache hierarchy, a state that launches which follow each
    other directly never see).  Measured on the 25.6 M-element plan, the same library on both sides: the gap
    that a record leaves between two launches went from 5.8 to 4.6 us and the event-timed calls from
    23.9 / 39.4 / 28.8 us to 22.5 / 36.9 / 24.8 us.  Times are read after a device synchronisation."""
    DISABLE_SYSTEM_FENCE = 0x20000000
    _hip = None

    @classmethod
    def runtime(cls):
        if cls._hip is None:
            import ctypes
            import torch  # noqa: F401  (its HIP runtime is the one already in the process)
            hip = ctypes.CDLL("libamdhip64.so.7")
            hip.hipEventCreateWithFlags.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint]
            hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
            hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
            hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
            cls._hip = hip
        return cls._hip

    def __init__(self):
        import ctypes
        self.handle = ctypes.c_void_p()
        status = self.runtime().hipEventCreateWithFlags(ctypes.byref(self.handle), self.DISABLE_SYSTEM_FENCE)
        if status != 0:
            raise RuntimeError("hipEventCreateWithFlags failed with status %d" % status)

    def record(self, stream=None):
        import torch
        s = stream if stream is not None else torch.cuda.current_stream()
        status = self.runtime().hipEventRecord(self.handle, getattr(s, "cuda_stream", s))
        if status != 0:
            raise RuntimeError("hipEventRecord failed with status %d" % status)

    def elapsed_time(self, later):
        import ctypes
        ms = ctypes.c_float()
        status = self.runtime().hipEventElapsedTime(ctypes.byref(ms), self.handle, later.handle)
        if status != 0:
            raise RuntimeError("hipEventElapsedTime failed with status %d" % status)
        return float(ms.value)

    def __del__(self):
        if self.handle and self._hip is not None and not sys.is_finalizing():
            self._hip.hipEventDestroy(self.handle)
            self.handle = None


def algorithmic_bytes(tiles, bucket, elem_bytes, W, meta_per_bucket=8):
    """Bytes the method itself must move per launch, evaluated from the plan:
    quantize reads S and writes b/8 per element plus 8 per bucket (4 for the
    norm-and-sign form; pass-through: S in, S out); dequant-reduce reads W times
    the packed stream and meta and writes 4 per element."""
    import numpy as np
    bits = (tiles["info"] & 15).astype(np.int64)
    count = tiles["count"].astype(np.int64)
    q = bits > 0
    payload = np.where(q, (count * bits + 7) // 8, count * elem_bytes).sum()
    buckets = np.where(q, (count + bucket - 1) // bucket, 0).sum()
    n = int(count.sum())
    packed_meta = int(payload + meta_per_bucket * buckets)
    return {
        "n": n,
        "packed_meta": packed_meta,
        "quantize": n * elem_bytes + packed_meta,
        "dequant_reduce": W * packed_meta + 4 * n,
        "requantize": 4 * n + int(np.where(q, (count * bits + 7) // 8, count * 4).sum() + meta_per_bucket * buckets),
    }


def read_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed counter summary of this workload
    (profiles/hbm_traffic_<workload>.txt: lines `kernel fetch_bytes write_bytes`), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % workload)
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 3 and parts[0] == kernel:
                    return int(float(parts[1]) + float(parts[2]))
    except OSError:
        pass
    return None


def rate(nbytes, ms):
    """{ms, algorithmic bytes, GB/s, fraction of the HBM peak} of one launch."""
    return {"ms": round(ms, 5), "algorithmic_bytes": int(nbytes),
            "algorithmic_GBps": round(nbytes / ms / 1e6, 1),
            "hbm_frac": round(nbytes / ms / 1e6 / HBM_PEAK_GBPS, 4)}


def measure(name, args, extras=True):
    """Times the step of one workload and its kernels; returns (result dict, workload, host gradient)."""
    import numpy as np
    import torch

    from paper_2111_08617_amd import binding as cgx
    from paper_2111_08617_amd import workloads as wl

    dev = torch.device("cuda:0")
    w = wl.WORKLOADS[name]()
    W = w.W
    S = 2 if w.dt == wl.F16 else 4

    # the reduce step runs on one rank's share when the buffer is large (1/W of it), else on the full buffer
    on_share = name in ("gpt2_medium", "decoder_1p3b", "bert_base")
    if on_share:
        first, r_off, r_bits = wl.share_subplan(w.offsets, w.bits, w.bucket, W, W // 2)
    else:
        first, r_off, r_bits = 0, w.offsets, w.bits
    q_plan = cgx.Plan(w.offsets, w.bits, w.bucket, w.dt)
    r_plan = cgx.Plan(r_off, r_bits, w.bucket, w.dt)         # reduce: chunks in the storage type's layout
    rq_plan = cgx.Plan(r_off, r_bits, w.bucket, wl.F32)       # requantize: binary32 sum in
    m = r_plan.n
    q_pb, q_mb = cgx.cgx_sizes(q_plan)
    r_pb, r_mb = cgx.cgx_sizes(r_plan)
    rq_pb, rq_mb = cgx.cgx_sizes(rq_plan)

    q_alg = algorithmic_bytes(cgx.cgx_plan_tiles(q_plan), w.bucket, S, W)["quantize"]
    r_algs = algorithmic_bytes(cgx.cgx_plan_tiles(r_plan), w.bucket, S, W)
    alg = {"quantize": q_alg, "dequant_reduce": r_algs["dequant_reduce"], "requantize": r_algs["requantize"]}
    chunk_bytes = r_algs["packed_meta"]                       # one peer's packed stream + meta of the share

    traffic = q_alg + alg["dequant_reduce"] + alg["requantize"]
    R = args.rotate if args.rotate > 0 else max(2, min(8, int(np.ceil(2.5e9 / traffic))))

    # ---- inputs, resident in HBM before timing
    t0 = time.time()
    host_grad = w.gradient(0, threads=16)
    grads = [torch.from_numpy(host_grad).to(dev)]
    for _ in range(1, R):
        grads.append(grads[0].clone())
    share_grads = [torch.from_numpy(w.gradient(p, first, first + m, threads=16)).to(dev) for p in range(W)]
    chunk_sets = []
    for r in range(R):
        ps, ms = [], []
        for p in range(W):
            packed = torch.empty(r_pb, dtype=torch.uint8, device=dev)
            meta = torch.empty(max(r_mb // 4, 4), dtype=torch.float32, device=dev)
            cgx.cgx_quantize(share_grads[p], r_plan, w.quant_seed(p) + 1000 * r, packed, meta)
            ps.append(packed)
            ms.append(meta)
        chunk_sets.append((ps, ms))
    locals32 = [share_grads[0].float().clone() for _ in range(R)] if extras else None
    del share_grads
    q_out = [(torch.empty(q_pb, dtype=torch.uint8, device=dev),
              torch.empty(max(q_mb // 4, 4), dtype=torch.float32, device=dev)) for _ in range(R)]
    sums = [torch.empty(m, dtype=torch.float32, device=dev) for _ in range(R)]
    rq_out = [(torch.empty(rq_pb, dtype=torch.uint8, device=dev),
               torch.empty(max(rq_mb // 4, 4), dtype=torch.float32, device=dev)) for _ in range(R)]
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    def step(i, ev=None, only=None):
        """One step; ev: four events recorded around the three calls (only = j: just the two around call j).
        An event record costs about 3 us of stream time, so the timed region carries few of them."""
        r = i % R
        if ev and only in (None, 0):
            ev[0].record()
        cgx.cgx_quantize(grads[r], q_plan, 17 + i, q_out[r][0], q_out[r][1])
        if ev and only in (None, 0, 1):
            ev[1].record()
        cgx.cgx_dequant_reduce(chunk_sets[r][0], chunk_sets[r][1], r_plan, sums[r])
        if ev and only in (None, 1, 2):
            ev[2].record()
        cgx.cgx_requantize(sums[r], rq_plan, 29 + i, rq_out[r][0], rq_out[r][1])
        if ev and only in (None, 2):
            ev[3].record()

    def new_events(k, per=4):
        return [[TimingEvent() for _ in range(per)] for _ in range(k)]

    def all_ms(evs, j):
        return np.array([e[j].elapsed_time(e[j + 1]) for e in evs])

    def mean_ms(evs, j):
        return float(np.mean(all_ms(evs, j)))

    # spin-up (part of the set-up): the step itself, until the clocks have settled
    spin_steps = 0
    t_spin = time.perf_counter()
    while (time.perf_counter() - t_spin) * 1e3 < args.spin_up_ms:
        for _ in range(8):
            step(spin_steps)
            spin_steps += 1
        torch.cuda.synchronize()

    # warmup, with events on every call: it also tells which kernel dominates the step
    warm_events = new_events(args.warmup)
    for i in range(args.warmup):
        step(i, warm_events[i])
    torch.cuda.synchronize()
    if args.warmup > 0:
        dom = int(np.argmax([mean_ms(warm_events[args.warmup // 2:], j) for j in range(3)]))
    else:
        dom = int(np.argmax([alg[k] for k in NAMES]))

    # timed region: exactly `steps` steps; the dominant kernel is bracketed by two events on every
    # `stride`-th step (about 25 samples), nothing else sits between the launches
    stride = max(1, args.steps // 25)
    events = new_events(args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i % stride == 0:
            step(i, events[i], only=dom)
        else:
            step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    dominant_ms = mean_ms(events[::stride], dom)

    # per-kernel breakdown, outside the timed region: the same steps with events around every call
    all_events = new_events(args.steps)
    for i in range(args.steps):
        step(i, all_events[i])
    torch.cuda.synchronize()

    def timed(fn, reps=None):
        """Mean event time of fn(i) over some launches (outside the timed region)."""
        for i in range(max(args.warmup // 2, 2)):
            fn(i)
        reps = reps or max(args.steps // 2, 5)
        evs = new_events(reps, 2)
        torch.cuda.synchronize()
        for i in range(reps):
            evs[i][0].record()
            fn(i)
            evs[i][1].record()
        torch.cuda.synchronize()
        return float(np.mean([a.elapsed_time(b) for a, b in evs]))

    # the same step with the quantize (own buffer) and the reduce + requantize (received chunks) on two
    # streams of equal priority: the two are independent in a scatter-reduce, so one's tail fills
    # with the other's head
    overlapped = None
    if extras:
        s_a, s_b = torch.cuda.Stream(), torch.cuda.Stream()

        def overlapped_step(i):
            r = i % R
            cgx.cgx_quantize(grads[r], q_plan, 17 + i, q_out[r][0], q_out[r][1], stream=s_a)
            cgx.cgx_dequant_reduce(chunk_sets[r][0], chunk_sets[r][1], r_plan, sums[r], stream=s_b)
            cgx.cgx_requantize(sums[r], rq_plan, 29 + i, rq_out[r][0], rq_out[r][1], stream=s_b)

        torch.cuda.synchronize()
        for i in range(args.warmup):
            overlapped_step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            overlapped_step(i)
        torch.cuda.synchronize()
        ov_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        overlapped = {"step": "cgx_quantize on one stream, cgx_dequant_reduce + cgx_requantize on another",
                      "ms_per_step": round(ov_ms, 5),
                      "value": round((w.n * S + 8 * m) / (ov_ms * 1e6), 1)}

    # the same step as one captured graph of R steps (one per buffer set), replayed: what the launches of the
    # three calls cost when the host is out of the way (the plans' tables exist by now, so capture is legal)
    graph_leg = None
    if extras:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for r in range(R):
                step(r)
        torch.cuda.synchronize()
        replays = max(1, -(-args.steps // R))
        for _ in range(max(1, args.warmup // R)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - t0) * 1e3 / (replays * R)
        graph_leg = {"step": "the three calls of %d steps captured in one graph, replayed %d times" % (R, replays),
                     "ms_per_step": round(g_ms, 5), "value": round((w.n * S + 8 * m) / (g_ms * 1e6), 1)}
        del graph

    # the same rank's work with the fused entry point: quantize + dequant_reduce_requantize
    fused = None
    if W <= cgx.MAX_FUSED_PEERS and (extras or args.with_fused):
        def fused_step(i):
            r = i % R
            cgx.cgx_quantize(grads[r], q_plan, 17 + i, q_out[r][0], q_out[r][1])
            cgx.cgx_dequant_reduce_requantize(chunk_sets[r][0], chunk_sets[r][1], r_plan, 29 + i, rq_out[r][0],
                                              rq_out[r][1])

        for i in range(args.warmup):
            fused_step(i)
        fe = new_events(args.steps, 2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            r = i % R
            cgx.cgx_quantize(grads[r], q_plan, 17 + i, q_out[r][0], q_out[r][1])
            fe[i][0].record()
            cgx.cgx_dequant_reduce_requantize(chunk_sets[r][0], chunk_sets[r][1], r_plan, 29 + i, rq_out[r][0],
                                              rq_out[r][1])
            fe[i][1].record()
        torch.cuda.synchronize()
        fused_wall = (time.perf_counter() - t0) * 1e3 / args.steps
        fused_kernel_ms = float(np.mean([a.elapsed_time(b) for a, b in fe]))
        fused_alg = alg["dequant_reduce"] - 4 * m + (alg["requantize"] - 4 * m)
        # the fused kernel is bound by the vector ALUs, not by HBM: 46 vector instructions per element at 4 bit
        # and W = 8 (stored: profiles/alu_counters_rocprofv3.md, SQ_INSTS_VALU per wave / elements per wave)
        # against 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3 T lane-instructions/s
        alu_peak = 256 * 4 * 16 * 2.4e9
        fused = {"step": "cgx_quantize(full buffer) + cgx_dequant_reduce_requantize(W chunks)",
                 "ms_per_step": round(fused_wall, 5),
                 "dequant_reduce_requantize": dict(rate(fused_alg, fused_kernel_ms),
                                                   raw_gradient_GBps=round(4 * m / fused_kernel_ms / 1e6, 1),
                                                   bound="alu",
                                                   alu_frac_at_46_instructions_per_element=round(
                                                       46.0 * m / (fused_kernel_ms * 1e-3) / alu_peak, 4))}

    # the remaining calls of a rank's scatter-reduce / all-gather: decompression of a gathered chunk into the
    # storage type, and the reduce with the rank's own contribution still uncompressed
    next_rows = None
    if extras:
        out32 = sums
        out16 = [torch.empty(m, dtype=torch.float16, device=dev) for _ in range(min(R, 2))]
        deq32 = timed(lambda i: cgx.cgx_dequantize(chunk_sets[i % R][0][0], chunk_sets[i % R][1][0], r_plan, wl.F32,
                                                   out32[i % R]))
        deq16 = timed(lambda i: cgx.cgx_dequantize(chunk_sets[i % R][0][0], chunk_sets[i % R][1][0], r_plan, wl.F16,
                                                   out16[i % len(out16)]))
        add = timed(lambda i: cgx.cgx_dequant_reduce_add(locals32[i % R], wl.F32, chunk_sets[i % R][0][:W - 1],
                                                         chunk_sets[i % R][1][:W - 1], r_plan, sums[i % R]))
        next_rows = {
            "dequantize_to_f32": dict(rate(chunk_bytes + 4 * m, deq32), W=1),
            "dequantize_to_f16": dict(rate(chunk_bytes + 2 * m, deq16), W=1),
            "dequant_reduce_add": dict(rate((W - 1) * chunk_bytes + 4 * m + 4 * m, add), W=W - 1,
                                       local="binary32, uncompressed"),
            "bytes": "dequantize: packed + meta of one chunk + S_out per element; reduce_add: (W-1) chunks + the "
                     "local binary32 term + the binary32 sum",
        }
        del out16
    del locals32

    # the same step with the norm-and-sign form of the quantizer (Sec. 2.3, Q_s), timed per kernel
    norm_sign = None
    if extras and not (w.bits == 1).any():
        ns_meta = lambda mb: torch.empty(max(mb // 8, 4), dtype=torch.float32, device=dev)
        ns_chunks = []
        share = [torch.from_numpy(w.gradient(p, first, first + m, threads=16)).to(dev) for p in range(W)]
        for r in range(R):
            ps, ms = [], []
            for p in range(W):
                packed = torch.empty(r_pb, dtype=torch.uint8, device=dev)
                meta = ns_meta(r_mb)
                cgx.cgx_qsgd_quantize(share[p], r_plan, w.quant_seed(p) + 1000 * r, packed, meta)
                ps.append(packed)
                ms.append(meta)
            ns_chunks.append((ps, ms))
        del share
        ns_q = [ns_meta(q_mb) for _ in range(R)]
        ns_rq = [ns_meta(rq_mb) for _ in range(R)]

        def ns_step(i, ev=None):
            r = i % R
            if ev:
                ev[0].record()
            cgx.cgx_qsgd_quantize(grads[r], q_plan, 17 + i, q_out[r][0], ns_q[r])
            if ev:
                ev[1].record()
            cgx.cgx_qsgd_dequant_reduce(ns_chunks[r][0], ns_chunks[r][1], r_plan, sums[r])
            if ev:
                ev[2].record()
            cgx.cgx_qsgd_quantize(sums[r], rq_plan, 29 + i, rq_out[r][0], ns_rq[r])
            if ev:
                ev[3].record()

        for i in range(args.warmup):
            ns_step(i)
        ne = new_events(args.steps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            ns_step(i, ne[i])
        torch.cuda.synchronize()
        ns_wall = (time.perf_counter() - t0) * 1e3 / args.steps
        ns_alg = {"quantize": algorithmic_bytes(cgx.cgx_plan_tiles(q_plan), w.bucket, S, W, 4)["quantize"]}
        ns_r = algorithmic_bytes(cgx.cgx_plan_tiles(r_plan), w.bucket, S, W, 4)
        ns_alg.update(dequant_reduce=ns_r["dequant_reduce"], requantize=ns_r["requantize"])
        norm_sign = {"step": "cgx_qsgd_quantize + cgx_qsgd_dequant_reduce + cgx_qsgd_quantize(sum)",
                     "ms_per_step": round(ns_wall, 5)}
        for j, k in enumerate(NAMES):
            norm_sign[k] = rate(ns_alg[k], mean_ms(ne, j))
        del ns_chunks

    # per-layer statistics of the adaptive scheme: squared norms of the full buffer, squared
    # compression error of the full buffer's chunk (read-only kernels: bytes in / time)
    layer_stats = None
    if extras:
        ws_bytes = max(cgx.cgx_layer_stats_workspace(q_plan), cgx.cgx_layer_stats_workspace(q_plan, for_sqnorms=True), 16)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        stat_out = torch.empty(w.L, dtype=torch.float64, device=dev)
        for r in range(R):
            cgx.cgx_quantize(grads[r], q_plan, 17 + r, q_out[r][0], q_out[r][1])
        sqn_ms = timed(lambda i: cgx.cgx_layer_sqnorms(grads[i % R], q_plan, stat_out, ws))
        sqe_ms = timed(lambda i: cgx.cgx_layer_sqerrors(grads[i % R], q_out[i % R][0], q_out[i % R][1], q_plan, stat_out, ws))
        layer_stats = {"sqnorms": rate(w.n * S, sqn_ms), "sqerrors": rate(alg["quantize"], sqe_ms),
                       "note": "each figure covers the tile kernel and the per-layer sum kernel (two launches)"}
        del ws

    # what the memory system gives a plain streaming kernel with each call's read:write mix at its size
    # (in the kernel's own shape: bytes of the larger side per wave, non-temporal loads and stores, 256 threads)
    def probe_ms(read_bytes, write_bytes, slice_bytes):
        rb, wb = read_bytes // 16 * 16, write_bytes // 16 * 16
        srcs = [torch.empty(rb, dtype=torch.uint8, device=dev) for _ in range(R)]
        dsts = [torch.empty(max(wb, 16), dtype=torch.uint8, device=dev) for _ in range(R)]
        return timed(lambda i: cgx.cgx_stream_probe_shaped(srcs[i % R], rb, dsts[i % R], wb, slice_bytes))

    probe = None
    if extras:
        probe = {
            "quantize": probe_ms(w.n * S, alg["quantize"] - w.n * S, 4096),       # a chunk is 4 KB of input
            "dequant_reduce": probe_ms(alg["dequant_reduce"] - 4 * m, 4 * m, 8192),  # a chunk is 8 KB of sums
            "requantize": probe_ms(4 * m, alg["requantize"] - 4 * m, 4096),
        }

    kern_ms = {k: mean_ms(all_events, j) for j, k in enumerate(NAMES)}
    raw_bytes = {"quantize": w.n * S, "dequant_reduce": 4 * m, "requantize": 4 * m}
    kernels = {}
    for k in NAMES:
        ms_k = all_ms(all_events, NAMES.index(k))
        kernels[k] = dict(rate(alg[k], kern_ms[k]), ms_median=round(float(np.median(ms_k)), 5),
                          ms_min=round(float(np.min(ms_k)), 5),
                          raw_gradient_GBps=round(raw_bytes[k] / kern_ms[k] / 1e6, 1))
        if k == "dequant_reduce":
            # the W chunks stand for W gradients of the share: can exceed the HBM peak, not a roofline figure
            kernels[k]["represented_gradient_GBps"] = round(4 * W * m / kern_ms[k] / 1e6, 1)
        if probe:
            kernels[k].update(stream_probe_ms=round(probe[k], 5),
                              stream_probe_GBps=round(alg[k] // 16 * 16 / probe[k] / 1e6, 1),
                              frac_of_stream_probe=round(probe[k] / kern_ms[k], 4))
    dominant = NAMES[dom]
    achieved = alg[dominant] / dominant_ms / 1e6
    value = sum(raw_bytes.values()) / (ms_per_step * 1e6)

    result = {
        "value": round(value, 1),
        "ms_per_step": round(ms_per_step, 5),
        "dtype": "f16" if w.dt == wl.F16 else "f32",
        "config": {
            "workload": w.name,
            "description": w.description,
            "elements": w.n,
            "reduce_elements": m,
            "reduce_on": "1/%d share of the buffer" % W if on_share else "full buffer",
            "W": W,
            "bucket": w.bucket,
            "step": "cgx_quantize(full buffer) + cgx_dequant_reduce(W chunks) + cgx_requantize(sum)",
            "value_definition": "raw gradient bytes entering quantize + leaving dequant_reduce + entering "
                                "requantize, per second of step wall time (the three calls on one stream)",
            "buffer_sets_rotated": R,
            "spin_up_steps_before_warmup": spin_steps,
        },
        "kernels": kernels,
        "kernels_timing": "a pass of the same steps after the timed region, HIP events around every call",
        "roofline": {
            "bound": "hbm",
            "kernel": dominant,
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": read_traffic(w.name, dominant),
            "traffic_source": "stored: profiles/hbm_traffic_%s.txt, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs "
                              "of this command (not measured in this run)" % w.name,
            "launch_ms": round(dominant_ms, 5),
            "timing": "HIP events around %d of the %d launches of the timed region (every %d-th step)"
                      % (len(events[::stride]), args.steps, stride),
        },
        "two_streams": overlapped,
        "graph": graph_leg,
        "fused": fused,
        "next_rows": next_rows,
        "norm_sign": norm_sign,
        "layer_stats": layer_stats,
        "setup_s": round(setup_s, 1),
    }
    return result, w, host_grad


def cpu_baseline(w, host_grad):
    """The oracle, as it stands, on a bounded sample of the workload: one whole step."""
    import numpy as np

    import oracle
    from paper_2111_08617_amd import workloads as wl

    W = w.W
    S = 2 if w.dt == wl.F16 else 4
    cores = oracle.get_max_threads()
    # bounded sample: whole step for small workloads, else the first tensors up to ~64M elements
    cap = 64_000_000
    L_s = int(np.searchsorted(w.offsets, cap, side="right")) - 1 if w.n > cap else w.L
    L_s = max(L_s, 1)
    off_s, bits_s = w.offsets[:L_s + 1], w.bits[:L_s]
    n_s = int(off_s[-1])
    g_s = host_grad[:n_s]
    cpu_bytes = n_s * S + 4 * n_s + 4 * n_s

    def oracle_step():
        t0 = time.perf_counter()
        cp, cm = oracle.quantize(g_s, off_s, bits_s, w.bucket, 17, w.dt)
        t1 = time.perf_counter()
        s32 = oracle.dequant_reduce([cp] * W, [cm] * W, off_s, bits_s, w.bucket, w.dt, want=("sum32",))["sum32"]
        t2 = time.perf_counter()
        oracle.quantize(s32, off_s, bits_s, w.bucket, 29, wl.F32)
        t3 = time.perf_counter()
        return np.array([t1 - t0, t2 - t1, t3 - t2])

    # all threads: repeated until about 3 s have passed (at least twice), mean of the repeats
    runs = [oracle_step()]
    while len(runs) < 2 or (sum(r.sum() for r in runs) < 3.0 and len(runs) < 20):
        runs.append(oracle_step())
    t_all = np.mean(runs, axis=0)
    # one thread, once
    single = None
    if n_s <= 128_000_000:
        oracle.set_threads(1)
        t_one = oracle_step()
        oracle.set_threads(cores)
        single = {"value": round(cpu_bytes / t_one.sum() / 1e9, 3), "unit": "GB/s", "cores": 1,
                  "seconds": [round(float(t), 3) for t in t_one]}
    return {
        "value": round(cpu_bytes / t_all.sum() / 1e9, 3),
        "unit": "GB/s",
        "cores": cores,
        "kind": "oracle",
        "sample": "one step (quantize + dequant_reduce W=%d + requantize) on the first %d tensors / %d "
                  "elements of %s, OpenMP over buckets, mean of %d repeats" % (W, L_s, n_s, w.name, len(runs)),
        "seconds": {"quantize": round(float(t_all[0]), 3), "dequant_reduce": round(float(t_all[1]), 3),
                    "requantize": round(float(t_all[2]), 3)},
        "single_thread": single,
    }


CEILING_CASES = [
    # name, bytes read, bytes written: the read:write mixes and sizes of the calls of the two target workloads,
    # and pure reads / writes / copies of the same sizes
    ("quantize resnet50 (8:1, 115 MB)", 102_228_128, 13_167_184),
    ("dequant_reduce resnet50 (1:1, 208 MB)", 105_337_472, 102_228_128),
    ("quantize decoder_1p3b (6:1, 6.1 GB)", 5_262_893_056, 844_533_008),
    ("dequant_reduce decoder_1p3b share (5:4, 1.5 GB)", 811_545_472, 657_858_560),
    ("requantize decoder_1p3b share (6:1, 0.76 GB)", 657_858_560, 101_443_184),
    ("dequantize decoder_1p3b share (1:8, 0.74 GB)", 83_500_000, 657_858_560),
    ("dequantize resnet50 (1:8, 115 MB)", 13_167_184, 102_228_128),
    ("read only, 115 MB", 115_343_360, 0),
    ("read only, 1.5 GB", 1_500_000_256, 0),
    ("read only, 6 GB", 6_000_000_000, 0),
    ("write only, 115 MB", 0, 115_343_360),
    ("write only, 1.5 GB", 0, 1_500_000_256),
    ("write only, 6 GB", 0, 6_000_000_000),
    ("copy 1:1, 115 MB", 57_671_680, 57_671_680),
    ("copy 1:1, 1.5 GB", 750_000_128, 750_000_128),
    ("copy 1:1, 6 GB", 3_000_000_000, 3_000_000_000),
]


def issue_rates(args):
    """Cost of each vector instruction form in cycles of a SIMD at the nominal clock: every SIMD of the chip
    holds 8 waves that each execute 16 * iterations instructions of the form in independent chains."""
    import torch

    from paper_2111_08617_amd import binding as cgx

    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    cus, clock_ghz, iterations, blocks = 256, 2.4, 2000, 256 * 8
    out = torch.empty(blocks * 256, dtype=torch.int32, device="cuda")
    rows = []
    for form, text in enumerate(cgx.cgx_issue_probe_forms()):
        cgx.cgx_issue_probe(form, blocks, 10, out)
        times = []
        for _ in range(max(3, args.steps // 4)):
            a, b = TimingEvent(), TimingEvent()
            a.record(stream)
            cgx.cgx_issue_probe(form, blocks, iterations, out)
            b.record(stream)
            torch.cuda.synchronize()
            times.append(a.elapsed_time(b))
        ms = min(times)
        per_simd = blocks * 4 * 16 * iterations / (cus * 4)
        rows.append({"form": text, "ms": round(ms, 4), "cycles_per_instruction": round(ms * 1e-3 * clock_ghz * 1e9 / per_simd, 2),
                     "T_lane_ops_per_s": round(blocks * 4 * 16 * iterations * 64 / ms / 1e9, 2)})
    print(json.dumps({"mode": "issue_rates", "compute_units": cus, "clock_GHz": clock_ghz, "waves_per_simd": 8,
                      "instructions_per_wave": 16 * iterations, "forms": rows}))


def size_sweep(args):
    """Launch time against size: cgx_quantize, cgx_dequant_reduce (W = 8) and the streaming probe in the kernels'
    shape on single-layer plans of 8 to 200 M elements (4 bit, buckets of 1024).  A straight-line fit of time
    against algorithmic bytes separates what a launch costs once (the intercept) from what it sustains while it
    streams (the slope).  Event-timed here; under `rocprofv3 --kernel-trace` the dispatches give the pure
    kernel times (the last 12 launches of each kernel at each size are the timed ones)."""
    import numpy as np
    import torch

    from paper_2111_08617_amd import binding as cgx

    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    reps, W = 12, 8
    rows = []
    for mega in (8, 16, 25, 50, 100, 200):
        n = mega * 1024 * 1024
        plan = cgx.Plan(np.array([0, n], np.int64), np.array([4], np.uint8), 1024)
        pb, mb = cgx.cgx_sizes(plan)
        R = max(2, min(8, int(2.5e9 / (n * 4.5))))
        g = [torch.randn(n, device=dev) for _ in range(R)]
        # R sets of W chunks: no launch finds its input in the memory-side cache
        outs = [(torch.empty(pb, dtype=torch.uint8, device=dev), torch.empty(mb // 4, device=dev)) for _ in range(W * R)]
        for p in range(W * R):
            cgx.cgx_quantize(g[p % R], plan, p, outs[p][0], outs[p][1])
        sets = [([o[0] for o in outs[r * W:(r + 1) * W]], [o[1] for o in outs[r * W:(r + 1) * W]]) for r in range(R)]
        calls = {
            "quantize": (n * 4 + pb + mb,
                         lambda i: cgx.cgx_quantize(g[i % R], plan, i, outs[i % (W * R)][0], outs[i % (W * R)][1])),
            "probe_quantize_shape": (n * 4 + pb // 16 * 16,
                                     lambda i: cgx.cgx_stream_probe_shaped(g[i % R], n * 4, outs[i % (W * R)][0],
                                                                           pb // 16 * 16, 4096, 256, "nt", "nt")),
            "dequant_reduce": (W * (pb + mb) + 4 * n,
                               lambda i: cgx.cgx_dequant_reduce(sets[i % R][0], sets[i % R][1], plan, g[(i + 1) % R])),
        }
        for name, (nbytes, fn) in calls.items():
            # the call itself for 40 ms first: the clocks swing for the first 10 to 15 ms of a load
            t_spin, i = time.perf_counter(), 0
            while (time.perf_counter() - t_spin) * 1e3 < 40.0:
                for _ in range(8):
                    fn(i)
                    i += 1
                torch.cuda.synchronize()
            evs = [[TimingEvent() for _ in range(2)] for _ in range(reps)]
            torch.cuda.synchronize()
            for i in range(reps):
                evs[i][0].record(stream)
                fn(i)
                evs[i][1].record(stream)
            torch.cuda.synchronize()
            ms = float(np.median([a.elapsed_time(b) for a, b in evs]))
            rows.append({"call": name, "elements": n, "bytes": nbytes, "ms": round(ms, 5),
                         "hbm_frac": round(nbytes / ms / 1e6 / HBM_PEAK_GBPS, 4)})
        del g, outs
        torch.cuda.empty_cache()
    fits = {}
    for name in ("quantize", "probe_quantize_shape", "dequant_reduce"):
        x = np.array([r["bytes"] / 1e6 for r in rows if r["call"] == name])
        y = np.array([r["ms"] * 1e3 for r in rows if r["call"] == name])
        slope, intercept = np.polyfit(x, y, 1)
        fits[name] = {"us_per_MB": round(float(slope), 4), "us_per_launch": round(float(intercept), 2),
                      "streaming_frac_of_peak": round(1.0 / float(slope) / (HBM_PEAK_GBPS / 1e3), 4)}
    print(json.dumps({"mode": "size_sweep", "timed_launches_per_size": reps, "rows": rows, "fits_by_events": fits}))


def bucket_sizes(args):
    """cgx_quantize, cgx_dequant_reduce (W = 8) and cgx_dequant_reduce_requantize on one layer of 64 M elements
    (4 bit) for bucket sizes that are powers of two and sizes that are not.  Event-timed; under
    `rocprofv3 --kernel-trace` every call is a run of 13 launches of one kernel (3 warm-up + 10 timed) after the
    8 quantize launches that make the chunks."""
    import numpy as np
    import torch

    from paper_2111_08617_amd import binding as cgx

    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    rows = []
    for bucket in (128, 1024, 2048, 96, 160, 672, 992, 1056, 2016):
        n = 64 * 1024 * 1024 // (bucket * 32) * (bucket * 32)
        plan = cgx.Plan(np.array([0, n], np.int64), np.array([4], np.uint8), bucket)
        pb, mb = cgx.cgx_sizes(plan)
        g = [torch.randn(n, device=dev) for _ in range(3)]
        outs = [(torch.empty(pb, dtype=torch.uint8, device=dev), torch.empty(mb // 4, device=dev)) for _ in range(8)]
        for p in range(8):
            cgx.cgx_quantize(g[p % 3], plan, p, outs[p][0], outs[p][1])
        total = torch.empty(n, device=dev)
        fused_out = (torch.empty(pb, dtype=torch.uint8, device=dev), torch.empty(mb // 4, device=dev))
        packed, metas = [o[0] for o in outs], [o[1] for o in outs]

        def timed(fn, reps=10):
            for i in range(3):
                fn(i)
            ev = [[TimingEvent() for _ in range(2)] for _ in range(reps)]
            torch.cuda.synchronize()
            for i in range(reps):
                ev[i][0].record(stream)
                fn(i)
                ev[i][1].record(stream)
            torch.cuda.synchronize()
            return float(np.median([a.elapsed_time(b) for a, b in ev]))

        q = timed(lambda i: cgx.cgx_quantize(g[i % 3], plan, i, outs[i % 8][0], outs[i % 8][1]))
        r = timed(lambda i: cgx.cgx_dequant_reduce(packed, metas, plan, total))
        f = timed(lambda i: cgx.cgx_dequant_reduce_requantize(packed, metas, plan, i, fused_out[0], fused_out[1]))
        q_bytes, r_bytes, f_bytes = n * 4 + pb + mb, 8 * (pb + mb) + 4 * n, 9 * (pb + mb)
        rows.append({"bucket": bucket, "elements": n,
                     "quantize": rate(q_bytes, q), "dequant_reduce": rate(r_bytes, r),
                     "dequant_reduce_requantize": rate(f_bytes, f)})
        del g, outs, total, fused_out, packed, metas
        torch.cuda.empty_cache()
    print(json.dumps({"mode": "bucket_sizes", "bits": 4, "W": 8, "rows": rows}))


def ceilings(args):
    """What a kernel that only moves bytes sustains, by launch shape and cache policy: a staged sweep of
    cgx_stream_probe_shaped per (size, read:write mix).  Stage 1: every load x store policy at the kernels' own
    shape; stage 2: slice size x block size x die-contiguous numbering for the best three policy pairs; stage 3:
    persistent grids for the best shape.  Event-timed, median of `reps` launches over rotated buffers."""
    import numpy as np
    import torch

    from paper_2111_08617_amd import binding as cgx

    dev = torch.device("cuda:0")
    reps = max(args.steps // 2, 7)
    out = {"mode": "ceilings", "peak_GBps": HBM_PEAK_GBPS, "reps": reps, "cases": []}
    pick = [c for c in CEILING_CASES if args.ceilings_case in c[0]]
    for name, rb, wb in pick:
        rb, wb = rb // 16 * 16, wb // 16 * 16
        R = max(2, min(8, int(np.ceil(2.5e9 / (rb + wb)))))
        srcs = [torch.zeros(max(rb, 16), dtype=torch.uint8, device=dev) for _ in range(R)]
        dsts = [torch.empty(max(wb, 16), dtype=torch.uint8, device=dev) for _ in range(R)]
        tried, order = {}, []

        def run(slice_bytes=8192, block=256, loads="nt", stores="nt", xcd=False, max_blocks=0):
            key = (slice_bytes, block, loads, stores, xcd, max_blocks)
            if key in tried:
                return tried[key]
            call = lambda i: cgx.cgx_stream_probe_shaped(srcs[i % R], rb, dsts[i % R], wb, slice_bytes, block, loads,
                                                         stores, xcd, max_blocks)
            for i in range(2):
                call(i)
            evs = [[TimingEvent() for _ in range(2)] for _ in range(reps)]
            torch.cuda.synchronize()
            for i in range(reps):
                evs[i][0].record()
                call(i)
                evs[i][1].record()
            torch.cuda.synchronize()
            ms = float(np.median([a.elapsed_time(b) for a, b in evs]))
            tried[key] = ms
            order.append(list(key))
            return ms

        base = run()
        for loads in cgx.LOAD_POLICIES if rb else ("nt",):
            for stores in cgx.STORE_POLICIES if wb else ("nt",):
                run(loads=loads, stores=stores)
        best_pol = [kv[0] for kv in sorted({(k[2], k[3]): v for k, v in tried.items()}.items(), key=lambda kv: kv[1])[:3]]
        if ("nt", "nt") not in best_pol:
            best_pol.append(("nt", "nt"))                    # the kernels' own policies: always swept over the shapes
        for loads, stores in best_pol:
            for slice_bytes in (2048, 4096, 8192, 16384, 32768, 65536):
                for block in (64, 256, 1024):
                    for xcd in (False, True):
                        run(slice_bytes, block, loads, stores, xcd)
        best = min(tried, key=tried.get)
        for max_blocks in (256, 512, 1024, 2048, 4096, 8192):
            for slice_bytes in (8192, 65536, 1 << 20):
                run(slice_bytes, best[1], best[2], best[3], best[4], max_blocks)
        best = min(tried, key=tried.get)
        rows = [{"slice_bytes": k[0], "block_threads": k[1], "loads": k[2], "stores": k[3], "die_contiguous": k[4],
                 "max_blocks": k[5], "ms": round(v, 5), "GBps": round((rb + wb) / v / 1e6, 1),
                 "hbm_frac": round((rb + wb) / v / 1e6 / HBM_PEAK_GBPS, 4)} for k, v in sorted(tried.items(), key=lambda kv: kv[1])]
        out["cases"].append({"case": name, "read_bytes": rb, "write_bytes": wb, "buffer_sets_rotated": R,
                             "kernels_own_shape": {"ms": round(base, 5),
                                                   "hbm_frac": round((rb + wb) / base / 1e6 / HBM_PEAK_GBPS, 4)},
                             "best": rows[0], "configs_tried": len(rows), "top": rows[:12],
                             "policies_at_own_shape": [r for r in rows if (r["slice_bytes"], r["block_threads"],
                                                                             r["die_contiguous"], r["max_blocks"]) ==
                                                       (8192, 256, False, 0)],
                             "all": rows if args.ceilings_all else None,
                             # execution order, 2 + reps launches each (to match a kernel trace of this run)
                             "order": order if args.ceilings_all else None})
        del srcs, dsts
        torch.cuda.empty_cache()
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="decoder_1p3b",
                    choices=["single_1m", "resnet50", "bert_base", "gpt2_medium", "decoder_1p3b"],
                    help="the headline workload")
    ap.add_argument("--also", default="resnet50",
                    help="a second workload measured in the same run and reported as a block of its own "
                         "('none': only the headline workload)")
    ap.add_argument("--also-steps", type=int, default=1000,
                    help="the second workload is timed over at least this many steps (its step is short)")
    ap.add_argument("--rotate", type=int, default=0,
                    help="distinct buffer sets cycled through so that launches do not re-hit the 256 MB "
                         "memory-side cache (0 = enough for 2.5 GB of traffic)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--spin-up-ms", type=float, default=50.0,
                    help="untimed steps run for this long before the warmup steps, so that the clocks have "
                         "settled whatever --warmup is (the first ~10 ms of activity run slower)")
    ap.add_argument("--step-only", action="store_true",
                    help="time the step alone: no two-stream / fused / other entry points / norm-and-sign / "
                         "statistics / probe legs and no second workload (for counter runs, where every dispatch "
                         "is slow)")
    ap.add_argument("--with-fused", action="store_true",
                    help="with --step-only: run the fused leg (quantize + dequant_reduce_requantize) as well")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain elementwise kernel that reads 1 GiB and writes 1 GiB three times: "
                         "under `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE` its known size gives the factor "
                         "that scales the counters to bytes")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of the step: sweep the arithmetic-free streaming probe over launch shapes and cache "
                         "policies at the sizes and read:write mixes of the calls (what the memory system allows)")
    ap.add_argument("--issue-rates", action="store_true",
                    help="instead of the benchmark: what each vector instruction form of the kernels' inner loops costs "
                         "a SIMD (cgx_issue_probe), one JSON line")
    ap.add_argument("--size-sweep", action="store_true",
                    help="instead of the benchmark: quantize, dequant_reduce and the probe on single-layer plans of "
                         "8 to 200 M elements, with a straight-line fit of time against bytes")
    ap.add_argument("--bucket-sizes", action="store_true",
                    help="instead of the benchmark: quantize, dequant_reduce and the fused call on one 64 M-element layer "
                         "for bucket sizes that are powers of two and sizes that are not")
    ap.add_argument("--ceilings-case", default="", help="with --ceilings: only the cases whose name contains this")
    ap.add_argument("--ceilings-all", action="store_true", help="with --ceilings: list every configuration tried")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the W peers of the reduce step are W compressed "
                 "chunks resident in HBM); run with --gpus 1")

    import torch

    from paper_2111_08617_amd import binding as cgx

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    cgx.lib()
    if args.issue_rates:
        issue_rates(args)
        return
    if args.size_sweep:
        size_sweep(args)
        return
    if args.bucket_sizes:
        bucket_sizes(args)
        return
    if args.ceilings:
        ceilings(args)
        return

    head, w, host_grad = measure(args.workload, args, extras=not args.step_only)
    result = {
        "metric": "GB/s of fp32 gradient quantized and dequant-reduced (W=8); % of HBM peak",
        "value": head.pop("value"),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head.pop("ms_per_step"),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": head.pop("dtype"),
        "data": "synthetic",
    }
    result.update(head)

    if args.calibration_copy:
        # an elementwise kernel that reads 1 GiB and writes 1 GiB (grid unlike any cgx launch)
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    result["cpu_baseline"] = None if args.no_cpu_baseline else cpu_baseline(w, host_grad)
    del host_grad

    if args.also != "none" and args.also != args.workload and not args.step_only:
        torch.cuda.empty_cache()
        # A step of the second workload is short (about 90 us for resnet50): 20 of them say little, and they would
        # be timed right after the heavy legs of the headline workload.  It gets at least --also-steps steps.
        import copy
        also_args = copy.copy(args)
        also_args.steps = max(args.steps, args.also_steps)
        also_args.warmup = max(args.warmup, min(50, args.also_steps // 10))
        second, _, _ = measure(args.also, also_args, extras=True)
        second["unit"] = "GB/s"
        second["steps"] = also_args.steps
        second["warmup"] = also_args.warmup
        result[args.also] = second

    print(json.dumps(result))


if __name__ == "__main__":
    main()
