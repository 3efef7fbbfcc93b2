"""Seeded synthetic gradient workloads.

This module only builds layer tables and draws input values; it holds none of
the quantizer's arithmetic and is the one piece shared by the GPU path's tests,
the CPU oracle's tests and the benchmark.

The paper evaluates on training runs of ResNet-50, BERT, GPT-2 and other
models (Sec. 6, "Experimental Validation"); their gradients are replaced here
by synthetic buffers that take those models' parameter shapes, fused in
parameter order into one buffer with a layer offset table (Sec. 4.1, fused
buffers and layer offsets).  Small one-dimensional tensors (bias,
normalisation) are marked pass-through (bits = 0), following the layer filter
of Sec. 4.1 and the evaluation set-up of Sec. 6.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Callable, List, Sequence, Tuple

import numpy as np

F32, F16 = 0, 1


# --------------------------------------------------------------------------
# parameter shapes, in parameter order
# --------------------------------------------------------------------------

def resnet50_shapes() -> List[Tuple[int, ...]]:
    shapes: List[Tuple[int, ...]] = [(64, 3, 7, 7), (64,), (64,)]
    inplanes = 64
    for planes, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for blk in range(blocks):
            shapes += [(planes, inplanes, 1, 1), (planes,), (planes,),
                       (planes, planes, 3, 3), (planes,), (planes,),
                       (planes * 4, planes, 1, 1), (planes * 4,), (planes * 4,)]
            if blk == 0:
                shapes += [(planes * 4, inplanes, 1, 1), (planes * 4,), (planes * 4,)]
            inplanes = planes * 4
    shapes += [(1000, 2048), (1000,)]
    return shapes


def bert_base_shapes() -> List[Tuple[int, ...]]:
    h, ffn = 768, 3072
    shapes: List[Tuple[int, ...]] = [(30522, h), (512, h), (2, h), (h,), (h,)]
    for _ in range(12):
        for _ in range(4):                      # query, key, value, attention output
            shapes += [(h, h), (h,)]
        shapes += [(h,), (h,)]                  # attention LayerNorm
        shapes += [(ffn, h), (ffn,), (h, ffn), (h,)]
        shapes += [(h,), (h,)]                  # output LayerNorm
    shapes += [(h, h), (h,)]                    # pooler
    return shapes


def gpt2_shapes(hidden: int, ffn: int, layers: int, vocab: int, ctx: int) -> List[Tuple[int, ...]]:
    shapes: List[Tuple[int, ...]] = [(vocab, hidden), (ctx, hidden)]
    for _ in range(layers):
        shapes += [(hidden,), (hidden,),
                   (hidden, 3 * hidden), (3 * hidden,),
                   (hidden, hidden), (hidden,),
                   (hidden,), (hidden,),
                   (hidden, ffn), (ffn,),
                   (ffn, hidden), (hidden,)]
    shapes += [(hidden,), (hidden,)]
    return shapes


# --------------------------------------------------------------------------
# value distributions (binary32 draws; tensor t of peer w has its own stream)
# --------------------------------------------------------------------------

def _normal(rng, n, scale):
    return rng.standard_normal(n, dtype=np.float32) * np.float32(scale)


def _student_t3(rng, n, scale):
    z = rng.standard_normal(n, dtype=np.float32)
    chi2 = rng.standard_gamma(1.5, n, dtype=np.float32) * np.float32(2.0)     # chi-square, 3 d.o.f.
    return z / np.sqrt(chi2 / np.float32(3.0)) * np.float32(scale)


def _sparse_normal(rng, n, scale):
    x = rng.standard_normal(n, dtype=np.float32) * np.float32(scale)
    x[rng.random(n, dtype=np.float32) < np.float32(0.2)] = 0.0
    return x


def _laplace_outliers(rng, n, scale):
    mag = rng.standard_exponential(n, dtype=np.float32) * np.float32(scale)
    u = rng.random(n, dtype=np.float32)
    x = np.where(u < np.float32(0.5), -mag, mag)
    x[rng.random(n, dtype=np.float32) < np.float32(0.001)] *= np.float32(100.0)
    return x


@dataclass
class Workload:
    """A fused gradient buffer: layer table, per-layer bits, bucket, value recipe."""
    name: str
    shapes: List[Tuple[int, ...]]
    bits: np.ndarray                 # uint8[L]; 0 = pass-through
    bucket: int
    dt: int                          # storage type of the gradient: F32 or F16
    W: int                           # peers in the reduce step
    seed: int
    draw: Callable = field(repr=False, default=_normal)
    scales: np.ndarray = field(repr=False, default=None)   # per-tensor scale
    description: str = ""

    def __post_init__(self):
        sizes = np.array([int(np.prod(s)) for s in self.shapes], dtype=np.int64)
        self.offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
        self.bits = np.ascontiguousarray(self.bits, dtype=np.uint8)
        assert self.bits.size == len(self.shapes)

    @property
    def n(self) -> int:
        return int(self.offsets[-1])

    @property
    def L(self) -> int:
        return len(self.shapes)

    @property
    def np_dtype(self):
        return np.float16 if self.dt == F16 else np.float32

    def quant_seed(self, peer: int) -> int:
        """Seed peer w passes to the quantizer."""
        return self.seed + peer

    def layer_values(self, layer: int, peer: int = 0) -> np.ndarray:
        lo, hi = int(self.offsets[layer]), int(self.offsets[layer + 1])
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([self.seed, layer, peer])))
        return self.draw(rng, hi - lo, float(self.scales[layer])).astype(self.np_dtype, copy=False)

    def gradient(self, peer: int = 0, lo: int = 0, hi: int | None = None, threads: int = 8) -> np.ndarray:
        """Elements [lo, hi) of peer w's fused gradient buffer, in the storage type."""
        hi = self.n if hi is None else hi
        out = np.empty(hi - lo, dtype=self.np_dtype)
        todo = [l for l in range(self.L) if self.offsets[l + 1] > lo and self.offsets[l] < hi
                and self.offsets[l + 1] > self.offsets[l]]

        def fill(l):
            a, b = int(self.offsets[l]), int(self.offsets[l + 1])
            v = self.layer_values(l, peer)
            s, e = max(a, lo), min(b, hi)
            out[s - lo:e - lo] = v[s - a:e - a]

        if threads > 1 and len(todo) > 1:
            with ThreadPoolExecutor(max_workers=threads) as ex:
                list(ex.map(fill, todo))
        else:
            for l in todo:
                fill(l)
        return out


def random_plan(seed: int) -> Workload:
    """A seeded random plan: layer lengths from nothing to a few chunks (whole chunks, whole
    buckets, odd lengths, empty layers), any width per layer, any bucket size, either
    storage type, 1 to 9 peers, per-tensor scales over five decades."""
    rng = np.random.default_rng(1000 + seed)
    bucket = int(rng.choice([32, 64, 96, 128, 256, 512, 1024, 2048, 4096, 8192]))
    L = int(rng.integers(1, 14))
    sizes = []
    for _ in range(L):
        kind = rng.integers(0, 6)
        if kind == 0:
            sizes.append(int(rng.integers(0, 40)))
        elif kind == 1:
            sizes.append(2048 * int(rng.integers(1, 7)))
        elif kind == 2:
            sizes.append(bucket * int(rng.integers(1, 9)))
        elif kind == 3:
            sizes.append(2048 * int(rng.integers(1, 5)) + int(rng.integers(1, 2048)))
        else:
            sizes.append(int(rng.integers(1, 30000)))
    bits = rng.integers(0, 9, L).astype(np.uint8)
    dt = F16 if rng.integers(0, 2) else F32
    scales = 10.0 ** rng.uniform(-4, 1, L)
    draw = [_normal, _student_t3, _sparse_normal, _laplace_outliers][int(rng.integers(0, 4))]
    return Workload(f"random{seed}", [(int(t),) for t in sizes], bits, bucket, dt, int(rng.integers(1, 10)), seed, draw,
                    scales)


def _log_uniform_scales(seed: int, L: int, lo: float, hi: float) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0x5ca1e5])))
    return np.exp(rng.uniform(np.log(lo), np.log(hi), L))


def _bits_for(shapes: Sequence[Tuple[int, ...]], choices: Sequence[int], seed: int,
              passthrough: Callable[[Tuple[int, ...]], bool]) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0xb175])))
    drawn = rng.choice(np.asarray(choices, dtype=np.uint8), size=len(shapes))
    return np.array([0 if passthrough(s) else int(b) for s, b in zip(shapes, drawn)], dtype=np.uint8)


def _one_dim(shape) -> bool:
    return len(shape) == 1


def single_tensor(seed: int = 0) -> Workload:
    shapes = [(1 << 20,)]
    return Workload("single_1m", shapes, np.array([4], np.uint8), 128, F32, 2, seed, _normal,
                    np.array([0.01]), "one binary32 tensor of 2^20 elements ~ N(0, 0.01^2), 4 bit, bucket 128")


def resnet50(seed: int = 1) -> Workload:
    shapes = resnet50_shapes()
    bits = np.array([0 if int(np.prod(s)) <= 2048 else 4 for s in shapes], np.uint8)
    return Workload("resnet50", shapes, bits, 1024, F32, 8, seed, _normal,
                    _log_uniform_scales(seed, len(shapes), 1e-4, 1e-1),
                    "161 ResNet-50 tensors, N(0, s^2) with s log-uniform in [1e-4, 1e-1], 4 bit, bucket 1024, "
                    "tensors <= 2048 elements pass-through")


def bert_base(seed: int = 2) -> Workload:
    shapes = bert_base_shapes()
    return Workload("bert_base", shapes, _bits_for(shapes, (2, 3, 4, 8), seed, _one_dim), 512, F32, 8, seed,
                    _student_t3, _log_uniform_scales(seed, len(shapes), 1e-4, 1e-1),
                    "199 BERT-base tensors, Student-t(3) scaled per tensor, bits in {2,3,4,8}, bucket 512, "
                    "1-D tensors pass-through")


def gpt2_medium(seed: int = 3) -> Workload:
    shapes = gpt2_shapes(1024, 4096, 24, 50257, 1024)
    bits = np.array([0 if _one_dim(s) else 4 for s in shapes], np.uint8)
    return Workload("gpt2_medium", shapes, bits, 128, F16, 8, seed, _sparse_normal,
                    np.full(len(shapes), 1e-3),
                    "292 GPT-2-medium tensors in binary16 storage, 20% exact zeros, rest N(0, 1e-3^2), 4 bit, "
                    "bucket 128, 1-D tensors pass-through")


def decoder_1p3b(seed: int = 4) -> Workload:
    shapes = gpt2_shapes(2048, 8192, 24, 50257, 2048)
    return Workload("decoder_1p3b", shapes, _bits_for(shapes, (2, 4, 8), seed, _one_dim), 1024, F32, 8, seed,
                    _laplace_outliers, _log_uniform_scales(seed, len(shapes), 1e-4, 1e-1),
                    "292 tensors of a 1.3B decoder (hidden 2048, FFN 8192, 24 layers, context 2048), Laplace values "
                    "with 0.1% outliers x100, bits in {2,4,8}, bucket 1024, 1-D tensors pass-through")


WORKLOADS = {
    "single_1m": single_tensor,
    "resnet50": resnet50,
    "bert_base": bert_base,
    "gpt2_medium": gpt2_medium,
    "decoder_1p3b": decoder_1p3b,
}


def tiny_mixed(seed: int = 7, dt: int = F32, bucket: int = 64) -> Workload:
    """A small buffer with every kind of layer the plan allows: all bit widths,
    pass-through layers, empty layers, layers shorter than a bucket, ragged
    last buckets and offsets that are not multiples of 8."""
    sizes = [5000, 37, 0, 64, 4096 + 13, 1, 8 * bucket, 2 * bucket + 31, 1000, 3, 12345, 777, 2048]
    bits = [4, 0, 3, 2, 8, 5, 1, 3, 0, 4, 6, 7, 2]
    shapes = [(s,) for s in sizes]
    return Workload("tiny_mixed", shapes, np.array(bits, np.uint8), bucket, dt, 3, seed, _normal,
                    _log_uniform_scales(seed, len(shapes), 1e-3, 1.0), "edge-case plan for the parity tests")


# --------------------------------------------------------------------------
# one rank's share of a scatter-reduce, as a clipped sub-plan
# --------------------------------------------------------------------------

def share_subplan(offsets: np.ndarray, bits: np.ndarray, bucket: int, W: int, r: int):
    """Rank r's share of the buffer in a W-way scatter-reduce (Sec. 4.1,
    Scatter-Reduce-Allgather: the vector is divided into N chunks).

    The cut points k*n/W are moved down to the start of the bucket (quantized
    layers) or to a multiple of 8 elements (pass-through layers) they fall in.
    Returns (first_element, sub_offsets, sub_bits): a plan over the share alone,
    whose first layer may be the tail of a layer of the full plan.
    """
    offsets = np.asarray(offsets, dtype=np.int64)
    n, L = int(offsets[-1]), len(bits)

    def cut(k: int) -> int:
        if k <= 0:
            return 0
        if k >= W:
            return n
        c = (n * k) // W
        l = int(np.searchsorted(offsets, c, side="right") - 1)
        l = min(max(l, 0), L - 1)
        step = bucket if bits[l] else 8
        return int(offsets[l] + ((c - offsets[l]) // step) * step)

    a, b = cut(r), cut(r + 1)
    sub_off, sub_bits = [0], []
    for l in range(L):
        s, e = max(int(offsets[l]), a), min(int(offsets[l + 1]), b)
        if e > s:
            sub_off.append(sub_off[-1] + (e - s))
            sub_bits.append(int(bits[l]))
    return a, np.array(sub_off, dtype=np.int64), np.array(sub_bits, dtype=np.uint8)
