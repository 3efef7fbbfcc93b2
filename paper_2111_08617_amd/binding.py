"""ctypes binding of ``libcgx.so``: the functions of ``include/cgx.h`` under the
same names.  Argument marshalling only -- every step runs in the HIP kernels.

Device buffers are torch tensors (PyTorch supplies device memory and the
stream, nothing else); plan arrays are numpy arrays on the host.  There is no
CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Sequence, Tuple

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcgx.so")

F32, F16 = 0, 1
MAX_PEERS = 64
MAX_FUSED_PEERS = 16

EXPORTS = ("cgx_sizes", "cgx_quantize", "cgx_dequant_reduce", "cgx_dequant_reduce_add", "cgx_dequantize",
           "cgx_requantize",
           "cgx_dequant_reduce_requantize", "cgx_qsgd_sizes", "cgx_qsgd_quantize", "cgx_qsgd_dequant_reduce",
           "cgx_qsgd_dequant_reduce_requantize", "cgx_layer_stats_workspace", "cgx_layer_sqnorms",
           "cgx_layer_sqnorms_noalloc", "cgx_layer_sqerrors", "cgx_qsgd_layer_sqerrors", "cgx_assign_bits_kmeans", "cgx_assign_bits_linear",
           "cgx_assign_buckets_from_bits", "cgx_layered_sizes", "cgx_layered_quantize", "cgx_layered_dequant_reduce", "cgx_layered_requantize",
           "cgx_layered_dequant_reduce_requantize", "cgx_layered_dequant_reduce_add", "cgx_layered_dequantize",
           "cgx_layered_stats_workspace", "cgx_layered_layer_sqerrors", "cgx_qsgd_layered_sizes",
           "cgx_qsgd_layered_quantize", "cgx_qsgd_layered_dequant_reduce", "cgx_qsgd_layered_dequant_reduce_requantize",
           "cgx_plan_tiles", "cgx_plan_tiles_chunk", "cgx_stream_probe", "cgx_stream_probe_shaped",
           "cgx_issue_probe", "cgx_issue_probe_form", "cgx_status_string", "cgx_shutdown")

TILE_DTYPE = np.dtype([("elem0", "<i8"), ("packed_off", "<i8"), ("bucket0", "<u4"), ("count", "<u4"),
                       ("info", "<u4"), ("pad", "<u4")])

_lib = None


class CgxError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def lib() -> ctypes.CDLL:
    """Loads the built library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2111_08617_amd.build` "
                "(there is no fallback implementation)")
        L = ctypes.CDLL(LIB_PATH)
        c = ctypes
        plan = [c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_int32]
        L.cgx_sizes.argtypes = plan + [c.c_int, c.POINTER(c.c_size_t), c.POINTER(c.c_size_t)]
        L.cgx_quantize.argtypes = [c.c_void_p] + plan + [c.c_uint64, c.c_int, c.c_void_p, c.c_void_p, c.c_void_p]
        L.cgx_requantize.argtypes = [c.c_void_p] + plan + [c.c_uint64, c.c_void_p, c.c_void_p, c.c_void_p]
        L.cgx_dequant_reduce.argtypes = [c.c_void_p, c.c_void_p, c.c_int32] + plan + [c.c_int, c.c_void_p, c.c_void_p]
        L.cgx_dequant_reduce_add.argtypes = [c.c_void_p, c.c_int, c.c_void_p, c.c_void_p, c.c_int32] + plan + \
            [c.c_int, c.c_void_p, c.c_void_p]
        L.cgx_dequantize.argtypes = [c.c_void_p, c.c_void_p] + plan + [c.c_int, c.c_int, c.c_void_p, c.c_void_p]
        L.cgx_dequant_reduce_requantize.argtypes = [c.c_void_p, c.c_void_p, c.c_int32] + plan + \
            [c.c_int, c.c_uint64, c.c_void_p, c.c_void_p, c.c_void_p]
        layered = [c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p]
        L.cgx_layered_sizes.argtypes = layered + [c.c_int, c.POINTER(c.c_size_t), c.POINTER(c.c_size_t)]
        L.cgx_layered_quantize.argtypes = [c.c_void_p] + layered + [c.c_uint64, c.c_int, c.c_void_p, c.c_void_p,
                                                                     c.c_void_p]
        L.cgx_layered_requantize.argtypes = [c.c_void_p] + layered + [c.c_uint64, c.c_void_p, c.c_void_p, c.c_void_p]
        L.cgx_layered_dequant_reduce.argtypes = [c.c_void_p, c.c_void_p, c.c_int32] + layered + \
            [c.c_int, c.c_void_p, c.c_void_p]
        L.cgx_layered_dequant_reduce_requantize.argtypes = [c.c_void_p, c.c_void_p, c.c_int32] + layered + \
            [c.c_int, c.c_uint64, c.c_void_p, c.c_void_p, c.c_void_p]
        L.cgx_layered_dequant_reduce_add.argtypes = [c.c_void_p, c.c_int, c.c_void_p, c.c_void_p, c.c_int32] + layered + \
            [c.c_int, c.c_void_p, c.c_void_p]
        L.cgx_layered_dequantize.argtypes = [c.c_void_p, c.c_void_p] + layered + [c.c_int, c.c_int, c.c_void_p, c.c_void_p]
        L.cgx_layered_stats_workspace.argtypes = layered + [c.c_int, c.POINTER(c.c_size_t)]
        L.cgx_layered_layer_sqerrors.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p] + layered + \
            [c.c_int, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
        L.cgx_qsgd_layered_sizes.argtypes = L.cgx_layered_sizes.argtypes
        L.cgx_qsgd_layered_quantize.argtypes = L.cgx_layered_quantize.argtypes
        L.cgx_qsgd_layered_dequant_reduce.argtypes = L.cgx_layered_dequant_reduce.argtypes
        L.cgx_qsgd_layered_dequant_reduce_requantize.argtypes = L.cgx_layered_dequant_reduce_requantize.argtypes
        L.cgx_qsgd_sizes.argtypes = L.cgx_sizes.argtypes
        L.cgx_qsgd_quantize.argtypes = L.cgx_quantize.argtypes
        L.cgx_qsgd_dequant_reduce.argtypes = L.cgx_dequant_reduce.argtypes
        L.cgx_qsgd_dequant_reduce_requantize.argtypes = L.cgx_dequant_reduce_requantize.argtypes
        L.cgx_layer_stats_workspace.argtypes = plan + [c.c_int, c.POINTER(c.c_size_t)]
        L.cgx_layer_sqnorms.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_void_p, c.c_int, c.c_void_p, c.c_void_p,
                                        c.c_size_t, c.c_void_p]
        L.cgx_layer_sqnorms_noalloc.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_void_p, c.c_int, c.c_void_p,
                                                c.c_void_p]
        L.cgx_layer_sqerrors.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p] + plan + \
            [c.c_int, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
        L.cgx_qsgd_layer_sqerrors.argtypes = L.cgx_layer_sqerrors.argtypes
        L.cgx_assign_bits_kmeans.argtypes = [c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32,
                                             c.c_int32, c.c_void_p]
        L.cgx_assign_bits_linear.argtypes = [c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32,
                                             c.c_void_p]
        L.cgx_assign_buckets_from_bits.argtypes = [c.c_int32, c.c_void_p, c.c_void_p, c.c_int32, c.c_void_p, c.c_int32,
                                                   c.c_void_p]
        L.cgx_stream_probe.argtypes = [c.c_void_p, c.c_size_t, c.c_void_p, c.c_size_t, c.c_void_p]
        L.cgx_stream_probe_shaped.argtypes = [c.c_void_p, c.c_size_t, c.c_void_p, c.c_size_t, c.c_void_p, c.c_void_p]
        L.cgx_plan_tiles.argtypes = plan + [c.c_int, c.c_void_p, c.c_int64, c.POINTER(c.c_int64)]
        L.cgx_plan_tiles_chunk.argtypes = plan + [c.c_int, c.c_int32, c.c_void_p, c.c_int64, c.POINTER(c.c_int64)]
        L.cgx_issue_probe.argtypes = [c.c_int32, c.c_int32, c.c_int32, c.c_void_p, c.c_size_t, c.c_void_p]
        L.cgx_issue_probe_form.restype = c.c_char_p
        L.cgx_issue_probe_form.argtypes = [c.c_int32]
        L.cgx_status_string.restype = c.c_char_p
        L.cgx_status_string.argtypes = [c.c_int]
        L.cgx_shutdown.argtypes = []
        for name in EXPORTS:
            if name not in ("cgx_status_string", "cgx_issue_probe_form"):
                getattr(L, name).restype = c.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().cgx_status_string(int(status)).decode()


class Plan:
    """Host arrays of a plan, kept alive and contiguous for the C calls."""

    def __init__(self, layer_offsets, bits_per_layer, bucket: int, dt: int = F32):
        self.offsets = np.ascontiguousarray(layer_offsets, dtype=np.int64)
        self.bits = np.ascontiguousarray(bits_per_layer, dtype=np.uint8)
        if self.offsets.ndim != 1 or self.bits.ndim != 1 or self.offsets.size != self.bits.size + 1:
            raise ValueError("layer_offsets must have one more entry than bits_per_layer")
        self.bucket = int(bucket)
        self.dt = int(dt)
        self.n = int(self.offsets[-1])
        self.L = int(self.bits.size)

    @property
    def args(self):
        return (self.n, self.L, self.offsets.ctypes.data, self.bits.ctypes.data, self.bucket)


class LayeredPlan:
    """A plan with a bucket size per layer (the cgx_layered_* calls)."""

    def __init__(self, layer_offsets, bits_per_layer, buckets_per_layer, dt: int = F32):
        self.offsets = np.ascontiguousarray(layer_offsets, dtype=np.int64)
        self.bits = np.ascontiguousarray(bits_per_layer, dtype=np.uint8)
        self.buckets = np.ascontiguousarray(buckets_per_layer, dtype=np.int32)
        if self.offsets.ndim != 1 or self.offsets.size != self.bits.size + 1 or self.buckets.shape != self.bits.shape:
            raise ValueError("one bits and one bucket entry per layer, one more layer offset")
        self.dt = int(dt)
        self.n = int(self.offsets[-1])
        self.L = int(self.bits.size)

    @property
    def args(self):
        return (self.n, self.L, self.offsets.ctypes.data, self.bits.ctypes.data, self.buckets.ctypes.data)


def _check(status: int, where: str) -> None:
    if status != 0:
        raise CgxError(status, where)


def _stream(stream) -> int:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    return int(getattr(stream, "cuda_stream", stream))


_TORCH_DTYPES = {F32: "float32", F16: "float16"}


_dtype_objects = {}


def _torch_dtype(name: str):
    if name not in _dtype_objects:
        import torch
        _dtype_objects[name] = getattr(torch, name)
    return _dtype_objects[name]


def _device_buffer(t, what, nbytes: int, dtype: str = None) -> int:
    """Address of a device tensor after the checks the C ABI cannot make (it sees no sizes): a contiguous
    device tensor of the expected element type holding at least nbytes bytes.  Raises ValueError.
    `what` names the argument in the message (a string, or a tuple of parts joined only when needed)."""
    try:
        ok = t.is_cuda and t.is_contiguous() and (dtype is None or t.dtype is _torch_dtype(dtype)) and \
            t.numel() * t.element_size() >= nbytes
    except AttributeError:
        ok = False
    if ok:
        return t.data_ptr()
    def flat(w):
        return [str(w)] if not isinstance(w, tuple) else [x for part in w for x in flat(part)]
    what = what if isinstance(what, str) else ": ".join([flat(what)[0], " ".join(flat(what)[1:])])
    if not hasattr(t, "data_ptr") or not hasattr(t, "is_cuda"):
        raise ValueError(f"{what}: a device tensor is needed, got {type(t).__name__}")
    if not t.is_cuda:
        raise ValueError(f"{what}: the tensor lives on {t.device}, the kernels need device memory")
    if not t.is_contiguous():
        raise ValueError(f"{what}: the tensor is not contiguous")
    if dtype is not None and t.dtype is not _torch_dtype(dtype):
        raise ValueError(f"{what}: element type {t.dtype}, expected torch.{dtype}")
    raise ValueError(f"{what}: {t.numel() * t.element_size()} bytes, the call needs {nbytes}")


def _elements(t, what, n: int, dt: int) -> int:
    """A buffer of n elements of storage type dt."""
    return _device_buffer(t, what, n * (2 if dt == F16 else 4), _TORCH_DTYPES[dt])


def _chunk(packed, meta, what, packed_bytes: int, meta_bytes: int):
    """One compressed chunk: the packed stream (any element type) and its float32 meta."""
    if meta_bytes:
        m = _device_buffer(meta, (what, "meta"), meta_bytes, "float32")
    else:
        m = _device_buffer(meta, (what, "meta"), 0) if meta is not None else 0
    return _device_buffer(packed, (what, "packed"), packed_bytes), m


def _peers(packed: Sequence, meta: Sequence, what: str, packed_bytes: int, meta_bytes: int):
    W = len(packed)
    if len(meta) != W:
        raise ValueError("as many meta tensors as packed tensors")
    pp, mp = (ctypes.c_void_p * max(W, 1))(), (ctypes.c_void_p * max(W, 1))()
    for w in range(W):
        pp[w], mp[w] = _chunk(packed[w], meta[w], (what, "chunk", w), packed_bytes, meta_bytes)
    return W, pp, mp


def _sizes_of(plan, qsgd: bool = False, dt: int = None) -> Tuple[int, int]:
    """(packed_bytes, meta_bytes) of a Plan or LayeredPlan, for either quantizer, optionally at another storage type."""
    dt = plan.dt if dt is None else dt
    cache = plan.__dict__.setdefault("_sizes", {})           # a plan's arrays are not changed after construction
    if (qsgd, dt) in cache:
        return cache[(qsgd, dt)]
    pb, mb = ctypes.c_size_t(), ctypes.c_size_t()
    if isinstance(plan, LayeredPlan):
        fn, name = (lib().cgx_qsgd_layered_sizes, "cgx_qsgd_layered_sizes") if qsgd else \
            (lib().cgx_layered_sizes, "cgx_layered_sizes")
    else:
        fn, name = (lib().cgx_qsgd_sizes, "cgx_qsgd_sizes") if qsgd else (lib().cgx_sizes, "cgx_sizes")
    _check(fn(*plan.args, dt, ctypes.byref(pb), ctypes.byref(mb)), name)
    cache[(qsgd, dt)] = (int(pb.value), int(mb.value))
    return cache[(qsgd, dt)]


def cgx_sizes(plan: Plan) -> Tuple[int, int]:
    """(packed_bytes, meta_bytes) of a plan."""
    return _sizes_of(plan)


def cgx_plan_tiles(plan: Plan, chunk: int = 2048) -> np.ndarray:
    """The tile table of a plan, for kernels with chunks of `chunk` elements (1024 or 2048), as a
    structured numpy array (host only)."""
    count = ctypes.c_int64()
    _check(lib().cgx_plan_tiles_chunk(*plan.args, plan.dt, chunk, None, 0, ctypes.byref(count)), "cgx_plan_tiles_chunk")
    tiles = np.zeros(count.value, dtype=TILE_DTYPE)
    _check(lib().cgx_plan_tiles_chunk(*plan.args, plan.dt, chunk, tiles.ctypes.data, count.value, ctypes.byref(count)),
           "cgx_plan_tiles_chunk")
    return tiles


_M64 = 2**64 - 1


def _quantize(name: str, qsgd: bool, grad, plan, seed: int, packed, meta, stream, requantize: bool = False) -> None:
    in_dt = F32 if requantize else plan.dt
    pb, mb = _sizes_of(plan, qsgd, in_dt)
    g = _elements(grad, (name, "input"), plan.n, in_dt)
    p, m = _chunk(packed, meta, (name, "output"), pb, mb)
    dt_arg = () if requantize else (plan.dt,)
    _check(getattr(lib(), name)(g, *plan.args, seed & _M64, *dt_arg, p, m, _stream(stream)), name)


def _reduce(name: str, qsgd: bool, packed, meta, plan, total, stream, local=None, local_dt: int = None) -> None:
    pb, mb = _sizes_of(plan, qsgd)
    W, pp, mp = _peers(packed, meta, name, pb, mb)
    out = _elements(total, (name, "sum"), plan.n, F32)
    head = () if local is None else (_elements(local, (name, "local"), plan.n, local_dt), local_dt)
    _check(getattr(lib(), name)(*head, pp, mp, W, *plan.args, plan.dt, out, _stream(stream)), name)


def _fused(name: str, qsgd: bool, packed, meta, plan, seed: int, packed_out, meta_out, stream) -> None:
    pb, mb = _sizes_of(plan, qsgd)
    ob, omb = _sizes_of(plan, qsgd, F32)
    W, pp, mp = _peers(packed, meta, name, pb, mb)
    po, mo = _chunk(packed_out, meta_out, (name, "output"), ob, omb)
    _check(getattr(lib(), name)(pp, mp, W, *plan.args, plan.dt, seed & _M64, po, mo, _stream(stream)), name)


def _dequantize(name: str, packed, meta, plan, out_dt: int, out, stream) -> None:
    if out_dt not in (F32, F16):
        raise ValueError(f"{name}: out_dt must be F32 or F16")
    pb, mb = _sizes_of(plan)
    p, m = _chunk(packed, meta, (name, "input"), pb, mb)
    o = _elements(out, (name, "output"), plan.n, out_dt)
    _check(getattr(lib(), name)(p, m, *plan.args, plan.dt, out_dt, o, _stream(stream)), name)


def cgx_quantize(grad, plan: Plan, seed: int, packed, meta, stream=None) -> None:
    """grad: device tensor of n elements (float32 or float16 per plan.dt);
    packed: device tensor of >= packed_bytes; meta: device float32 tensor of >= meta_bytes/4 elements."""
    _quantize("cgx_quantize", False, grad, plan, seed, packed, meta, stream)


def cgx_requantize(total, plan: Plan, seed: int, packed, meta, stream=None) -> None:
    """total: device float32 tensor of n elements (the reduced chunk); outputs sized for dt = F32."""
    _quantize("cgx_requantize", False, total, plan, seed, packed, meta, stream, requantize=True)


def cgx_dequant_reduce(packed: Sequence, meta: Sequence, plan: Plan, total, stream=None) -> None:
    """packed / meta: W device tensors each; total: device float32 tensor of n elements (output)."""
    _reduce("cgx_dequant_reduce", False, packed, meta, plan, total, stream)


def cgx_dequant_reduce_add(local, local_dt: int, packed: Sequence, meta: Sequence, plan: Plan, total, stream=None) -> None:
    """total = local + sum of the W dequantized chunks; local: device tensor of n elements (float32 / float16)."""
    if local_dt not in (F32, F16):
        raise ValueError("cgx_dequant_reduce_add: local_dt must be F32 or F16")
    _reduce("cgx_dequant_reduce_add", False, packed, meta, plan, total, stream, local, local_dt)


def cgx_dequantize(packed, meta, plan: Plan, out_dt: int, out, stream=None) -> None:
    """out: device tensor of n elements of out_dt (float32 or float16) receiving the decompressed chunk."""
    _dequantize("cgx_dequantize", packed, meta, plan, out_dt, out, stream)


def cgx_dequant_reduce_requantize(packed: Sequence, meta: Sequence, plan: Plan, seed: int, packed_out, meta_out,
                                  stream=None) -> None:
    """packed / meta: W <= 16 device tensors each (chunks of `plan`); packed_out / meta_out: device
    tensors sized by cgx_sizes of the same plan with dt = F32."""
    _fused("cgx_dequant_reduce_requantize", False, packed, meta, plan, seed, packed_out, meta_out, stream)


def cgx_layered_sizes(plan: LayeredPlan) -> Tuple[int, int]:
    """(packed_bytes, meta_bytes) of a plan with a bucket size per layer."""
    return _sizes_of(plan)


def cgx_layered_quantize(grad, plan: LayeredPlan, seed: int, packed, meta, stream=None) -> None:
    """As cgx_quantize, every layer with its own bucket size."""
    _quantize("cgx_layered_quantize", False, grad, plan, seed, packed, meta, stream)


def cgx_layered_requantize(total, plan: LayeredPlan, seed: int, packed, meta, stream=None) -> None:
    """As cgx_requantize, every layer with its own bucket size."""
    _quantize("cgx_layered_requantize", False, total, plan, seed, packed, meta, stream, requantize=True)


def cgx_layered_dequant_reduce(packed: Sequence, meta: Sequence, plan: LayeredPlan, total, stream=None) -> None:
    """As cgx_dequant_reduce, every layer with its own bucket size."""
    _reduce("cgx_layered_dequant_reduce", False, packed, meta, plan, total, stream)


def cgx_layered_dequant_reduce_requantize(packed: Sequence, meta: Sequence, plan: LayeredPlan, seed: int, packed_out,
                                          meta_out, stream=None) -> None:
    """As cgx_dequant_reduce_requantize, every layer with its own bucket size."""
    _fused("cgx_layered_dequant_reduce_requantize", False, packed, meta, plan, seed, packed_out, meta_out, stream)


def cgx_layered_dequant_reduce_add(local, local_dt: int, packed: Sequence, meta: Sequence, plan: LayeredPlan, total,
                                   stream=None) -> None:
    """As cgx_dequant_reduce_add, every layer with its own bucket size."""
    if local_dt not in (F32, F16):
        raise ValueError("cgx_layered_dequant_reduce_add: local_dt must be F32 or F16")
    _reduce("cgx_layered_dequant_reduce_add", False, packed, meta, plan, total, stream, local, local_dt)


def cgx_layered_dequantize(packed, meta, plan: LayeredPlan, out_dt: int, out, stream=None) -> None:
    """As cgx_dequantize, every layer with its own bucket size."""
    _dequantize("cgx_layered_dequantize", packed, meta, plan, out_dt, out, stream)


def cgx_layered_stats_workspace(plan: LayeredPlan) -> int:
    """Bytes of device workspace cgx_layered_layer_sqerrors needs for this plan."""
    nbytes = ctypes.c_size_t()
    _check(lib().cgx_layered_stats_workspace(*plan.args, plan.dt, ctypes.byref(nbytes)), "cgx_layered_stats_workspace")
    return int(nbytes.value)


def _sqerrors(name: str, qsgd: bool, grad, packed, meta, plan, sqerr, workspace, stream) -> None:
    pb, mb = _sizes_of(plan, qsgd)
    g = _elements(grad, f"{name}: grad", plan.n, plan.dt)
    p, m = _chunk(packed, meta, f"{name}: chunk", pb, mb)
    out = _device_buffer(sqerr, f"{name}: sqerr", 8 * plan.L, "float64")
    ws = _device_buffer(workspace, f"{name}: workspace", 0)        # its size travels with the call: the library checks it
    _check(getattr(lib(), name)(g, p, m, *plan.args, plan.dt, out, ws, workspace.numel() * workspace.element_size(),
                                _stream(stream)), name)


def cgx_layered_layer_sqerrors(grad, packed, meta, plan: LayeredPlan, sqerr, workspace, stream=None) -> None:
    """sqerr (device float64[L]) = per-layer squared l2 norm of grad - dequantize(packed, meta)."""
    _sqerrors("cgx_layered_layer_sqerrors", False, grad, packed, meta, plan, sqerr, workspace, stream)


def cgx_qsgd_layered_sizes(plan: LayeredPlan) -> Tuple[int, int]:
    return _sizes_of(plan, qsgd=True)


def cgx_qsgd_layered_quantize(grad, plan: LayeredPlan, seed: int, packed, meta, stream=None) -> None:
    _quantize("cgx_qsgd_layered_quantize", True, grad, plan, seed, packed, meta, stream)


def cgx_qsgd_layered_dequant_reduce(packed: Sequence, meta: Sequence, plan: LayeredPlan, total, stream=None) -> None:
    _reduce("cgx_qsgd_layered_dequant_reduce", True, packed, meta, plan, total, stream)


def cgx_qsgd_layered_dequant_reduce_requantize(packed: Sequence, meta: Sequence, plan: LayeredPlan, seed: int,
                                               packed_out, meta_out, stream=None) -> None:
    _fused("cgx_qsgd_layered_dequant_reduce_requantize", True, packed, meta, plan, seed, packed_out, meta_out, stream)


def cgx_qsgd_sizes(plan: Plan) -> Tuple[int, int]:
    """(packed_bytes, meta_bytes) of a plan under the norm-and-sign quantizer (one float of meta per bucket)."""
    return _sizes_of(plan, qsgd=True)


def cgx_qsgd_quantize(grad, plan: Plan, seed: int, packed, meta, stream=None) -> None:
    """As cgx_quantize, norm-and-sign codes; buffers sized by cgx_qsgd_sizes."""
    _quantize("cgx_qsgd_quantize", True, grad, plan, seed, packed, meta, stream)


def cgx_qsgd_dequant_reduce(packed: Sequence, meta: Sequence, plan: Plan, total, stream=None) -> None:
    """As cgx_dequant_reduce, for chunks written by cgx_qsgd_quantize."""
    _reduce("cgx_qsgd_dequant_reduce", True, packed, meta, plan, total, stream)


def cgx_qsgd_dequant_reduce_requantize(packed: Sequence, meta: Sequence, plan: Plan, seed: int, packed_out,
                                       meta_out, stream=None) -> None:
    """As cgx_dequant_reduce_requantize, norm-and-sign codes on both sides."""
    _fused("cgx_qsgd_dequant_reduce_requantize", True, packed, meta, plan, seed, packed_out, meta_out, stream)


def cgx_layer_stats_workspace(plan: Plan, for_sqnorms: bool = False) -> int:
    """Bytes of device workspace the per-layer statistics need for this plan."""
    nbytes = ctypes.c_size_t()
    bits = None if for_sqnorms else plan.bits.ctypes.data
    _check(lib().cgx_layer_stats_workspace(plan.n, plan.L, plan.offsets.ctypes.data, bits, plan.bucket, plan.dt,
                                           ctypes.byref(nbytes)), "cgx_layer_stats_workspace")
    return int(nbytes.value)


def cgx_layer_sqnorms(buf, plan: Plan, sqnorm, workspace, stream=None) -> None:
    """sqnorm (device float64[L]) = per-layer sums of squares of buf; workspace: device uint8 tensor."""
    b = _elements(buf, "cgx_layer_sqnorms: buf", plan.n, plan.dt)
    out = _device_buffer(sqnorm, "cgx_layer_sqnorms: sqnorm", 8 * plan.L, "float64")
    ws = _device_buffer(workspace, "cgx_layer_sqnorms: workspace", 0)   # sized check: in the library
    _check(lib().cgx_layer_sqnorms(b, plan.n, plan.L, plan.offsets.ctypes.data, plan.dt, out, ws,
                                   workspace.numel() * workspace.element_size(), _stream(stream)), "cgx_layer_sqnorms")


NOALLOC_MAX_LAYERS, NOALLOC_MAX_TILES = 4096, 262144


def cgx_layer_sqnorms_noalloc(buf, plan: Plan, sqnorm, stream=None) -> None:
    """cgx_layer_sqnorms without workspace and without device allocations (fixed tables inside the library)."""
    b = _elements(buf, "cgx_layer_sqnorms_noalloc: buf", plan.n, plan.dt)
    out = _device_buffer(sqnorm, "cgx_layer_sqnorms_noalloc: sqnorm", 8 * plan.L, "float64")
    _check(lib().cgx_layer_sqnorms_noalloc(b, plan.n, plan.L, plan.offsets.ctypes.data, plan.dt, out, _stream(stream)),
           "cgx_layer_sqnorms_noalloc")


def cgx_layer_sqerrors(grad, packed, meta, plan: Plan, sqerr, workspace, stream=None, qsgd: bool = False) -> None:
    """sqerr (device float64[L]) = per-layer squared l2 norm of grad - dequantize(packed, meta)."""
    _sqerrors("cgx_qsgd_layer_sqerrors" if qsgd else "cgx_layer_sqerrors", qsgd, grad, packed, meta, plan, sqerr,
              workspace, stream)


def _assign_inputs(layer_offsets, layer_norms, bits_in, candidates):
    off = np.ascontiguousarray(layer_offsets, dtype=np.int64)
    norms = np.ascontiguousarray(layer_norms, dtype=np.float64)
    bits = np.ascontiguousarray(bits_in, dtype=np.uint8)
    cand = np.ascontiguousarray(candidates, dtype=np.uint8)
    if off.size != bits.size + 1 or norms.size != bits.size:
        raise ValueError("one norm and one bits_in entry per layer, one more offset")
    return off, norms, bits, cand, np.zeros(bits.size, dtype=np.uint8)


def cgx_assign_bits_kmeans(layer_offsets, layer_norms, bits_in, candidates, max_iter: int = 100) -> np.ndarray:
    """bits_per_layer chosen by the k-means assigner (host arrays in, uint8[L] out)."""
    off, norms, bits, cand, out = _assign_inputs(layer_offsets, layer_norms, bits_in, candidates)
    _check(lib().cgx_assign_bits_kmeans(bits.size, off.ctypes.data, norms.ctypes.data, bits.ctypes.data,
                                        cand.ctypes.data, cand.size, max_iter, out.ctypes.data),
           "cgx_assign_bits_kmeans")
    return out


def cgx_assign_bits_linear(layer_offsets, layer_norms, bits_in, candidates) -> np.ndarray:
    """bits_per_layer chosen by the sort-and-interpolate heuristic."""
    off, norms, bits, cand, out = _assign_inputs(layer_offsets, layer_norms, bits_in, candidates)
    _check(lib().cgx_assign_bits_linear(bits.size, off.ctypes.data, norms.ctypes.data, bits.ctypes.data,
                                        cand.ctypes.data, cand.size, out.ctypes.data), "cgx_assign_bits_linear")
    return out


def cgx_assign_buckets_from_bits(bits_per_layer, width_candidates, bucket_candidates) -> np.ndarray:
    """buckets_per_layer (int32) to go with widths chosen by an assigner: fewest bits, longest buckets."""
    bits = np.ascontiguousarray(bits_per_layer, dtype=np.uint8)
    widths = np.ascontiguousarray(width_candidates, dtype=np.uint8)
    sizes = np.ascontiguousarray(bucket_candidates, dtype=np.int32)
    out = np.zeros(bits.size, dtype=np.int32)
    _check(lib().cgx_assign_buckets_from_bits(bits.size, bits.ctypes.data, widths.ctypes.data, widths.size,
                                              sizes.ctypes.data, sizes.size, out.ctypes.data),
           "cgx_assign_buckets_from_bits")
    return out


def cgx_stream_probe(src, read_bytes: int, dst, write_bytes: int, stream=None) -> None:
    """Measurement aid: one launch reading read_bytes from src and writing write_bytes to dst."""
    _check(lib().cgx_stream_probe(_device_buffer(src, "cgx_stream_probe: src", read_bytes), read_bytes,
                                  _device_buffer(dst, "cgx_stream_probe: dst", write_bytes), write_bytes,
                                  _stream(stream)), "cgx_stream_probe")


LOAD_POLICIES = ("plain", "nt", "sc1", "sc0 sc1")
STORE_POLICIES = ("plain", "nt", "sc0 sc1", "sc0 sc1 nt", "sc1")


def cgx_stream_probe_shaped(src, read_bytes: int, dst, write_bytes: int, slice_bytes: int = 8192,
                            block_threads: int = 256, loads: str = "nt", stores: str = "nt",
                            xcd_contiguous: bool = False, max_blocks: int = 0, paired_loads: bool = False,
                            alu_ops_per_pass: int = 0, lds_bytes_per_block: int = 0, stream=None) -> None:
    """The probe with its launch shape and cache policies chosen by the caller (see cgx_diag.h)."""
    shape = (ctypes.c_int32 * 9)(slice_bytes, block_threads, LOAD_POLICIES.index(loads), STORE_POLICIES.index(stores),
                                 int(xcd_contiguous), max_blocks, int(paired_loads), alu_ops_per_pass,
                                 lds_bytes_per_block)
    _check(lib().cgx_stream_probe_shaped(_device_buffer(src, "cgx_stream_probe_shaped: src", read_bytes), read_bytes,
                                         _device_buffer(dst, "cgx_stream_probe_shaped: dst", write_bytes),
                                         write_bytes, shape, _stream(stream)), "cgx_stream_probe_shaped")


def cgx_issue_probe_forms() -> list:
    """The instruction forms cgx_issue_probe knows, in order (see cgx_diag.h)."""
    forms = []
    while True:
        text = lib().cgx_issue_probe_form(len(forms))
        if text is None:
            return forms
        forms.append(text.decode())


def cgx_issue_probe(form: int, blocks: int, iterations: int, out, stream=None) -> None:
    """One launch of the issue-rate probe; out: device buffer of at least blocks * 1024 bytes."""
    nbytes = out.numel() * out.element_size()
    _check(lib().cgx_issue_probe(form, blocks, iterations, _device_buffer(out, "cgx_issue_probe: out", blocks * 1024),
                                 nbytes, _stream(stream)), "cgx_issue_probe")


def cgx_shutdown() -> None:
    _check(lib().cgx_shutdown(), "cgx_shutdown")
