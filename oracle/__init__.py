"""ctypes front end of the plain CPU oracle (``cgx_oracle.c``).

TEST INFRASTRUCTURE: only the tests, the smoke check and the benchmark's
``cpu_baseline`` leg import this package.  It holds no GPU code and imports
nothing from the GPU library.

All arrays are numpy arrays on the host.  ``dt`` is 0 for binary32 storage and
1 for binary16 storage of the gradient.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cgx_oracle.c")
_LIB = os.path.join(_HERE, "libcgx_oracle.so")

F32, F16 = 0, 1

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  Contraction and fast-math stay off so that
    every binary32 operation is the IEEE one the comments state."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c = ctypes
        lib.oracle_rng32.restype = c.c_uint32
        lib.oracle_rng32.argtypes = [c.c_uint64, c.c_uint64]
        lib.oracle_u16.restype = c.c_uint32
        lib.oracle_u16.argtypes = [c.c_uint64, c.c_uint64]
        lib.oracle_fill_u16.restype = None
        lib.oracle_fill_u16.argtypes = [c.c_uint64, c.c_uint64, c.c_int64, c.c_void_p]
        plan = [c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_int32]
        lib.oracle_sizes.argtypes = plan + [c.c_int32, c.POINTER(c.c_uint64), c.POINTER(c.c_uint64)]
        lib.oracle_quantize.argtypes = [c.c_void_p] + plan + [c.c_uint64, c.c_int32, c.c_void_p, c.c_void_p]
        lib.oracle_quantize_window.argtypes = [c.c_void_p] + plan + [c.c_uint64, c.c_int32, c.c_uint64, c.c_void_p, c.c_void_p]
        lib.oracle_quantize_with_draws.argtypes = [c.c_void_p] + plan + [c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p]
        lib.oracle_dequant_reduce.argtypes = [c.c_void_p, c.c_void_p, c.c_int32] + plan + \
            [c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p]
        lib.oracle_dequant_reduce_add.argtypes = [c.c_void_p, c.c_int32, c.c_void_p, c.c_void_p, c.c_int32] + plan + \
            [c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p]
        lib.oracle_float_to_half.restype = None
        lib.oracle_float_to_half.argtypes = [c.c_void_p, c.c_int64, c.c_void_p]
        lib.oracle_qsgd_sizes.argtypes = plan + [c.c_int32, c.POINTER(c.c_uint64), c.POINTER(c.c_uint64)]
        lib.oracle_qsgd_quantize.argtypes = [c.c_void_p] + plan + [c.c_uint64, c.c_int32, c.c_void_p, c.c_void_p]
        lib.oracle_qsgd_quantize_with_draws.argtypes = [c.c_void_p] + plan + [c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p]
        lib.oracle_qsgd_dequant_reduce.argtypes = [c.c_void_p, c.c_void_p, c.c_int32] + plan + \
            [c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p]
        lib.oracle_layer_sqnorms.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_void_p, c.c_int32, c.c_void_p]
        lib.oracle_layer_sqerrors.argtypes = [c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p] + plan + \
            [c.c_int32, c.c_void_p]
        lib.oracle_unpack_codes.argtypes = [c.c_void_p] + plan + [c.c_int32, c.c_void_p]
        layered = [c.c_int64, c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p]
        lib.oracle_layered_sizes.argtypes = layered + [c.c_int32, c.POINTER(c.c_uint64), c.POINTER(c.c_uint64)]
        lib.oracle_layered_quantize.argtypes = [c.c_void_p] + layered + [c.c_uint64, c.c_int32, c.c_void_p, c.c_void_p]
        lib.oracle_layered_dequant_reduce.argtypes = [c.c_void_p, c.c_void_p, c.c_int32] + layered + \
            [c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p]
        lib.oracle_layered_dequant_reduce_add.argtypes = [c.c_void_p, c.c_int32, c.c_void_p, c.c_void_p, c.c_int32] + \
            layered + [c.c_int32, c.c_void_p, c.c_void_p, c.c_void_p]
        lib.oracle_qsgd_quantize_window.argtypes = [c.c_void_p] + plan + [c.c_uint64, c.c_int32, c.c_uint64, c.c_void_p,
                                                                          c.c_void_p]
        lib.oracle_qsgd_layered_sizes.argtypes = lib.oracle_layered_sizes.argtypes
        lib.oracle_qsgd_layered_quantize.argtypes = lib.oracle_layered_quantize.argtypes
        lib.oracle_qsgd_layered_dequant_reduce.argtypes = lib.oracle_layered_dequant_reduce.argtypes
        lib.oracle_layered_layer_sqerrors.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p] + layered + [c.c_int32, c.c_void_p]
        _lib = lib
    return _lib


def set_threads(k: int) -> None:
    """Number of OpenMP threads the oracle's bucket loops use (1 = sequential)."""
    omp = ctypes.CDLL("libgomp.so.1")
    omp.omp_set_num_threads(int(k))


def get_max_threads() -> int:
    omp = ctypes.CDLL("libgomp.so.1")
    return int(omp.omp_get_max_threads())


def _plan(offsets, bits):
    off = np.ascontiguousarray(offsets, dtype=np.int64)
    bt = np.ascontiguousarray(bits, dtype=np.uint8)
    if off.ndim != 1 or bt.ndim != 1 or off.size != bt.size + 1:
        raise ValueError("layer_offsets must have one more entry than bits_per_layer")
    return off, bt, int(off[-1]), int(bt.size)


def _ptr(a):
    return a.ctypes.data if a is not None else None


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"{what}: oracle rejected the arguments (rc={rc})")


def rng32(seed: int, pair: int) -> int:
    return int(_load().oracle_rng32(seed & (2**64 - 1), pair & (2**64 - 1)))


def u16(seed: int, i: int) -> int:
    return int(_load().oracle_u16(seed & (2**64 - 1), i & (2**64 - 1)))


def draws(seed: int, i0: int, count: int) -> np.ndarray:
    """The 16-bit draws of elements i0 .. i0+count-1."""
    out = np.zeros(count, dtype=np.uint16)
    _load().oracle_fill_u16(seed & (2**64 - 1), i0 & (2**64 - 1), count, _ptr(out))
    return out


def sizes(offsets, bits, bucket: int, dt: int = F32):
    """(packed_bytes, meta_bytes) of a plan."""
    off, bt, n, L = _plan(offsets, bits)
    pb, mb = ctypes.c_uint64(), ctypes.c_uint64()
    _check(_load().oracle_sizes(n, L, _ptr(off), _ptr(bt), bucket, dt, ctypes.byref(pb), ctypes.byref(mb)), "sizes")
    return int(pb.value), int(mb.value)


def _grad(grad, n, dt):
    want = np.float16 if dt == F16 else np.float32
    g = np.ascontiguousarray(grad)
    if g.dtype != want or g.size != n:
        raise ValueError(f"gradient must be {want.__name__} with {n} elements")
    return g


def quantize(grad, offsets, bits, bucket: int, seed: int, dt: int = F32, draws=None, index_base: int = 0):
    """Returns (packed uint8[packed_bytes], meta float32[n_buckets, 2] = (unit, mn)).
    index_base: position of grad[0] in the whole buffer when grad is a window of it."""
    off, bt, n, L = _plan(offsets, bits)
    g = _grad(grad, n, dt)
    pb, mb = sizes(off, bt, bucket, dt)
    packed = np.zeros(pb, dtype=np.uint8)
    meta = np.zeros((mb // 8, 2), dtype=np.float32)
    lib = _load()
    if draws is None:
        rc = lib.oracle_quantize_window(_ptr(g), n, L, _ptr(off), _ptr(bt), bucket, seed & (2**64 - 1), dt,
                                        index_base, _ptr(packed), _ptr(meta))
    else:
        d = np.ascontiguousarray(draws, dtype=np.uint16)
        if d.size != n:
            raise ValueError("one draw per element")
        rc = lib.oracle_quantize_with_draws(_ptr(g), n, L, _ptr(off), _ptr(bt), bucket, dt, _ptr(d),
                                            _ptr(packed), _ptr(meta))
    _check(rc, "quantize")
    return packed, meta


def float_to_half(x) -> np.ndarray:
    """binary32 -> binary16 (as uint16 bit patterns), round to nearest even."""
    a = np.ascontiguousarray(x, dtype=np.float32)
    out = np.zeros(a.size, dtype=np.uint16)
    _load().oracle_float_to_half(_ptr(a), a.size, _ptr(out))
    return out.reshape(a.shape)


def dequantize(packed, meta, offsets, bits, bucket: int, dt: int = F32, out_dt: int = F32) -> np.ndarray:
    """One chunk decompressed into binary32, or into binary16 (rounded to nearest even)."""
    d = dequant_reduce([packed], [meta], offsets, bits, bucket, dt, want=("sum32",))["sum32"]
    return float_to_half(d).view(np.float16) if out_dt == F16 else d


def dequant_reduce(packed_list, meta_list, offsets, bits, bucket: int, dt: int = F32,
                   want=("sum32", "sum64", "abs64"), local=None):
    """Returns a dict with the requested arrays (see cgx_oracle.c).  `local` (float32 or
    float16 array of n elements) is the rank's own uncompressed term, added first."""
    off, bt, n, L = _plan(offsets, bits)
    W = len(packed_list)
    if W < 1 or len(meta_list) != W:
        raise ValueError("need W >= 1 packed chunks and as many meta arrays")
    pb, mb = sizes(off, bt, bucket, dt)
    pk = [np.ascontiguousarray(p, dtype=np.uint8) for p in packed_list]
    mt = [np.ascontiguousarray(m, dtype=np.float32) for m in meta_list]
    for p, m in zip(pk, mt):
        if p.size != pb or m.size * 4 != mb:
            raise ValueError("chunk sizes do not match the plan")
    pp = (ctypes.c_void_p * W)(*[p.ctypes.data for p in pk])
    mp = (ctypes.c_void_p * W)(*[m.ctypes.data for m in mt])
    out = {
        "sum32": np.zeros(n, dtype=np.float32) if "sum32" in want else None,
        "sum64": np.zeros(n, dtype=np.float64) if "sum64" in want else None,
        "abs64": np.zeros(n, dtype=np.float64) if "abs64" in want else None,
    }
    loc, loc_dt = None, F32
    if local is not None:
        loc = np.ascontiguousarray(local)
        if loc.dtype not in (np.float32, np.float16) or loc.size != n:
            raise ValueError("local must be float32 or float16 with n elements")
        loc_dt = F16 if loc.dtype == np.float16 else F32
    rc = _load().oracle_dequant_reduce_add(_ptr(loc), loc_dt, pp, mp, W, n, L, _ptr(off), _ptr(bt), bucket, dt,
                                           _ptr(out["sum32"]), _ptr(out["sum64"]), _ptr(out["abs64"]))
    _check(rc, "dequant_reduce")
    return {k: v for k, v in out.items() if v is not None}


def unpack_codes(packed, offsets, bits, bucket: int, dt: int = F32):
    """One byte per element: its code, or 0xff in pass-through layers."""
    off, bt, n, L = _plan(offsets, bits)
    p = np.ascontiguousarray(packed, dtype=np.uint8)
    codes = np.zeros(n, dtype=np.uint8)
    _check(_load().oracle_unpack_codes(_ptr(p), n, L, _ptr(off), _ptr(bt), bucket, dt, _ptr(codes)), "unpack_codes")
    return codes


# ---- a bucket size per layer

def _layer_buckets(buckets, L):
    bk = np.ascontiguousarray(buckets, dtype=np.int32)
    if bk.ndim != 1 or bk.size != L:
        raise ValueError("one bucket size per layer")
    return bk


def layered_sizes(offsets, bits, buckets, dt: int = F32):
    """(packed_bytes, meta_bytes) of a plan whose layer l has bucket size buckets[l]."""
    off, bt, n, L = _plan(offsets, bits)
    bk = _layer_buckets(buckets, L)
    pb, mb = ctypes.c_uint64(), ctypes.c_uint64()
    _check(_load().oracle_layered_sizes(n, L, _ptr(off), _ptr(bt), _ptr(bk), dt, ctypes.byref(pb), ctypes.byref(mb)),
           "layered_sizes")
    return int(pb.value), int(mb.value)


def layered_quantize(grad, offsets, bits, buckets, seed: int, dt: int = F32):
    """quantize() with a bucket size per layer."""
    off, bt, n, L = _plan(offsets, bits)
    bk = _layer_buckets(buckets, L)
    g = _grad(grad, n, dt)
    pb, mb = layered_sizes(off, bt, bk, dt)
    packed = np.zeros(pb, dtype=np.uint8)
    meta = np.zeros((mb // 8, 2), dtype=np.float32)
    _check(_load().oracle_layered_quantize(_ptr(g), n, L, _ptr(off), _ptr(bt), _ptr(bk), seed & (2**64 - 1), dt,
                                           _ptr(packed), _ptr(meta)), "layered_quantize")
    return packed, meta


def layered_dequant_reduce(packed_list, meta_list, offsets, bits, buckets, dt: int = F32, local=None):
    """dequant_reduce() with a bucket size per layer; returns sum32, sum64 and abs64.  `local`
    (float32 or float16 array of n elements) is the rank's own uncompressed term, added first."""
    off, bt, n, L = _plan(offsets, bits)
    bk = _layer_buckets(buckets, L)
    W = len(packed_list)
    if W < 1 or len(meta_list) != W:
        raise ValueError("need W >= 1 packed chunks and as many meta arrays")
    pb, mb = layered_sizes(off, bt, bk, dt)
    pk = [np.ascontiguousarray(p, dtype=np.uint8) for p in packed_list]
    mt = [np.ascontiguousarray(m, dtype=np.float32) for m in meta_list]
    for p, m in zip(pk, mt):
        if p.size != pb or m.size * 4 != mb:
            raise ValueError("chunk sizes do not match the plan")
    pp = (ctypes.c_void_p * W)(*[p.ctypes.data for p in pk])
    mp = (ctypes.c_void_p * W)(*[m.ctypes.data for m in mt])
    out = {"sum32": np.zeros(n, dtype=np.float32), "sum64": np.zeros(n, dtype=np.float64),
           "abs64": np.zeros(n, dtype=np.float64)}
    loc, loc_dt = None, F32
    if local is not None:
        loc = np.ascontiguousarray(local)
        if loc.dtype not in (np.float32, np.float16) or loc.size != n:
            raise ValueError("local must be float32 or float16 with n elements")
        loc_dt = F16 if loc.dtype == np.float16 else F32
    _check(_load().oracle_layered_dequant_reduce_add(_ptr(loc), loc_dt, pp, mp, W, n, L, _ptr(off), _ptr(bt), _ptr(bk),
                                                     dt, _ptr(out["sum32"]), _ptr(out["sum64"]), _ptr(out["abs64"])),
           "layered_dequant_reduce")
    return out


def layered_layer_sqerrors(grad, packed, meta, offsets, bits, buckets, dt: int = F32):
    """layer_sqerrors() for a chunk written with a bucket size per layer (min/max form)."""
    off, bt, n, L = _plan(offsets, bits)
    bk = _layer_buckets(buckets, L)
    g = _grad(grad, n, dt)
    pk = np.ascontiguousarray(packed, dtype=np.uint8)
    mt = np.ascontiguousarray(meta, dtype=np.float32).reshape(-1)
    pb, mb = layered_sizes(off, bt, bk, dt)
    if pk.size != pb or mt.size * 4 != mb:
        raise ValueError("chunk sizes do not match the plan")
    out = np.zeros(L, dtype=np.float64)
    _check(_load().oracle_layered_layer_sqerrors(_ptr(g), _ptr(pk), _ptr(mt), n, L, _ptr(off), _ptr(bt), _ptr(bk), dt,
                                                 _ptr(out)), "layered_layer_sqerrors")
    return out


# ---- the norm-and-sign form (see the second half of cgx_oracle.c)

def qsgd_sizes(offsets, bits, bucket: int, dt: int = F32):
    off, bt, n, L = _plan(offsets, bits)
    pb, mb = ctypes.c_uint64(), ctypes.c_uint64()
    _check(_load().oracle_qsgd_sizes(n, L, _ptr(off), _ptr(bt), bucket, dt, ctypes.byref(pb), ctypes.byref(mb)),
           "qsgd_sizes")
    return int(pb.value), int(mb.value)


def qsgd_quantize(grad, offsets, bits, bucket: int, seed: int, dt: int = F32, draws=None, index_base: int = 0):
    """Returns (packed uint8[packed_bytes], meta float32[n_buckets] = unit).
    index_base: position of grad[0] in the whole buffer when grad is a window of it."""
    off, bt, n, L = _plan(offsets, bits)
    g = _grad(grad, n, dt)
    pb, mb = qsgd_sizes(off, bt, bucket, dt)
    packed = np.zeros(pb, dtype=np.uint8)
    meta = np.zeros(mb // 4, dtype=np.float32)
    lib = _load()
    if draws is None:
        rc = lib.oracle_qsgd_quantize_window(_ptr(g), n, L, _ptr(off), _ptr(bt), bucket, seed & (2**64 - 1), dt,
                                             index_base, _ptr(packed), _ptr(meta))
    else:
        d = np.ascontiguousarray(draws, dtype=np.uint16)
        if d.size != n:
            raise ValueError("one draw per element")
        rc = lib.oracle_qsgd_quantize_with_draws(_ptr(g), n, L, _ptr(off), _ptr(bt), bucket, dt, _ptr(d),
                                                 _ptr(packed), _ptr(meta))
    _check(rc, "qsgd_quantize")
    return packed, meta


def qsgd_dequant_reduce(packed_list, meta_list, offsets, bits, bucket: int, dt: int = F32,
                        want=("sum32", "sum64", "abs64")):
    off, bt, n, L = _plan(offsets, bits)
    W = len(packed_list)
    if W < 1 or len(meta_list) != W:
        raise ValueError("need W >= 1 packed chunks and as many meta arrays")
    pb, mb = qsgd_sizes(off, bt, bucket, dt)
    pk = [np.ascontiguousarray(p, dtype=np.uint8) for p in packed_list]
    mt = [np.ascontiguousarray(m, dtype=np.float32) for m in meta_list]
    for p, m in zip(pk, mt):
        if p.size != pb or m.size * 4 != mb:
            raise ValueError("chunk sizes do not match the plan")
    pp = (ctypes.c_void_p * W)(*[p.ctypes.data for p in pk])
    mp = (ctypes.c_void_p * W)(*[m.ctypes.data for m in mt])
    out = {
        "sum32": np.zeros(n, dtype=np.float32) if "sum32" in want else None,
        "sum64": np.zeros(n, dtype=np.float64) if "sum64" in want else None,
        "abs64": np.zeros(n, dtype=np.float64) if "abs64" in want else None,
    }
    rc = _load().oracle_qsgd_dequant_reduce(pp, mp, W, n, L, _ptr(off), _ptr(bt), bucket, dt,
                                            _ptr(out["sum32"]), _ptr(out["sum64"]), _ptr(out["abs64"]))
    _check(rc, "qsgd_dequant_reduce")
    return {k: v for k, v in out.items() if v is not None}


# ---- per-layer statistics for the adaptive scheme

def layer_sqnorms(buf, offsets, dt: int = F32):
    """float64[L]: sum of squares of every layer of the buffer."""
    off = np.ascontiguousarray(offsets, dtype=np.int64)
    n, L = int(off[-1]), off.size - 1
    g = _grad(buf, n, dt)
    out = np.zeros(L, dtype=np.float64)
    _check(_load().oracle_layer_sqnorms(_ptr(g), n, L, _ptr(off), dt, _ptr(out)), "layer_sqnorms")
    return out


def layer_sqerrors(grad, packed, meta, offsets, bits, bucket: int, dt: int = F32, scheme: int = 0):
    """float64[L]: squared l2 norm of grad - dequantize(packed, meta) per layer
    (scheme 0: min/max form, 1: norm-and-sign form)."""
    off, bt, n, L = _plan(offsets, bits)
    g = _grad(grad, n, dt)
    pk = np.ascontiguousarray(packed, dtype=np.uint8)
    mt = np.ascontiguousarray(meta, dtype=np.float32).reshape(-1)
    pb, mb = (qsgd_sizes if scheme == 1 else sizes)(off, bt, bucket, dt)
    if pk.size != pb or mt.size * 4 != mb:
        raise ValueError("chunk sizes do not match the plan")
    out = np.zeros(L, dtype=np.float64)
    _check(_load().oracle_layer_sqerrors(scheme, _ptr(g), _ptr(pk), _ptr(mt), n, L, _ptr(off), _ptr(bt), bucket, dt,
                                         _ptr(out)), "layer_sqerrors")
    return out


# ---- the norm-and-sign form with a bucket size per layer

def qsgd_layered_sizes(offsets, bits, buckets, dt: int = F32):
    off, bt, n, L = _plan(offsets, bits)
    bk = _layer_buckets(buckets, L)
    pb, mb = ctypes.c_uint64(), ctypes.c_uint64()
    _check(_load().oracle_qsgd_layered_sizes(n, L, _ptr(off), _ptr(bt), _ptr(bk), dt, ctypes.byref(pb),
                                             ctypes.byref(mb)), "qsgd_layered_sizes")
    return int(pb.value), int(mb.value)


def qsgd_layered_quantize(grad, offsets, bits, buckets, seed: int, dt: int = F32):
    off, bt, n, L = _plan(offsets, bits)
    bk = _layer_buckets(buckets, L)
    g = _grad(grad, n, dt)
    pb, mb = qsgd_layered_sizes(off, bt, bk, dt)
    packed = np.zeros(pb, dtype=np.uint8)
    meta = np.zeros(mb // 4, dtype=np.float32)
    _check(_load().oracle_qsgd_layered_quantize(_ptr(g), n, L, _ptr(off), _ptr(bt), _ptr(bk), seed & (2**64 - 1), dt,
                                                _ptr(packed), _ptr(meta)), "qsgd_layered_quantize")
    return packed, meta


def qsgd_layered_dequant_reduce(packed_list, meta_list, offsets, bits, buckets, dt: int = F32):
    off, bt, n, L = _plan(offsets, bits)
    bk = _layer_buckets(buckets, L)
    W = len(packed_list)
    if W < 1 or len(meta_list) != W:
        raise ValueError("need W >= 1 packed chunks and as many meta arrays")
    pb, mb = qsgd_layered_sizes(off, bt, bk, dt)
    pk = [np.ascontiguousarray(p, dtype=np.uint8) for p in packed_list]
    mt = [np.ascontiguousarray(m, dtype=np.float32) for m in meta_list]
    for p, m in zip(pk, mt):
        if p.size != pb or m.size * 4 != mb:
            raise ValueError("chunk sizes do not match the plan")
    pp = (ctypes.c_void_p * W)(*[p.ctypes.data for p in pk])
    mp = (ctypes.c_void_p * W)(*[m.ctypes.data for m in mt])
    out = {"sum32": np.zeros(n, dtype=np.float32), "sum64": np.zeros(n, dtype=np.float64),
           "abs64": np.zeros(n, dtype=np.float64)}
    _check(_load().oracle_qsgd_layered_dequant_reduce(pp, mp, W, n, L, _ptr(off), _ptr(bt), _ptr(bk), dt,
                                                      _ptr(out["sum32"]), _ptr(out["sum64"]), _ptr(out["abs64"])),
           "qsgd_layered_dequant_reduce")
    return out
