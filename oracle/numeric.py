"""ctypes front end of the numeric oracle (test infrastructure, not product).

Loads ``oracle/libhzp_oracle.so`` (plain C, see ``numeric.c``; built by
``oracle.build()``) and exposes it on numpy arrays.  bf16 data travels as
``uint16`` bit patterns.  Only tests, the smoke check and the benchmark's
CPU-baseline leg may import this module; it imports nothing of the GPU path.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# HZP_ORACLE_LIBRARY names another build of numeric.c (the sanitizer build of the tests); it is loaded as it is
_SO = os.environ.get("HZP_ORACLE_LIBRARY") or os.path.join(_HERE, "libhzp_oracle.so")
_SRC = os.path.join(_HERE, "numeric.c")
_lib = None


def build(force=True):
    """Compile numeric.c with gcc (contraction and fast-math off)."""
    if not force and os.path.exists(_SO) and os.path.getmtime(_SO) >= os.path.getmtime(_SRC):
        return _SO
    cmd = ["gcc", "-O2", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-fPIC",
           "-shared", "-o", _SO, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _SO


class _Hyper(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("step", ctypes.c_uint32)]


def lib():
    global _lib
    if _lib is None:
        if not os.environ.get("HZP_ORACLE_LIBRARY"):
            build(force=False)
        L = ctypes.CDLL(_SO)
        L.hzp_oracle_threads.restype = ctypes.c_int
        L.hzp_oracle_bf16_to_f32.restype = ctypes.c_float
        L.hzp_oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        L.hzp_oracle_f32_to_bf16.restype = ctypes.c_uint16
        L.hzp_oracle_f32_to_bf16.argtypes = [ctypes.c_float]
        vp, u32, u64 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64
        L.hzp_oracle_f32_to_bf16_array.restype = None
        L.hzp_oracle_f32_to_bf16_array.argtypes = [vp, u64, vp]
        L.hzp_oracle_reduce.restype = None
        L.hzp_oracle_reduce.argtypes = [vp, u32, ctypes.c_int, u64, ctypes.c_float,
                                        ctypes.c_int, vp]
        for f in (L.hzp_oracle_adamw_f64, L.hzp_oracle_adamw_f32):
            f.restype = None
            f.argtypes = [ctypes.POINTER(_Hyper), u64, vp, vp, vp, vp, vp, vp, vp]
        L.hzp_oracle_gather_concat.restype = None
        L.hzp_oracle_gather_concat.argtypes = [vp, u32, u64, u32, vp]
        L.hzp_oracle_unpack_tensor.restype = None
        L.hzp_oracle_unpack_tensor.argtypes = [vp, u64, u32, u64, u64, vp]
        _lib = L
    return _lib


def threads():
    return int(lib().hzp_oracle_threads())


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def _ptr_array(arrays):
    arr = (ctypes.c_void_p * len(arrays))(*[a.ctypes.data for a in arrays])
    return arr


def _check(a, dtype):
    if a.dtype != dtype or not a.flags["C_CONTIGUOUS"] or a.ndim != 1:
        raise TypeError("expected a contiguous 1-D %s array" % np.dtype(dtype).name)


def bf16_to_f32(h):
    """Widen uint16 bf16 patterns (scalar or array) to float32, element by element."""
    L = lib()
    h = np.asarray(h, dtype=np.uint16)
    out = np.empty(h.shape, dtype=np.float32)
    flat_in, flat_out = h.reshape(-1), out.reshape(-1)
    for i in range(flat_in.size):
        flat_out[i] = L.hzp_oracle_bf16_to_f32(int(flat_in[i]))
    return out


def f32_to_bf16(f):
    """Narrow float32 (scalar or array) to uint16 bf16 patterns, element by element."""
    L = lib()
    f = np.asarray(f, dtype=np.float32)
    out = np.empty(f.shape, dtype=np.uint16)
    flat_in, flat_out = f.reshape(-1), out.reshape(-1)
    for i in range(flat_in.size):
        flat_out[i] = L.hzp_oracle_f32_to_bf16(ctypes.c_float(flat_in[i]))
    return out


def f32_to_bf16_array(f):
    """The same narrowing over a contiguous float32 array in one call (a loop over the scalar cast)."""
    _check(f, np.float32)
    out = np.empty(f.size, dtype=np.uint16)
    lib().hzp_oracle_f32_to_bf16_array(_ptr(f), f.size, _ptr(out))
    return out


def reduce(slices, scale=1.0, accumulate=False, out=None):
    """Fixed-order fp32 sum of the R slices (uint16 bf16 patterns or float32)."""
    R = len(slices)
    is_f32 = slices[0].dtype == np.float32
    n = slices[0].size
    for s in slices:
        _check(s, np.float32 if is_f32 else np.uint16)
        if s.size != n:
            raise ValueError("slices differ in length")
    if out is None:
        if accumulate:
            raise ValueError("accumulate needs an existing output")
        out = np.empty(n, dtype=np.float32)
    _check(out, np.float32)
    pa = _ptr_array(slices)
    lib().hzp_oracle_reduce(pa, R, int(is_f32), n, ctypes.c_float(scale), int(accumulate),
                            _ptr(out))
    return out


def adamw(g, p, m, v, lr, beta1, beta2, eps, weight_decay, step, wd_mult=None,
          out_bf16=True, precision="f64"):
    """One AdamW step in place on p, m, v (float32).  Returns the cast/copied parameters."""
    for a in (g, p, m, v):
        _check(a, np.float32)
    n = g.size
    if wd_mult is not None:
        _check(wd_mult, np.float32)
    h = _Hyper(lr, beta1, beta2, eps, weight_decay, step)
    p16 = np.empty(n, dtype=np.uint16) if out_bf16 else None
    p32 = None if out_bf16 else np.empty(n, dtype=np.float32)
    fn = lib().hzp_oracle_adamw_f64 if precision == "f64" else lib().hzp_oracle_adamw_f32
    fn(ctypes.byref(h), n, _ptr(g), _ptr(wd_mult) if wd_mult is not None else None,
       _ptr(p), _ptr(m), _ptr(v),
       _ptr(p16) if p16 is not None else None, _ptr(p32) if p32 is not None else None)
    return p16 if out_bf16 else p32


def gather_concat(srcs):
    """dst[s*len + x] = src_s[x] for equal-length pieces (any 2- or 4-byte dtype)."""
    n = srcs[0].size
    dt = srcs[0].dtype
    for s in srcs:
        _check(s, dt)
        if s.size != n:
            raise ValueError("pieces differ in length")
    dst = np.empty(n * len(srcs), dtype=dt)
    lib().hzp_oracle_gather_concat(_ptr_array(srcs), len(srcs), n, dt.itemsize, _ptr(dst))
    return dst


def gather_shard(zero1_pieces, j, z3):
    """ZeRO-3 shard j of the bucket whose ZeRO-1 shards are `zero1_pieces` (all Z1 of them, in shard
    order): the bucket is their concatenation and shard j is its j-th of z3 equal parts.  This is the
    post-step parameter gather (Section 4.1.2, "Optimizer Step") for group sizes that need not nest."""
    bucket = gather_concat(zero1_pieces)
    if bucket.size % z3:
        raise ValueError("bucket length is not a multiple of Z3")
    S3 = bucket.size // z3
    return bucket[j * S3:(j + 1) * S3].copy()


def unpack_tensor(shards, offset, numel):
    """Copy tensor elements [offset, offset+numel) of the bucket out of its Z3 shards."""
    dt = shards[0].dtype
    S3 = shards[0].size
    for s in shards:
        _check(s, dt)
        if s.size != S3:
            raise ValueError("shards differ in length")
    if offset + numel > S3 * len(shards):
        raise ValueError("tensor exceeds the bucket")
    dst = np.empty(numel, dtype=dt)
    lib().hzp_oracle_unpack_tensor(_ptr_array(shards), S3, dt.itemsize, offset, numel, _ptr(dst))
    return dst
