"""ctypes view of the reference CPU codec (oracle/zcref.cpp).

Test infrastructure only: tests, the smoke check and the benchmark's CPU-baseline leg use
it; the product never does.  All buffers are numpy arrays on the host.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

OK, ERR_ARG, ERR_CAPACITY, ERR_FORMAT, ERR_NONFINITE, ERR_RANGE, ERR_BOUND, ERR_MISMATCH = range(8)

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.zcref_compress_bound.restype = C.c_size_t
        L.zcref_compress_bound.argtypes = [C.c_size_t]
        L.zcref_quantize.argtypes = [C.c_void_p, C.c_size_t, C.c_float, C.c_void_p]
        L.zcref_encode_codes.argtypes = [C.c_void_p, C.c_size_t, C.c_float, C.c_uint32, C.c_void_p,
                                         C.c_size_t, C.POINTER(C.c_size_t)]
        L.zcref_compress.argtypes = [C.c_void_p, C.c_size_t, C.c_float, C.c_void_p, C.c_size_t,
                                     C.POINTER(C.c_size_t)]
        L.zcref_decompress.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t,
                                       C.POINTER(C.c_size_t)]
        L.zcref_inspect.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p]
        L.zcref_quality.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.zcref_decompress_average.argtypes = L.zcref_decompress.argtypes
        L.zcref_decompress_range.argtypes = [C.c_void_p, C.c_size_t, C.c_size_t, C.c_size_t, C.c_void_p, C.c_size_t,
                                             C.POINTER(C.c_size_t)]
        L.zcref_reduce_step_op.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p, C.c_size_t,
                                           C.POINTER(C.c_size_t)]
        L.zcref_reduce_step.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t,
                                        C.POINTER(C.c_size_t)]
        L.zcref_reduce.argtypes = [C.POINTER(C.c_void_p), C.POINTER(C.c_size_t), C.c_int, C.c_void_p,
                                   C.c_size_t, C.POINTER(C.c_size_t)]
        L.zcref_reduce_op.argtypes = [C.POINTER(C.c_void_p), C.POINTER(C.c_size_t), C.c_int, C.c_int, C.c_void_p,
                                      C.c_size_t, C.POINTER(C.c_size_t)]
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def set_indexed(on):
    """Chooses the stream variant that is written and accepted: False plain, True indexed."""
    lib().zcref_set_indexed(1 if on else 0)


def compress_bound(n):
    return int(lib().zcref_compress_bound(n))


def quantize(x, abs_eb):
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.empty(x.size, dtype=np.int32)
    st = lib().zcref_quantize(_ptr(x), x.size, np.float32(abs_eb), _ptr(q))
    return st, q


def encode_codes(q, abs_eb, nsum=1, out_cap=None):
    q = np.ascontiguousarray(q, dtype=np.int32)
    cap = compress_bound(q.size) if out_cap is None else out_cap
    out = np.zeros(max(cap, 1), dtype=np.uint8)
    nbytes = C.c_size_t(0)
    st = lib().zcref_encode_codes(_ptr(q), q.size, np.float32(abs_eb), nsum, _ptr(out), cap, C.byref(nbytes))
    return st, out[: min(nbytes.value, cap)].copy() if st == OK else out[:0], nbytes.value


def compress(x, abs_eb, out_cap=None):
    """Returns (status, stream bytes as uint8 array, total_bytes reported)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    cap = compress_bound(x.size) if out_cap is None else out_cap
    out = np.zeros(max(cap, 1), dtype=np.uint8)
    nbytes = C.c_size_t(0)
    st = lib().zcref_compress(_ptr(x), x.size, np.float32(abs_eb), _ptr(out), cap, C.byref(nbytes))
    stream = out[: nbytes.value].copy() if st in (OK, ERR_BOUND) else out[:0]
    return st, stream, nbytes.value


def decompress(stream, out_cap_elems=None, average=False):
    """Returns (status, float32 array of n values, n reported).  average: the values divided by the stream's nsum."""
    stream = np.ascontiguousarray(stream, dtype=np.uint8)
    n = C.c_size_t(0)
    fn = lib().zcref_decompress_average if average else lib().zcref_decompress
    if out_cap_elems is None:
        st = fn(_ptr(stream), stream.size, None, 0, C.byref(n))
        if st not in (OK, ERR_CAPACITY):
            return st, np.empty(0, np.float32), 0
        out_cap_elems = n.value
    out = np.empty(max(out_cap_elems, 1), dtype=np.float32)
    st = fn(_ptr(stream), stream.size, _ptr(out), out_cap_elems, C.byref(n))
    return st, (out[: n.value].copy() if st == OK else out[:0]), n.value


def decompress_range(stream, first_value, count, out_cap_elems=None):
    """Values [first_value, first_value + count) of the stream.  Returns (status, float32 array, n reported)."""
    stream = np.ascontiguousarray(stream, dtype=np.uint8)
    n = C.c_size_t(0)
    cap = count if out_cap_elems is None else out_cap_elems
    out = np.empty(max(cap, 1), dtype=np.float32)
    st = lib().zcref_decompress_range(_ptr(stream), stream.size, int(first_value), int(count), _ptr(out), cap, C.byref(n))
    return st, (out[: n.value].copy() if st == OK else out[:0]), n.value


def inspect(stream):
    """Returns (status, codes int32[n], widths uint8[nb], payload byte offsets uint64[nb])."""
    stream = np.ascontiguousarray(stream, dtype=np.uint8)
    if stream.size < 32:
        return ERR_FORMAT, None, None, None
    n = int(stream[8:16].view("<u8")[0])
    if n > 2**31:
        return ERR_FORMAT, None, None, None
    nb = (n + 31) // 32
    q = np.empty(max(n, 1), np.int32)
    w = np.empty(max(nb, 1), np.uint8)
    off = np.empty(max(nb, 1), np.uint64)
    st = lib().zcref_inspect(_ptr(stream), stream.size, _ptr(q), _ptr(w), _ptr(off))
    if st != OK:
        return st, None, None, None
    return st, q[:n], w[:nb], off[:nb]


def reduce(streams, out_cap=None, op=0):
    """k streams -> the stream of their sum (op 0), elementwise maximum (1) or minimum (2) on the common grid.
    Returns (status, stream bytes, total_bytes reported)."""
    streams = [np.ascontiguousarray(s, dtype=np.uint8) for s in streams]
    k = len(streams)
    ptrs = (C.c_void_p * max(k, 1))(*[s.ctypes.data for s in streams])
    sizes = (C.c_size_t * max(k, 1))(*[s.size for s in streams])
    if out_cap is None:
        n = int(streams[0][8:16].view("<u8")[0]) if k and streams[0].size >= 32 else 0
        out_cap = compress_bound(min(n, 2**31))
    out = np.zeros(max(out_cap, 1), dtype=np.uint8)
    nbytes = C.c_size_t(0)
    if op == 0:
        st = lib().zcref_reduce(ptrs, sizes, k, _ptr(out), out_cap, C.byref(nbytes))
    else:
        st = lib().zcref_reduce_op(ptrs, sizes, k, int(op), _ptr(out), out_cap, C.byref(nbytes))
    return st, (out[: nbytes.value].copy() if st == OK else out[:0]), nbytes.value


OP_SUM, OP_MAX, OP_MIN = 0, 1, 2


def reduce_step(stream, local, out_cap=None, op=OP_SUM):
    """One ring round: decompress `stream`, combine with `local` (binary32 sum, max or min), compress again.
    Returns (status, stream bytes, total_bytes reported)."""
    stream = np.ascontiguousarray(stream, dtype=np.uint8)
    local = np.ascontiguousarray(local, dtype=np.float32)
    if out_cap is None:
        out_cap = compress_bound(local.size)
    out = np.zeros(max(out_cap, 1), dtype=np.uint8)
    nbytes = C.c_size_t(0)
    st = lib().zcref_reduce_step_op(_ptr(stream), stream.size, _ptr(local), local.size, int(op), _ptr(out), out_cap,
                                    C.byref(nbytes))
    return st, (out[: nbytes.value].copy() if st in (OK, ERR_BOUND) else out[:0]), nbytes.value


def quality(ref, test):
    """Returns (status, dict(max_err, sse, min, max, rmse, nrmse, psnr)) of `test` against `ref`."""
    ref = np.ascontiguousarray(ref, dtype=np.float32)
    test = np.ascontiguousarray(test, dtype=np.float32)
    out = np.zeros(4, dtype=np.float64)
    st = lib().zcref_quality(_ptr(ref), _ptr(test), ref.size, _ptr(out))
    return st, metrics(out, ref.size)


def metrics(out, n):
    """The derived measures from the four sums."""
    worst, sse, lo, hi = (float(v) for v in out)
    rng = hi - lo
    rmse = (sse / n) ** 0.5 if n else 0.0
    with np.errstate(divide="ignore", invalid="ignore"):
        nrmse = float(np.float64(rmse) / np.float64(rng)) if n else 0.0
        psnr = float(20.0 * np.log10(np.float64(rng) / np.float64(rmse))) if n else 0.0
    return dict(max_err=worst, sse=sse, min=lo, max=hi, rmse=rmse, nrmse=nrmse, psnr=psnr)
