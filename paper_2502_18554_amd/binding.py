"""ctypes binding of libzc.so: argument marshalling only.

Buffers are torch tensors on the GPU (PyTorch is used for device memory and streams only);
the functions have the names and argument order of include/zc.h.  There is no CPU fallback:
if the HIP library has not been built, loading it raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libzc.so")

ZC_OK, ZC_ERR_ARG, ZC_ERR_CAPACITY, ZC_ERR_FORMAT, ZC_ERR_NONFINITE, ZC_ERR_RANGE, ZC_ERR_BOUND, \
    ZC_ERR_MISMATCH, ZC_ERR_HIP = range(9)
ZC_MAX_K = 64

ZC_STREAM_PLAIN, ZC_TILES_BY_TICKET, ZC_CHAINS_COHERENT = 1, 2, 4

EXPORTS = [
    "zc_compress_bound", "zc_compress_bound_ex", "zc_workspace_bytes", "zc_compress", "zc_compress_ex", "zc_compress_noalloc",
    "zc_compress_part", "zc_decompress", "zc_decompress_ex", "zc_decompress_many", "zc_reduce_compressed",
    "zc_reduce_compressed_ex", "zc_reduce_compressed_op", "zc_reduce_compressed_part", "zc_reduce_step_part", "zc_reduce_step", "zc_reduce_step_op", "zc_decompress_average", "zc_decompress_range",
    "zc_quality", "zc_finish", "zc_peek_header", "zc_strerror", "zc_debug_quantize", "zc_debug_block_offsets", "zc_debug_stream",
    "zc_profile_enable", "zc_profile_collect",
]

_lib = None


class ZcError(RuntimeError):
    def __init__(self, status, what):
        super().__init__(f"{what}: {zc_strerror(status)} (status {status})")
        self.status = status


def lib():
    """Loads libzc.so (built by paper_2502_18554_amd/build.py); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} not found: build it with `python -m paper_2502_18554_amd.build` "
                               "(there is no CPU fallback)")
        L = C.CDLL(_LIB_PATH)
        vp, sz, szp = C.c_void_p, C.c_size_t, C.POINTER(C.c_size_t)
        u = C.c_uint
        L.zc_compress_bound.restype = sz
        L.zc_compress_bound.argtypes = [sz]
        L.zc_compress_bound_ex.restype = sz
        L.zc_compress_bound_ex.argtypes = [sz, u]
        L.zc_workspace_bytes.restype = sz
        L.zc_workspace_bytes.argtypes = [sz, C.c_int]
        L.zc_compress.argtypes = [vp, sz, C.c_float, vp, sz, szp, vp, sz, vp]
        L.zc_compress_ex.argtypes = [vp, sz, C.c_float, vp, sz, szp, vp, sz, vp, u]
        L.zc_compress_noalloc.argtypes = [vp, sz, C.c_float, vp, sz, szp, vp]
        L.zc_compress_part.argtypes = [vp, sz, C.c_float, sz, sz, vp, sz, szp, vp, sz, vp, u]
        L.zc_decompress.argtypes = [vp, sz, vp, sz, szp, vp, sz, vp]
        L.zc_decompress_ex.argtypes = [vp, sz, vp, sz, szp, vp, sz, vp, u]
        L.zc_reduce_compressed.argtypes = [C.POINTER(vp), szp, C.c_int, vp, sz, szp, vp, sz, vp]
        L.zc_reduce_compressed_ex.argtypes = [C.POINTER(vp), szp, C.c_int, vp, sz, szp, vp, sz, vp, u]
        L.zc_reduce_compressed_op.argtypes = [C.POINTER(vp), szp, C.c_int, C.c_int, vp, sz, szp, vp, sz, vp, u]
        L.zc_reduce_compressed_part.argtypes = [C.POINTER(vp), szp, C.c_int, sz, sz, sz, vp, sz, szp, vp, sz, vp, u]
        L.zc_reduce_step_part.argtypes = [vp, sz, vp, sz, C.c_int, sz, sz, vp, sz, szp, vp, sz, vp, u]
        L.zc_reduce_step.argtypes = [vp, sz, vp, sz, vp, sz, szp, vp, sz, vp]
        L.zc_reduce_step_op.argtypes = [vp, sz, vp, sz, C.c_int, vp, sz, szp, vp, sz, vp, u]
        L.zc_decompress_average.argtypes = [vp, sz, vp, sz, szp, vp, sz, vp, u]
        L.zc_decompress_range.argtypes = [vp, sz, sz, sz, vp, sz, szp, vp, sz, vp, u]
        L.zc_quality.argtypes = [vp, vp, sz, C.POINTER(C.c_double), vp, sz, vp]
        L.zc_decompress_many.argtypes = [C.POINTER(vp), szp, C.c_int, C.POINTER(vp), szp, szp, vp, sz, vp, u]
        L.zc_finish.argtypes = [vp, szp, vp]
        L.zc_peek_header.argtypes = [vp, sz, szp, C.POINTER(C.c_float), C.POINTER(C.c_uint), szp, C.POINTER(C.c_uint), vp]
        L.zc_strerror.restype = C.c_char_p
        L.zc_strerror.argtypes = [C.c_int]
        L.zc_debug_quantize.argtypes = [vp, sz, C.c_float, vp, vp, sz, vp]
        L.zc_debug_block_offsets.argtypes = [vp, sz, vp, sz, vp, sz, vp, u]
        L.zc_debug_stream.argtypes = [vp, vp, sz, C.c_int, C.c_int, vp]
        L.zc_profile_enable.argtypes = [C.c_int]
        L.zc_profile_collect.argtypes = [C.POINTER(C.c_float), C.POINTER(C.c_int), C.c_int]
        _lib = L
    return _lib


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _p(t):
    return C.c_void_p(t.data_ptr()) if t is not None else None


def zc_strerror(status):
    return lib().zc_strerror(int(status)).decode()


def zc_compress_bound(n, flags=0):
    return int(lib().zc_compress_bound_ex(int(n), int(flags))) if flags else int(lib().zc_compress_bound(int(n)))


def zc_workspace_bytes(n_max, k_max=1):
    return int(lib().zc_workspace_bytes(int(n_max), int(k_max)))


def _size(t):
    return t.numel() * t.element_size()


def zc_compress(d_in, n, abs_eb, d_out, d_ws, sync=True, stream=None, out_cap=None, flags=0):
    """Returns (status, total_bytes); total_bytes is None in the asynchronous form.  flags 0 goes through
    zc_compress, anything else through zc_compress_ex."""
    nbytes = C.c_size_t(0)
    cap = _size(d_out) if out_cap is None else out_cap
    args = [_p(d_in), n, abs_eb, _p(d_out), cap, C.byref(nbytes) if sync else None, _p(d_ws), _size(d_ws), _stream(stream)]
    st = lib().zc_compress_ex(*args, int(flags)) if flags else lib().zc_compress(*args)
    return st, (nbytes.value if sync else None)


ZC_NOALLOC_MAX_N = 1 << 27


def zc_compress_noalloc(d_in, n, abs_eb, d_out, sync=True, stream=None, out_cap=None):
    """zc_compress on the library's own static workspace.  Returns (status, total_bytes)."""
    nbytes = C.c_size_t(0)
    cap = _size(d_out) if out_cap is None else out_cap
    st = lib().zc_compress_noalloc(_p(d_in), n, abs_eb, _p(d_out), cap, C.byref(nbytes) if sync else None,
                                   _stream(stream))
    return st, (nbytes.value if sync else None)


def zc_compress_part(d_in, n, abs_eb, first_value, count, d_out, d_ws, sync=True, stream=None, out_cap=None, flags=0):
    """One part of a stream compressed in parts.  Returns (status, bytes of the stream final so far)."""
    nbytes = C.c_size_t(0)
    cap = _size(d_out) if out_cap is None else out_cap
    st = lib().zc_compress_part(_p(d_in), int(n), float(abs_eb), int(first_value), int(count), _p(d_out), cap,
                                C.byref(nbytes) if sync else None, _p(d_ws), _size(d_ws), _stream(stream), int(flags))
    return st, (nbytes.value if sync else None)


def zc_decompress(d_in, in_bytes, d_out, d_ws, sync=True, stream=None, out_cap_elems=None, flags=0):
    """Returns (status, n); n is None in the asynchronous form.  flags 0 goes through zc_decompress,
    anything else through zc_decompress_ex."""
    n = C.c_size_t(0)
    cap = (d_out.numel() if d_out is not None else 0) if out_cap_elems is None else out_cap_elems
    args = [_p(d_in), in_bytes, _p(d_out), cap, C.byref(n) if sync else None, _p(d_ws), _size(d_ws), _stream(stream)]
    st = lib().zc_decompress_ex(*args, int(flags)) if flags else lib().zc_decompress(*args)
    return st, (n.value if sync else None)


def zc_decompress_average(d_in, in_bytes, d_out, d_ws, sync=True, stream=None, out_cap_elems=None, flags=0):
    """zc_decompress with every value divided by the stream's nsum.  Returns (status, n)."""
    n = C.c_size_t(0)
    cap = (d_out.numel() if d_out is not None else 0) if out_cap_elems is None else out_cap_elems
    st = lib().zc_decompress_average(_p(d_in), in_bytes, _p(d_out), cap, C.byref(n) if sync else None,
                                     _p(d_ws), _size(d_ws), _stream(stream), int(flags))
    return st, (n.value if sync else None)


def zc_decompress_range(d_in, in_bytes, first_value, count, d_out, d_ws, sync=True, stream=None, out_cap_elems=None,
                        flags=0):
    """Values [first_value, first_value + count) of the stream into d_out.  Returns (status, n)."""
    n = C.c_size_t(0)
    cap = (d_out.numel() if d_out is not None else 0) if out_cap_elems is None else out_cap_elems
    st = lib().zc_decompress_range(_p(d_in), in_bytes, int(first_value), int(count), _p(d_out), cap,
                                   C.byref(n) if sync else None, _p(d_ws), _size(d_ws), _stream(stream), int(flags))
    return st, (n.value if sync else None)


def zc_reduce_compressed(d_chunks, chunk_bytes, d_out, d_ws, sync=True, stream=None, out_cap=None, flags=0):
    """d_chunks: list of device tensors holding the k operand streams.  Returns (status, total_bytes).
    flags 0 goes through zc_reduce_compressed, anything else through zc_reduce_compressed_ex."""
    k = len(d_chunks)
    ptrs = (C.c_void_p * max(k, 1))(*[t.data_ptr() for t in d_chunks])
    sizes = (C.c_size_t * max(k, 1))(*[int(b) for b in chunk_bytes])
    nbytes = C.c_size_t(0)
    cap = _size(d_out) if out_cap is None else out_cap
    args = [ptrs, sizes, k, _p(d_out), cap, C.byref(nbytes) if sync else None, _p(d_ws), _size(d_ws), _stream(stream)]
    st = lib().zc_reduce_compressed_ex(*args, int(flags)) if flags else lib().zc_reduce_compressed(*args)
    return st, (nbytes.value if sync else None)


def zc_reduce_compressed_op(d_chunks, chunk_bytes, op, d_out, d_ws, sync=True, stream=None, out_cap=None, flags=0):
    """zc_reduce_compressed for Sum, Max or Min (ZC_OP_*).  Returns (status, total_bytes)."""
    k = len(d_chunks)
    ptrs = (C.c_void_p * max(k, 1))(*[t.data_ptr() for t in d_chunks])
    sizes = (C.c_size_t * max(k, 1))(*[int(b) for b in chunk_bytes])
    nbytes = C.c_size_t(0)
    cap = _size(d_out) if out_cap is None else out_cap
    st = lib().zc_reduce_compressed_op(ptrs, sizes, k, int(op), _p(d_out), cap, C.byref(nbytes) if sync else None, _p(d_ws),
                                       _size(d_ws), _stream(stream), int(flags))
    return st, (nbytes.value if sync else None)


def zc_reduce_compressed_part(d_chunks, chunk_bytes, n, first_value, count, d_out, d_ws, sync=True, stream=None, out_cap=None,
                              flags=0):
    """One part of a k-way Sum done in parts.  Returns (status, bytes of the stream final so far)."""
    k = len(d_chunks)
    ptrs = (C.c_void_p * max(k, 1))(*[t.data_ptr() for t in d_chunks])
    sizes = (C.c_size_t * max(k, 1))(*[int(b) for b in chunk_bytes])
    nbytes = C.c_size_t(0)
    cap = _size(d_out) if out_cap is None else out_cap
    st = lib().zc_reduce_compressed_part(ptrs, sizes, k, int(n), int(first_value), int(count), _p(d_out), cap,
                                         C.byref(nbytes) if sync else None, _p(d_ws), _size(d_ws), _stream(stream), int(flags))
    return st, (nbytes.value if sync else None)


def zc_reduce_step_part(d_chunk, chunk_bytes, d_local, n_local, op, first_value, count, d_out, d_ws, sync=True, stream=None,
                        out_cap=None, flags=0):
    """One part of a ring round done in parts.  Returns (status, bytes of the stream final so far)."""
    nbytes = C.c_size_t(0)
    cap = _size(d_out) if out_cap is None else out_cap
    st = lib().zc_reduce_step_part(_p(d_chunk), int(chunk_bytes), _p(d_local), int(n_local), int(op), int(first_value),
                                   int(count), _p(d_out), cap, C.byref(nbytes) if sync else None, _p(d_ws), _size(d_ws),
                                   _stream(stream), int(flags))
    return st, (nbytes.value if sync else None)


def zc_decompress_many(d_chunks, chunk_bytes, d_outs, d_ws, sync=True, stream=None, out_cap_elems=None, flags=0):
    """d_chunks / d_outs: lists of k device tensors.  Returns (status, [n of every stream]) (None when not sync)."""
    k = len(d_chunks)
    ptrs = (C.c_void_p * max(k, 1))(*[t.data_ptr() for t in d_chunks])
    sizes = (C.c_size_t * max(k, 1))(*[int(b) for b in chunk_bytes])
    outs = (C.c_void_p * max(k, 1))(*[t.data_ptr() for t in d_outs])
    caps = (C.c_size_t * max(k, 1))(*([t.numel() for t in d_outs] if out_cap_elems is None else [int(c) for c in out_cap_elems]))
    ns = (C.c_size_t * max(k, 1))()
    st = lib().zc_decompress_many(ptrs, sizes, k, outs, caps, ns if sync else None, _p(d_ws), _size(d_ws),
                                  _stream(stream), int(flags))
    return st, ([int(ns[i]) for i in range(k)] if sync else None)


ZC_OP_SUM, ZC_OP_MAX, ZC_OP_MIN = 0, 1, 2


def zc_reduce_step(d_chunk, chunk_bytes, d_local, n_local, d_out, d_ws, sync=True, stream=None, out_cap=None, flags=0):
    """One ring round: received stream + local fp32 values -> stream of the sums.  Returns (status, total_bytes).
    flags 0 goes through zc_reduce_step, anything else through zc_reduce_step_op."""
    if flags:
        return zc_reduce_step_op(d_chunk, chunk_bytes, d_local, n_local, ZC_OP_SUM, d_out, d_ws, sync, stream, out_cap, flags)
    nbytes = C.c_size_t(0)
    cap = _size(d_out) if out_cap is None else out_cap
    st = lib().zc_reduce_step(_p(d_chunk), int(chunk_bytes), _p(d_local), int(n_local), _p(d_out), cap,
                              C.byref(nbytes) if sync else None, _p(d_ws), _size(d_ws), _stream(stream))
    return st, (nbytes.value if sync else None)


def zc_reduce_step_op(d_chunk, chunk_bytes, d_local, n_local, op, d_out, d_ws, sync=True, stream=None, out_cap=None,
                      flags=0):
    """zc_reduce_step for Sum, Max or Min.  Returns (status, total_bytes)."""
    nbytes = C.c_size_t(0)
    cap = _size(d_out) if out_cap is None else out_cap
    st = lib().zc_reduce_step_op(_p(d_chunk), int(chunk_bytes), _p(d_local), int(n_local), int(op), _p(d_out), cap,
                                 C.byref(nbytes) if sync else None, _p(d_ws), _size(d_ws), _stream(stream), int(flags))
    return st, (nbytes.value if sync else None)


def zc_quality(d_ref, d_test, n, d_ws, stream=None):
    """Returns (status, [max |ref - test|, sum of squared differences, min(ref), max(ref)])."""
    out = (C.c_double * 4)()
    st = lib().zc_quality(_p(d_ref), _p(d_test), int(n), out, _p(d_ws), d_ws.numel() * d_ws.element_size(),
                          _stream(stream))
    return st, [float(v) for v in out]


def zc_finish(d_ws, stream=None):
    """Returns (status, size result) of the last asynchronous call that used d_ws."""
    r = C.c_size_t(0)      # d_ws None: the call was zc_compress_noalloc
    st = lib().zc_finish(_p(d_ws), C.byref(r), _stream(stream))
    return st, r.value


def zc_peek_header(d_in, in_bytes, stream=None):
    """Returns (status, n, abs_eb, nsum, total_bytes, flags of the stream's variant)."""
    n, eb, nsum, total, flags = C.c_size_t(0), C.c_float(0), C.c_uint(0), C.c_size_t(0), C.c_uint(0)
    st = lib().zc_peek_header(_p(d_in), in_bytes, C.byref(n), C.byref(eb), C.byref(nsum), C.byref(total),
                              C.byref(flags), _stream(stream))
    return st, n.value, eb.value, nsum.value, total.value, flags.value


def zc_debug_quantize(d_in, n, abs_eb, d_q, d_ws, stream=None):
    return lib().zc_debug_quantize(_p(d_in), n, abs_eb, _p(d_q), _p(d_ws), _size(d_ws), _stream(stream))


def zc_debug_block_offsets(d_in, in_bytes, d_off_words, d_ws, stream=None, flags=0):
    return lib().zc_debug_block_offsets(_p(d_in), in_bytes, _p(d_off_words), d_off_words.numel(), _p(d_ws),
                                        _size(d_ws), _stream(stream), int(flags))


def zc_debug_stream(d_in, d_out, tiles, loads, stores, stream=None):
    """A kernel that only streams: workgroup t reads loads x 8 KiB of d_in and writes stores x 8 KiB of d_out."""
    return lib().zc_debug_stream(_p(d_in) if d_in is not None else None, _p(d_out) if d_out is not None else None,
                                 int(tiles), int(loads), int(stores), _stream(stream))


KERNEL_NAMES = {1: "compress", 2: "decompress", 3: "reduce", 4: "reduce_step", 5: "stream"}


def zc_profile_enable(on, only=None):
    """Times the main kernels from now on (on=True), or stops (False).  only: names from KERNEL_NAMES to time just those."""
    if on and only:
        code = sum(1 << k for k, name in KERNEL_NAMES.items() if name in only)
        return lib().zc_profile_enable(code)
    return lib().zc_profile_enable(1 if on else 0)


def zc_profile_collect(cap=65536):
    """Returns [(kernel name, milliseconds)] for the main kernels launched since zc_profile_enable(True)."""
    ms = (C.c_float * cap)()
    kind = (C.c_int * cap)()
    count = lib().zc_profile_collect(ms, kind, cap)
    if count < 0:
        raise ZcError(-count, "zc_profile_collect")
    return [(KERNEL_NAMES.get(kind[i], str(kind[i])), float(ms[i])) for i in range(count)]
