"""CPU tests of the HIP library's host-side logic: the shared library loads and exports every
symbol declared in include/zc.h, size helpers agree with the stream layout, argument checks
that need no GPU, and the in-register bit-matrix transposes (plain integer code shared by the
kernels) against numpy.packbits."""
import ctypes as C
import os
import re
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def libzc():
    path = os.path.join(ROOT, "paper_2502_18554_amd", "libzc.so")
    if not os.path.exists(path):
        pytest.skip("libzc.so not built (run __graft_entry__.build())")
    return C.CDLL(path)


def test_library_exports_every_declared_symbol(libzc):
    header = open(os.path.join(ROOT, "include", "zc.h")).read()
    names = set(re.findall(r"\b(zc_[a-z_]+)\s*\(", header))
    assert {"zc_compress", "zc_decompress", "zc_reduce_compressed", "zc_finish"} <= names
    for name in sorted(names):
        assert hasattr(libzc, name), name
    from paper_2502_18554_amd import binding
    assert set(binding.EXPORTS) == names


def test_size_helpers(libzc):
    libzc.zc_compress_bound.restype = C.c_size_t
    libzc.zc_compress_bound.argtypes = [C.c_size_t]
    libzc.zc_compress_bound_ex.restype = C.c_size_t
    libzc.zc_compress_bound_ex.argtypes = [C.c_size_t, C.c_uint]
    libzc.zc_workspace_bytes.restype = C.c_size_t
    libzc.zc_workspace_bytes.argtypes = [C.c_size_t, C.c_int]
    pad16 = lambda v: (v + 15) // 16 * 16
    for n in (0, 1, 31, 32, 33, 8192, 8193, 1 << 20, (1 << 27) + 5):
        nb = (n + 31) // 32
        indexed = 32 + pad16(4 * ((nb + 63) // 64 + 1)) + pad16(nb) + pad16(4 * nb) + 128 * nb
        assert libzc.zc_compress_bound(n) == indexed == libzc.zc_compress_bound_ex(n, 0)     # the default variant
        assert libzc.zc_compress_bound_ex(n, 1) == 32 + pad16(nb) + pad16(4 * nb) + 128 * nb  # ZC_STREAM_PLAIN
    assert libzc.zc_workspace_bytes(1 << 27, 1) < (1 << 22)      # under 1 % of the 512 MiB it serves
    assert libzc.zc_workspace_bytes(1 << 26, 8) < libzc.zc_workspace_bytes(1 << 27, 8)
    libzc.zc_strerror.restype = C.c_char_p
    assert b"bound" in libzc.zc_strerror(6) and libzc.zc_strerror(0) == b"ok"


def test_argument_checks_without_gpu(libzc):
    vp, sz = C.c_void_p, C.c_size_t
    libzc.zc_compress.argtypes = [vp, sz, C.c_float, vp, sz, C.POINTER(sz), vp, sz, vp]
    libzc.zc_decompress.argtypes = [vp, sz, vp, sz, C.POINTER(sz), vp, sz, vp]
    libzc.zc_reduce_compressed.argtypes = [C.POINTER(vp), C.POINTER(sz), C.c_int, vp, sz, C.POINTER(sz), vp, sz, vp]
    assert libzc.zc_compress(None, 10, 1e-3, None, 0, None, None, 0, None) == 1
    assert libzc.zc_compress(0x1000, 10, 0.0, 0x2000, 100, None, 0x3000, 4096, None) == 1      # eb
    assert libzc.zc_compress(0x1004, 10, 1e-3, 0x2000, 100, None, 0x3000, 4096, None) == 1     # alignment
    assert libzc.zc_compress(0x1000, 1 << 20, 1e-3, 0x2000, 100, None, 0x3000, 64, None) == 1  # workspace
    libzc.zc_compress_part.argtypes = [vp, sz, C.c_float, sz, sz, vp, sz, C.POINTER(sz), vp, sz, vp, C.c_uint]
    assert libzc.zc_compress_part(0x1000, 1 << 20, 1e-3, 100, 16384, 0x2000, 1 << 22, None, 0x3000, 1 << 20, None, 0) == 1   # not at a tile
    assert libzc.zc_compress_part(0x1000, 1 << 20, 1e-3, 0, 100, 0x2000, 1 << 22, None, 0x3000, 1 << 20, None, 0) == 1       # not a whole tile
    assert libzc.zc_compress_part(0x1000, 1 << 20, 1e-3, 1 << 20, 16384, 0x2000, 1 << 22, None, 0x3000, 1 << 20, None, 0) == 1  # past the end
    libzc.zc_compress_ex.argtypes = [vp, sz, C.c_float, vp, sz, C.POINTER(sz), vp, sz, vp, C.c_uint]
    assert libzc.zc_compress_ex(0x1000, 10, 1e-3, 0x2000, 100, None, 0x3000, 4096, None, 8) == 1   # unknown flag
    libzc.zc_debug_stream.argtypes = [vp, vp, sz, C.c_int, C.c_int, vp]
    assert libzc.zc_debug_stream(0x1000, 0x2000, 4, 0, 0, None) == 1        # nothing to do per lane
    assert libzc.zc_debug_stream(0x1000, 0x2000, 4, 17, 1, None) == 1       # more than 16 accesses
    assert libzc.zc_debug_stream(None, 0x2000, 4, 1, 1, None) == 1          # loads without a source
    assert libzc.zc_debug_stream(0x1008, 0x2000, 4, 1, 1, None) == 1        # alignment
    assert libzc.zc_decompress(None, 100, None, 0, None, None, 0, None) == 1
    assert libzc.zc_decompress(0x1000, 16, 0x2000, 8, None, 0x3000, 4096, None) == 3           # shorter than a header
    assert libzc.zc_reduce_compressed(None, None, 0, None, 0, None, None, 0, None) == 1
    ptrs = (vp * 1)(0x1000)
    sizes = (sz * 1)(100)
    assert libzc.zc_reduce_compressed(ptrs, sizes, 65, 0x2000, 100, None, 0x3000, 4096, None) == 1
    libzc.zc_reduce_step.argtypes = [vp, sz, vp, sz, vp, sz, C.POINTER(sz), vp, sz, vp]
    assert libzc.zc_reduce_step(None, 100, 0x1000, 8, 0x2000, 100, None, 0x3000, 4096, None) == 1
    assert libzc.zc_reduce_step(0x1000, 100, None, 8, 0x2000, 100, None, 0x3000, 4096, None) == 1      # no local values
    assert libzc.zc_reduce_step(0x1000, 100, 0x1008, 8, 0x2000, 100, None, 0x3000, 4096, None) == 1    # alignment
    assert libzc.zc_reduce_step(0x1000, 16, 0x4000, 8, 0x2000, 100, None, 0x3000, 4096, None) == 3     # shorter than a header
    libzc.zc_reduce_step_op.argtypes = [vp, sz, vp, sz, C.c_int, vp, sz, C.POINTER(sz), vp, sz, vp, C.c_uint]
    for op in (-1, 3):
        assert libzc.zc_reduce_step_op(0x1000, 100, 0x4000, 8, op, 0x2000, 100, None, 0x3000, 4096, None, 0) == 1   # unknown op
    assert libzc.zc_reduce_step_op(0x1000, 16, 0x4000, 8, 2, 0x2000, 100, None, 0x3000, 4096, None, 0) == 3
    assert libzc.zc_reduce_step_op(0x1000, 100, 0x4000, 8, 2, 0x2000, 100, None, 0x3000, 4096, None, 8) == 1   # unknown flag
    libzc.zc_decompress_average.argtypes = [vp, sz, vp, sz, C.POINTER(sz), vp, sz, vp, C.c_uint]
    assert libzc.zc_decompress_average(None, 100, None, 0, None, None, 0, None, 0) == 1
    assert libzc.zc_decompress_average(0x1000, 16, 0x2000, 8, None, 0x3000, 4096, None, 1) == 3
    assert libzc.zc_decompress_average(0x1000, 100, 0x2000, 8, None, 0x3000, 4096, None, 2) == 1      # a flag for writers only
    libzc.zc_decompress_range.argtypes = [vp, sz, sz, sz, vp, sz, C.POINTER(sz), vp, sz, vp, C.c_uint]
    assert libzc.zc_decompress_range(0x1000, 100, 100, 8, 0x2000, 8, None, 0x3000, 4096, None, 0) == 1     # not at a segment
    assert libzc.zc_decompress_range(0x1000, 16, 2048, 8, 0x2000, 8, None, 0x3000, 4096, None, 0) == 3
    assert libzc.zc_decompress_range(None, 100, 0, 8, 0x2000, 8, None, 0x3000, 4096, None, 0) == 1
    assert libzc.zc_reduce_step(0x1000, 100, 0x4000, 1 << 20, 0x2000, 100, None, 0x3000, 64, None) == 1  # workspace
    libzc.zc_decompress_many.argtypes = [C.POINTER(vp), C.POINTER(sz), C.c_int, C.POINTER(vp), C.POINTER(sz), C.POINTER(sz),
                                         vp, sz, vp, C.c_uint]
    outs = (vp * 1)(0x4000)
    caps = (sz * 1)(8)
    assert libzc.zc_decompress_many(ptrs, sizes, 0, outs, caps, None, 0x3000, 4096, None, 0) == 1
    assert libzc.zc_decompress_many(ptrs, sizes, 1, None, caps, None, 0x3000, 4096, None, 0) == 1
    assert libzc.zc_decompress_many(ptrs, (sz * 1)(16), 1, outs, caps, None, 0x3000, 4096, None, 0) == 3
    assert libzc.zc_decompress_many(ptrs, sizes, 1, (vp * 1)(0x4004), caps, None, 0x3000, 4096, None, 0) == 1
    libzc.zc_quality.argtypes = [vp, vp, sz, C.POINTER(C.c_double), vp, sz, vp]
    out4 = (C.c_double * 4)()
    assert libzc.zc_quality(0x1000, 0x2000, 8, None, 0x3000, 4096, None) == 1
    assert libzc.zc_quality(0x1000, None, 8, out4, 0x3000, 4096, None) == 1
    assert libzc.zc_quality(0x1000, 0x2000, 1 << 24, out4, 0x3000, 64, None) == 1                       # workspace


@pytest.fixture(scope="module")
def bm():
    src = os.path.join(ROOT, "tests", "host", "bitmatrix_host.cpp")
    lib = os.path.join(ROOT, "tests", "host", "libbitmatrix_host.so")
    hdr = os.path.join(ROOT, "paper_2502_18554_amd", "csrc", "zc_bitmatrix.h")
    if not os.path.exists(lib) or os.path.getmtime(lib) < max(os.path.getmtime(src), os.path.getmtime(hdr)):
        subprocess.run(["g++", "-std=c++17", "-O1", "-shared", "-fPIC", src, "-o", lib], check=True)
    return C.CDLL(lib)


@pytest.mark.parametrize("cls,maxw", [(8, 7), (816, 7), (16, 15), (32, 31)])
def test_bit_matrix_transposes_match_packbits(bm, cls, maxw):
    rng = np.random.default_rng(cls)
    p32, pi32 = C.POINTER(C.c_uint32), C.POINTER(C.c_int32)
    for trial in range(200):
        w = int(rng.integers(0, maxw + 1))
        mag = rng.integers(0, 1 << w, 32, dtype=np.uint64).astype(np.int64) if w else np.zeros(32, np.int64)
        if trial % 7 == 0 and w:
            mag[:] = (1 << w) - 1
        sign = rng.integers(0, 2, 32).astype(np.int64) * (mag != 0)      # a zero delta has sign 0
        d = np.where(sign == 1, -mag, mag).astype(np.int32)
        out = np.zeros(32, np.uint32)
        bm.bm_planes_from_deltas(d.ctypes.data_as(pi32), cls, out.ctypes.data_as(p32))
        want = np.zeros(32, np.uint32)
        want[0] = np.packbits(sign.astype(np.uint8), bitorder="little").view("<u4")[0]
        for p in range(maxw):
            want[1 + p] = np.packbits(((mag >> p) & 1).astype(np.uint8), bitorder="little").view("<u4")[0]
        assert np.array_equal(out, want), (cls, trial, w)
        d2 = np.zeros(32, np.int32)
        bm.bm_deltas_from_planes(out.ctypes.data_as(p32), 8 if cls == 816 else cls, d2.ctypes.data_as(pi32))
        assert np.array_equal(d2, d)


def test_calls_from_two_threads_share_no_setting(libzc):
    """The library keeps no settings: two host threads that want different stream variants and tile
    hand-outs say so in their calls and never see each other's choice.  (Without a GPU only the
    host side of the calls can run: the size helpers and the argument checks.)"""
    import threading
    vp, sz = C.c_void_p, C.c_size_t
    libzc.zc_compress_bound_ex.restype = sz
    libzc.zc_compress_bound_ex.argtypes = [sz, C.c_uint]
    libzc.zc_compress_ex.argtypes = [vp, sz, C.c_float, vp, sz, C.POINTER(sz), vp, sz, vp, C.c_uint]
    libzc.zc_decompress_ex.argtypes = [vp, sz, vp, sz, C.POINTER(sz), vp, sz, vp, C.c_uint]
    pad16 = lambda v: (v + 15) // 16 * 16
    failures = []

    def worker(flags, rounds):
        plain = bool(flags & 1)
        for i in range(rounds):
            n = 1000 + 37 * i
            nb = (n + 31) // 32
            want = 32 + (0 if plain else pad16(4 * ((nb + 63) // 64 + 1))) + pad16(nb) + pad16(4 * nb) + 128 * nb
            if libzc.zc_compress_bound_ex(n, flags) != want:
                failures.append(("bound", flags, n))
            # argument checks only (a misaligned input): no launch, whatever the flags say
            if libzc.zc_compress_ex(0x1004, n, 1e-3, 0x2000, 100, None, 0x3000, 1 << 20, None, flags) != 1:
                failures.append(("compress", flags, n))
            if libzc.zc_decompress_ex(0x1000, 16, 0x2000, 8, None, 0x3000, 4096, None, flags & 1) != 3:
                failures.append(("decompress", flags, n))

    threads = [threading.Thread(target=worker, args=(f, 2000)) for f in (0, 1, 2, 3)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not failures, failures[:5]
