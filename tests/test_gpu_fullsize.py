"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (asynchronous calls on device-resident buffers).

The two graded configurations (the 512^3 field at rel 1e-4, and the fused reduce of 8 x 2^26 values) are
compared with the reference CPU codec as wholes: stream bytes and reconstruction, bit for bit, in both
stream variants.  The reference cannot run every buffer of this size inside a test, but blocks are
independent: for the other configurations a block-aligned slice of the input, compressed alone by the
reference codec, must reproduce the GPU stream's width bytes, outliers and payload bytes of those blocks
(found through the exclusive sum of the GPU stream's own width table, computed with torch), and its
reconstruction must equal the GPU's bit for bit.  Slices are drawn with a fixed seed and always
include the first blocks and the ragged end.  On top of that come the properties that hold at
any size: error bound on every value, idempotence on the grid, header fields, sizes that add up.
"""
import numpy as np
import pytest
import torch

import gpuutil
from gpuutil import zc
from paper_2502_18554_amd import synth
from paper_2502_18554_amd.binding import ZC_OK

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
SLICE = 1 << 17          # values per sampled slice (4096 blocks: 16 tiles, crosses index groups)


def pad16(v):
    return (v + 15) // 16 * 16


def tables_end(nb):
    return 32 + pad16(nb) + pad16(4 * nb)


INDEXED = False          # the stream variant the library is set to (the reference stays plain)


@pytest.fixture(params=["plain", "indexed"], autouse=True)
def gpu_stream_variant(request):
    """Every test of this module runs on both stream variants of the library.  The reference
    compresses slices of the input into plain streams; their tables and payload are compared
    with the matching parts of the library's stream, whose index is checked against its own
    width table."""
    global INDEXED
    INDEXED = request.param == "indexed"
    gpuutil.set_variant(None, INDEXED)
    yield request.param
    INDEXED = False
    gpuutil.set_variant(None, False)


def u8(nbytes):
    return torch.empty(nbytes + 64, dtype=torch.uint8, device=DEV)


class Stream:
    """A GPU stream plus the block positions derived from its own width table."""

    def __init__(self, buf, total, n):
        self.buf, self.total, self.n = buf, total, n
        self.nb = (n + 31) // 32
        self.nseg = (self.nb + 63) // 64
        w0 = 32 + (pad16(4 * (self.nseg + 1)) if INDEXED else 0)
        self.index = buf[32:32 + 4 * (self.nseg + 1)].view(torch.int32) if INDEXED else None
        self.widths = buf[w0:w0 + self.nb]
        words = torch.where(self.widths > 0, self.widths.to(torch.int64) + 1, torch.zeros((), dtype=torch.int64, device=DEV))
        self.off = torch.cumsum(words, 0) - words            # exclusive, in words
        self.payload_words = int(words.sum())
        o0 = w0 + pad16(self.nb)
        self.outliers = buf[o0:o0 + 4 * self.nb].view(torch.int32)
        self.tend = o0 + pad16(4 * self.nb)

    def header(self):
        h = self.buf[:32].cpu().numpy()
        return dict(magic=int(h[0:4].view("<u4")[0]), version=int(h[4:6].view("<u2")[0]), n=int(h[8:16].view("<u8")[0]),
                    eb_bits=int(h[16:20].view("<u4")[0]),
                    nsum=int(h[20:24].view("<u4")[0]), total=int(h[24:32].view("<u8")[0]))

    def payload_of(self, b0, b1):
        lo = int(self.off[b0])
        hi = int(self.off[b1]) if b1 < self.nb else self.payload_words
        return self.buf[self.tend + 4 * lo: self.tend + 4 * hi].cpu().numpy()


def sample_starts(n, rng, count):
    nb = (n + 31) // 32
    span = SLICE // 32
    last = max(nb - span, 0)
    starts = {0, last}
    while len(starts) < min(count, last + 1):
        starts.add(int(rng.integers(0, last + 1)))
    return sorted(starts)


def compress_async(x, eb, ws):
    n = x.numel()
    out = u8(zc.zc_compress_bound(n))
    st, _ = zc.zc_compress(x, n, eb, out, ws, sync=False)
    assert st == ZC_OK
    st, total = zc.zc_finish(ws)
    return st, out, total


def decompress_async(stream, total, out, ws):
    st, _ = zc.zc_decompress(stream, total, out, ws, sync=False)
    assert st == ZC_OK
    return zc.zc_finish(ws)


def check_header_and_sizes(s, eb, nsum=1):
    h = s.header()
    assert h["magic"] == 0x314C435A and h["n"] == s.n and h["nsum"] == nsum and h["total"] == s.total
    assert h["eb_bits"] == int(np.float32(eb).view(np.uint32))
    assert s.total == s.tend + 4 * s.payload_words
    assert int(s.widths.max()) <= 31
    if INDEXED:          # the index is the exclusive sum of the block sizes at every 64th block, then the total
        assert h["version"] == (3 if int(s.widths.max()) > 15 else 2)
        want = torch.cat([s.off[::64], torch.tensor([s.payload_words], device=DEV)])
        assert torch.equal(s.index.to(torch.int64) & 0xFFFFFFFF, want), "segment index differs from the width table's sums"
        pad = s.buf[32 + 4 * (s.nseg + 1):32 + pad16(4 * (s.nseg + 1))]
        assert not bool(pad.any())
    else:
        assert h["version"] == 1


def check_slices_against_reference(zcref, x, eb, s, y, rng, count=6):
    for b0 in sample_starts(s.n, rng, count):
        v0, v1 = 32 * b0, min(s.n, 32 * b0 + SLICE)
        st, ref, total = zcref.compress(x[v0:v1].cpu().numpy(), eb)
        assert st == 0
        nbs = (v1 - v0 + 31) // 32
        assert np.array_equal(s.widths[b0:b0 + nbs].cpu().numpy(), ref[32:32 + nbs]), f"widths differ in slice at block {b0}"
        o0 = 32 + pad16(nbs)
        assert np.array_equal(s.outliers[b0:b0 + nbs].cpu().numpy(), ref[o0:o0 + 4 * nbs].view("<i4")), f"outliers differ at block {b0}"
        assert np.array_equal(s.payload_of(b0, b0 + nbs), ref[tables_end(nbs):total]), f"payload differs at block {b0}"
        if y is not None:
            st, y_ref, _ = zcref.decompress(ref)
            assert np.array_equal(y[v0:v1].cpu().numpy().view(np.uint32), y_ref.view(np.uint32)), f"floats differ at block {b0}"


def check_quality(zcref, x, y, eb, rng):
    """zc_quality on the whole buffers: its maximum is the torch maximum, a sampled slice agrees with
    the reference, and the NRMSE is that of a uniform quantiser of this step."""
    n = x.numel()
    st, q = zc.zc_quality(x, y, n, u8(zc.zc_workspace_bytes(n, 1)))
    assert st == ZC_OK
    assert q[0] == max_abs_err(x, y) and q[2] == float(x.min()) and q[3] == float(x.max())
    step = float(np.float32(eb)) * 63.0 / 32.0
    nrmse = (q[1] / n) ** 0.5 / (q[3] - q[2])
    assert abs(nrmse / (step / 12 ** 0.5 / (q[3] - q[2])) - 1) < 0.05
    v0 = 32 * int(rng.integers(0, max(1, (n - SLICE) // 32)))
    st, part = zc.zc_quality(x[v0:v0 + SLICE], y[v0:v0 + SLICE], min(SLICE, n - v0), u8(zc.zc_workspace_bytes(SLICE, 1)))
    _, want = zcref.quality(x[v0:v0 + SLICE].cpu().numpy(), y[v0:v0 + SLICE].cpu().numpy())
    assert part[0] == want["max_err"] and part[2] == want["min"] and part[3] == want["max"]
    assert abs(part[1] / want["sse"] - 1) < 1e-10


class reference_variant:
    """Inside the block the reference writes and accepts the stream variant the library is being run on
    (outside it stays on plain streams, which is what the slice comparisons expect)."""

    def __init__(self, zcref):
        self.zcref = zcref

    def __enter__(self):
        self.zcref.set_indexed(INDEXED)

    def __exit__(self, *exc):
        self.zcref.set_indexed(False)


def assert_same_bytes(d_buf, ref, what, chunk=1 << 26):
    """A device buffer against a numpy array, byte for byte, without a second copy of either."""
    assert d_buf.numel() == ref.size, f"{what}: {d_buf.numel()} bytes, reference {ref.size}"
    for i in range(0, ref.size, chunk):
        got = d_buf[i:i + chunk].cpu().numpy()
        if not np.array_equal(got, ref[i:i + chunk]):
            at = i + int(np.nonzero(got != ref[i:i + chunk])[0][0])
            raise AssertionError(f"{what} differs from the reference at byte {at}")


def max_abs_err(x, y, chunk=1 << 27):
    worst = 0.0
    for i in range(0, x.numel(), chunk):
        worst = max(worst, float((x[i:i + chunk].double() - y[i:i + chunk].double()).abs().max()))
    return worst


@pytest.mark.parametrize("rel", [1e-2, 1e-3, 1e-4])
def test_field_512cube(zcref, rel):
    """Benchmark configuration 2: the 512^3 power-law field at the three bounds."""
    rng = np.random.default_rng(int(round(-np.log10(rel))))
    x = synth.power_law_field((512, 512, 512), seed=0, device=DEV)
    n = x.numel()
    eb = synth.abs_bound(x, rel)
    ws = u8(zc.zc_workspace_bytes(n, 1))
    st, buf, total = compress_async(x, eb, ws)
    assert st == ZC_OK
    s = Stream(buf, total, n)
    check_header_and_sizes(s, eb)
    y = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    st, n_out = decompress_async(buf, total, y, ws)
    assert st == ZC_OK and n_out == n
    assert max_abs_err(x, y) <= eb
    check_slices_against_reference(zcref, x, eb, s, y, rng)
    check_quality(zcref, x, y, eb, rng)
    # idempotence on the grid: the reconstruction compresses to the same bytes
    st, buf2, total2 = compress_async(y, eb, ws)
    assert st == ZC_OK and total2 == total and torch.equal(buf2[:total], buf[:total])
    if rel == 1e-4:
        # the graded configuration: the whole stream and the whole reconstruction against the reference
        # run on the whole field (the index levels above one span only exist at this size)
        with reference_variant(zcref):
            st, ref, ref_total = zcref.compress(x.cpu().numpy(), eb)
            assert st == 0 and ref_total == total
            assert_same_bytes(buf[:total], ref, "compressed stream")
            st, y_ref, _ = zcref.decompress(ref)
        assert st == 0 and np.array_equal(y.cpu().numpy().view(np.uint32), y_ref.view(np.uint32))


def test_field_512cube_in_parts_and_chunks(zcref):
    """Configuration 2 produced by zc_compress_part in 8 parts and read back by zc_decompress_range in 8
    chunks: the stream is byte for byte that of zc_compress (whose slices the test above compares with the
    reference), every chunk holds the values of the whole decompression, and slices of both agree with
    the reference once more."""
    rng = np.random.default_rng(77)
    x = synth.power_law_field((512, 512, 512), seed=0, device=DEV)
    n = x.numel()
    eb = synth.abs_bound(x, 1e-3)
    ws = u8(zc.zc_workspace_bytes(n, 1))
    st, whole, total = compress_async(x, eb, ws)
    assert st == ZC_OK
    buf = u8(zc.zc_compress_bound(n))
    buf.fill_(0xA5)
    part = n // 8
    so_far = []
    for i in range(8):
        st, b = zc.zc_compress_part(x, n, eb, i * part, part, buf, ws)
        assert st == ZC_OK
        so_far.append(b)
    assert so_far == sorted(so_far) and so_far[-1] == total
    assert torch.equal(buf[:total], whole[:total])
    s = Stream(buf, total, n)
    check_header_and_sizes(s, eb)
    # the size after part i is where block i * part / 32 starts
    for i in range(7):
        assert so_far[i] == s.tend + 4 * int(s.off[(i + 1) * part // 32])
    y = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    y_whole = torch.empty(n, dtype=torch.float32, device=DEV)
    st, _ = decompress_async(buf, total, y_whole, ws)
    assert st == ZC_OK
    for i in range(8):
        st, m = zc.zc_decompress_range(buf, total, i * part, part, y[i * part:(i + 1) * part], ws)
        assert st == ZC_OK and m == part, (i, st, m)
    assert torch.equal(y.view(torch.int32), y_whole.view(torch.int32))
    # an odd chunk: starts at a segment that is not a tile's first, ends inside a block
    first, count = 2048 * 12345, 3 * 8192 + 17
    z = torch.full((count + 8,), float("nan"), dtype=torch.float32, device=DEV)
    st, m = zc.zc_decompress_range(buf, total, first, count, z, ws, out_cap_elems=count)
    assert st == ZC_OK and m == count
    assert torch.equal(z[:count].view(torch.int32), y_whole[first:first + count].view(torch.int32)) and bool(torch.isnan(z[count:]).all())
    check_slices_against_reference(zcref, x, eb, s, y, rng, count=3)


def _rank_buffers(k=8):
    return [synth.power_law_field((256, 512, 512), seed=100 + r, device=DEV) for r in range(k)]


def test_allgather_8x64M(zcref):
    """Configuration 3: 8 rank buffers compressed at rel 1e-3, all decompressed into one 2^29-value output."""
    rng = np.random.default_rng(3)
    xs = _rank_buffers()
    m = xs[0].numel()
    ws = u8(zc.zc_workspace_bytes(m, 1))
    out = torch.full((8 * m,), float("nan"), dtype=torch.float32, device=DEV)
    streams = []
    for x in xs:
        eb = synth.abs_bound(x, 1e-3)
        st, buf, total = compress_async(x, eb, ws)
        assert st == ZC_OK
        streams.append((Stream(buf, total, m), eb))
    for r in reversed(range(8)):                 # a call that overran its slice would damage one already checked
        s, eb = streams[r]
        st, n_out = decompress_async(s.buf, s.total, out[r * m:(r + 1) * m], ws)
        assert st == ZC_OK and n_out == m
    for r, (s, eb) in enumerate(streams):
        check_header_and_sizes(s, eb)
        assert max_abs_err(xs[r], out[r * m:(r + 1) * m]) <= eb
        if r in (0, 7):
            check_slices_against_reference(zcref, xs[r], eb, s, out[r * m:(r + 1) * m], rng, count=3)
    # the same eight streams in one call: bit for bit what the eight calls wrote
    del xs
    out2 = torch.full((8 * m,), float("nan"), dtype=torch.float32, device=DEV)
    ws8 = u8(zc.zc_workspace_bytes(m, 8))
    st, _ = zc.zc_decompress_many([s.buf for s, _ in streams], [s.total for s, _ in streams],
                                  [out2[r * m:(r + 1) * m] for r in range(8)], ws8, sync=False)
    assert st == ZC_OK
    st, total_n = zc.zc_finish(ws8)
    assert st == ZC_OK and total_n == 8 * m
    assert torch.equal(out.view(torch.int32), out2.view(torch.int32))


@pytest.mark.parametrize("hand_out", ["dispatch_order", "tickets"])
def test_allreduce_8x64M(zcref, hand_out):
    """Configuration 4: fused reduce of 8 compressed rank buffers at a common bound; error <= 8 eb.
    Run with both ways of handing out tiles (the other tests of this file use the default)."""
    gpuutil.set_tickets(hand_out == "tickets")
    try:
        _allreduce_8x64M(zcref)
    finally:
        gpuutil.set_tickets(False)


def _allreduce_8x64M(zcref):
    rng = np.random.default_rng(4)
    xs = _rank_buffers()
    m = xs[0].numel()
    eb = float(torch.tensor(2e-4, dtype=torch.float32))
    ws = u8(zc.zc_workspace_bytes(m, 8))
    streams = []
    for x in xs:
        st, buf, total = compress_async(x, eb, ws)
        assert st == ZC_OK
        streams.append(Stream(buf[:total].clone(), total, m))
    red = u8(zc.zc_compress_bound(m))
    st, _ = zc.zc_reduce_compressed([s.buf for s in streams], [s.total for s in streams], red, ws, sync=False)
    assert st == ZC_OK
    st, total = zc.zc_finish(ws)
    assert st == ZC_OK
    r = Stream(red, total, m)
    check_header_and_sizes(r, eb, nsum=8)
    y = torch.empty(m, dtype=torch.float32, device=DEV)
    st, n_out = decompress_async(red, total, y, ws)
    assert st == ZC_OK and n_out == m
    exact = torch.zeros(m, dtype=torch.float64, device=DEV)
    for x in xs:
        exact += x.double()
    assert float((y.double() - exact).abs().max()) <= 8 * eb
    # the Average aggregation: the same stream decoded and divided by its nsum; within eb of the exact
    # mean, and bit for bit the reference's averaging decompression on a sampled slice
    ya = torch.full((m,), float("nan"), dtype=torch.float32, device=DEV)
    st, _ = zc.zc_decompress_average(red, total, ya, ws, sync=False)
    assert st == ZC_OK
    st, n_avg = zc.zc_finish(ws)
    assert st == ZC_OK and n_avg == m
    assert float((ya.double() - exact / 8).abs().max()) <= eb * (1 + 1e-6)
    del exact
    b0 = sample_starts(m, rng, 3)[1]
    v0, v1 = 32 * b0, min(m, 32 * b0 + SLICE)
    st, ref, _ = zcref.reduce([zcref.compress(x[v0:v1].cpu().numpy(), eb)[1] for x in xs])
    assert st == 0
    st, ya_ref, _ = zcref.decompress(ref, average=True)
    assert st == 0 and np.array_equal(ya[v0:v1].cpu().numpy().view(np.uint32), ya_ref.view(np.uint32))
    if not gpuutil.TICKETS:
        # the graded configuration: the whole reduced stream against the reference's reduce of the whole operands
        with reference_variant(zcref):
            refs = [zcref.compress(x.cpu().numpy(), eb)[1] for x in xs]
            for s_gpu, ref in zip(streams, refs):
                assert_same_bytes(s_gpu.buf[:s_gpu.total], ref, "operand stream")
            st, ref, ref_total = zcref.reduce(refs)
            del refs
        assert st == 0 and ref_total == total
        assert_same_bytes(red[:total], ref, "reduced stream")
        del ref
    # the k-way Max and Min of the same operands: the quantiser is monotone, so the whole stream must be that of
    # the elementwise extreme of the buffers compressed once (a call pinned above), but for its nsum (8 against 1)
    red_x = u8(zc.zc_compress_bound(m))
    for op, fold in ((zc.binding.ZC_OP_MAX, torch.maximum), (zc.binding.ZC_OP_MIN, torch.minimum)):
        st, _ = zc.zc_reduce_compressed_op([s.buf for s in streams], [s.total for s in streams], op, red_x, ws, sync=False)
        assert st == ZC_OK
        st, total_x = zc.zc_finish(ws)
        assert st == ZC_OK
        ext = xs[0]
        for x in xs[1:]:
            ext = fold(ext, x)
        st, direct, total_d = compress_async(ext, eb, ws)
        assert st == ZC_OK and total_d == total_x, (op, total_d, total_x)
        assert torch.equal(red_x[:20], direct[:20]) and torch.equal(red_x[24:total_x], direct[24:total_x]), op
        assert int(red_x[20:24].cpu().numpy().view("<u4")[0]) == 8
        del ext, direct
    del red_x
    # sampled slices: the reference reduce of the operands' slices reproduces the GPU stream there
    for b0 in sample_starts(m, rng, 4):
        v0, v1 = 32 * b0, min(m, 32 * b0 + SLICE)
        refs = [zcref.compress(x[v0:v1].cpu().numpy(), eb)[1] for x in xs]
        st, ref, tot = zcref.reduce(refs)
        assert st == 0
        nbs = (v1 - v0 + 31) // 32
        assert np.array_equal(r.widths[b0:b0 + nbs].cpu().numpy(), ref[32:32 + nbs]), f"widths differ at block {b0}"
        o0 = 32 + pad16(nbs)
        assert np.array_equal(r.outliers[b0:b0 + nbs].cpu().numpy(), ref[o0:o0 + 4 * nbs].view("<i4"))
        assert np.array_equal(r.payload_of(b0, b0 + nbs), ref[tables_end(nbs):tot]), f"payload differs at block {b0}"


def test_ring_rounds_64M(zcref):
    """Three rounds of the ring reduce-scatter at the per-GPU shape of configuration 4 (a chunk
    of 2^26 values): compress rank 0, then add ranks 1..3 uncompressed, one round each.  Every
    round is checked on sampled slices against the reference round applied to the GPU's own
    received stream there, and by its bound; the end result by the N * eb bound of the chain."""
    rng = np.random.default_rng(9)
    xs = _rank_buffers(4)
    m = xs[0].numel()
    eb = float(torch.tensor(2e-4, dtype=torch.float32))
    ws = u8(zc.zc_workspace_bytes(m, 1))
    st, buf, total = compress_async(xs[0], eb, ws)
    assert st == ZC_OK
    cur = Stream(buf, total, m)
    y_prev = torch.empty(m, dtype=torch.float32, device=DEV)
    y_next = torch.empty(m, dtype=torch.float32, device=DEV)
    st, _ = decompress_async(cur.buf, cur.total, y_prev, ws)
    assert st == ZC_OK
    for i in range(1, 4):
        out = u8(zc.zc_compress_bound(m))
        st, _ = zc.zc_reduce_step(cur.buf, cur.total, xs[i], m, out, ws, sync=False)
        assert st == ZC_OK
        st, total = zc.zc_finish(ws)
        assert st == ZC_OK
        nxt = Stream(out, total, m)
        check_header_and_sizes(nxt, eb, nsum=i + 1)
        st, n_out = decompress_async(nxt.buf, nxt.total, y_next, ws)
        assert st == ZC_OK and n_out == m
        given = y_prev + xs[i]                                   # the binary32 sums the round quantises
        assert max_abs_err(given, y_next) <= eb
        del given
        for b0 in sample_starts(m, rng, 3):
            v0, v1 = 32 * b0, min(m, 32 * b0 + SLICE)
            nbs = (v1 - v0 + 31) // 32
            # the received stream of the slice, rebuilt from the GPU stream's own codes
            st, rec, _ = zcref.compress(y_prev[v0:v1].cpu().numpy(), eb)
            assert st == 0
            st, ref, tot = zcref.reduce_step(rec, xs[i][v0:v1].cpu().numpy())
            assert st == 0
            assert np.array_equal(nxt.widths[b0:b0 + nbs].cpu().numpy(), ref[32:32 + nbs]), f"round {i}: widths differ at block {b0}"
            o0 = 32 + pad16(nbs)
            assert np.array_equal(nxt.outliers[b0:b0 + nbs].cpu().numpy(), ref[o0:o0 + 4 * nbs].view("<i4"))
            assert np.array_equal(nxt.payload_of(b0, b0 + nbs), ref[tables_end(nbs):tot]), f"round {i}: payload differs at block {b0}"
        cur = nxt
        y_prev, y_next = y_next, y_prev
    exact = torch.zeros(m, dtype=torch.float64, device=DEV)
    for x in xs:
        exact += x.double()
    assert float((y_prev.double() - exact).abs().max()) <= 4 * eb
    del exact
    # the same ring with Max rounds: the result is the stream of the elementwise maximum compressed once
    st, buf, total = compress_async(xs[0], eb, ws)
    assert st == ZC_OK
    for i in range(1, 4):
        out = u8(zc.zc_compress_bound(m))
        st, _ = zc.zc_reduce_step_op(buf, total, xs[i], m, zc.binding.ZC_OP_MAX, out, ws, sync=False)
        assert st == ZC_OK
        st, total = zc.zc_finish(ws)
        assert st == ZC_OK
        buf = out
    top = torch.maximum(torch.maximum(xs[0], xs[1]), torch.maximum(xs[2], xs[3]))
    st, direct, total_d = compress_async(top, eb, ws)
    assert st == ZC_OK and total_d == total
    assert torch.equal(buf[:20], direct[:20]) and torch.equal(buf[24:total], direct[24:total])      # all but nsum (4 against 1)
    st, _ = decompress_async(buf, total, y_next, ws)
    assert st == ZC_OK and max_abs_err(top, y_next) <= eb


def test_hard_mix_256M(zcref):
    """Configuration 5: steps, spikes and exactly constant blocks at rel 1e-5."""
    rng = np.random.default_rng(5)
    n = 1 << 28
    x = synth.hard_mix(n, seed=0, device=DEV)
    eb = synth.abs_bound(x, 1e-5)
    ws = u8(zc.zc_workspace_bytes(n, 1))
    st, buf, total = compress_async(x, eb, ws)
    assert st == ZC_OK
    s = Stream(buf, total, n)
    check_header_and_sizes(s, eb)
    # exactly constant blocks cost no payload
    xb = x.reshape(-1, 32)
    const_blocks = (xb == xb[:, :1]).all(dim=1)
    assert float(const_blocks.float().mean()) > 0.09
    assert not bool(s.widths[const_blocks].any())
    assert int(s.widths.max()) >= 16          # the spikes make wide blocks
    y = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    st, n_out = decompress_async(buf, total, y, ws)
    assert st == ZC_OK and n_out == n
    assert max_abs_err(x, y) <= eb
    check_slices_against_reference(zcref, x, eb, s, y, rng)


def test_largest_input(zcref):
    """n = 2^31 - 77 (close to the largest size the interface takes, ragged): 64-bit offsets everywhere."""
    rng = np.random.default_rng(6)
    n = (1 << 31) - 77
    x = torch.empty(n, dtype=torch.float32, device=DEV)
    chunk = 1 << 27
    for i in range(0, n, chunk):                   # smooth waves plus small noise, made in chunks
        j = torch.arange(i, min(n, i + chunk), dtype=torch.float64, device=DEV)
        v = torch.sin(j * (2 * np.pi / 1e3)) + torch.sin(j * (2 * np.pi / 1e5)) + 0.5 * torch.sin(j * (2 * np.pi / 7e7))
        x[i:i + j.numel()] = (0.4 * v).to(torch.float32)
        del j, v
    g = torch.Generator(device=DEV)
    g.manual_seed(6)
    for i in range(0, n, chunk):
        m = min(n, i + chunk) - i
        x[i:i + m] += torch.randn(m, device=DEV, generator=g) * 0.08
    eb = float(np.float32(1e-5))                   # widths around 15, a few beyond: the stream exceeds 2^32 bytes
    assert float(x.abs().max()) <= eb * 2 ** 18    # inside the guaranteed domain
    ws = u8(zc.zc_workspace_bytes(n, 1))
    st, buf, total = compress_async(x, eb, ws)
    assert st == ZC_OK
    s = Stream(buf, total, n)
    check_header_and_sizes(s, eb)
    assert total > (1 << 32)
    y = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    st, n_out = decompress_async(buf, total, y, ws)
    assert st == ZC_OK and n_out == n
    assert max_abs_err(x, y) <= eb
    check_slices_against_reference(zcref, x, eb, s, y, rng, count=5)
