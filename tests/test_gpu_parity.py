"""GPU parity: the HIP library, called through its C ABI, against the reference CPU codec on the
same seeded inputs.  Bit-exact on codes, widths, offsets and stream bytes; reconstructed
floats bit-exact (the tolerance allowed is 1 ulp) and within eb of the input."""
import numpy as np
import pytest
import torch

import gpuutil
from gpuutil import zc
from paper_2502_18554_amd import synth
from paper_2502_18554_amd.binding import (ZC_ERR_ARG, ZC_ERR_BOUND, ZC_ERR_CAPACITY, ZC_ERR_FORMAT,
                                           ZC_ERR_MISMATCH, ZC_ERR_NONFINITE, ZC_ERR_RANGE, ZC_OK)

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("stream_variant")]

TILE = 8192


@pytest.fixture(params=["dispatch_order", "tickets"], autouse=True)
def tile_hand_out(request):
    """Every test of this module runs with both ways of handing out tiles to workgroups."""
    gpuutil.set_tickets(request.param == "tickets")
    yield request.param
    gpuutil.set_tickets(False)


def _u():
    import gpuutil
    return gpuutil


def _inputs():
    yield "sin_1M", lambda: synth.sinusoids(1 << 20, seed=0).numpy(), 1e-4          # config 1
    yield "grf_ragged", lambda: synth.power_law_field((24, 64, 64), seed=1).numpy()[: 3 * TILE + 777], 1e-3
    yield "grf_1e-2", lambda: synth.power_law_field((32, 64, 64), seed=2).numpy(), 1e-2
    yield "grf_1e-4", lambda: synth.power_law_field((32, 64, 64), seed=3).numpy(), 1e-4
    yield "hard", lambda: synth.hard_mix(5 * TILE + 4097, seed=4).numpy(), 1e-5


_IDS = [i[0] for i in _inputs()]


@pytest.mark.parametrize("name,make,rel", list(_inputs()), ids=_IDS)
def test_compress_stream_matches_reference(zcref, name, make, rel):
    u = _u()
    x = make()
    eb = synth.abs_bound(torch.from_numpy(x), rel)
    st_ref, s_ref, total_ref = zcref.compress(x, eb)
    # stage 1: quantisation codes
    d_q = torch.empty(x.size, dtype=torch.int32, device=u.DEV)
    st = zc.zc_debug_quantize(u.to_dev(x), x.size, eb, d_q, u.workspace(x.size))
    _, q_ref = zcref.quantize(x, eb)
    assert st == st_ref == ZC_OK
    assert np.array_equal(d_q.cpu().numpy(), q_ref), u.first_diff(d_q.cpu().numpy(), q_ref)
    # stage 2: the stream
    st, s, total = u.gpu_compress(x, eb)
    assert st == ZC_OK and total == total_ref
    nb = (x.size + 31) // 32
    _, _, w_ref, off_ref = zcref.inspect(s_ref)
    assert np.array_equal(u.widths_of(s, nb), w_ref), "widths: " + u.first_diff(u.widths_of(s, nb), w_ref)
    assert s.tobytes() == s_ref.tobytes(), u.first_diff(s, s_ref)
    # stage 3: block offsets recomputed from the stream
    d_off = torch.empty(nb, dtype=torch.int32, device=u.DEV)
    st = zc.zc_debug_block_offsets(u.to_dev(s), s.size, d_off, u.workspace(x.size))
    assert st == ZC_OK
    assert np.array_equal(d_off.cpu().numpy().astype(np.uint64) * 4, off_ref)


@pytest.mark.parametrize("name,make,rel", list(_inputs()), ids=_IDS)
def test_decompress_matches_reference(zcref, name, make, rel):
    u = _u()
    x = make()
    eb = synth.abs_bound(torch.from_numpy(x), rel)
    _, s_ref, _ = zcref.compress(x, eb)
    _, y_ref, _ = zcref.decompress(s_ref)
    st, y, n = u.gpu_decompress(s_ref, x.size)
    assert st == ZC_OK and n == x.size
    assert np.array_equal(y.view(np.uint32), y_ref.view(np.uint32)), u.first_diff(y, y_ref)
    assert np.max(np.abs(y.astype(np.float64) - x.astype(np.float64))) <= eb


@pytest.mark.parametrize("n", [0, 1, 2, 31, 32, 33, 63, 64, 65, 2047, 2048, 2049, 4095, 4096, 4097,
                               TILE - 1, TILE, TILE + 1, 2 * TILE + 31])
def test_edge_sizes_round_trip(zcref, n):
    u = _u()
    rng = np.random.default_rng(n)
    x = np.cumsum(rng.normal(0, 0.01, n)).astype(np.float32)
    eb = 1e-3
    st_ref, s_ref, total_ref = zcref.compress(x, eb)
    st, s, total = u.gpu_compress(x, eb)
    assert st == st_ref == ZC_OK and total == total_ref
    assert s.tobytes() == s_ref.tobytes(), u.first_diff(s, s_ref)
    st, y, m = u.gpu_decompress(s, max(n, 1))
    _, y_ref, _ = zcref.decompress(s_ref)
    assert st == ZC_OK and m == n
    assert np.array_equal(y.view(np.uint32), y_ref.view(np.uint32))


def test_constant_blocks_and_worked_example(zcref):
    u = _u()
    x = np.full(3 * TILE + 5, 3.25, np.float32)
    st, s, total = u.gpu_compress(x, 1e-2)
    nb = (x.size + 31) // 32
    assert st == ZC_OK and total == u.tables_end(nb)
    assert not u.widths_of(s, nb).any()
    assert s.tobytes() == zcref.compress(x, 1e-2)[1].tobytes()
    xw = np.array([10, 11, 13, 12, 12, 12, 9, 10] + [10] * 24, np.float32)
    st, s, total = u.gpu_compress(xw, 0.5)
    assert total == u.tables_end(1) + 12 and s[total - 12:total].tobytes() == bytes.fromhex("48000000CA00000044000000")


def test_wide_widths_and_bound_status(zcref):
    """Widths up to 31 come from inputs outside the guaranteed domain; status and stream must
    still agree with the reference."""
    u = _u()
    rng = np.random.default_rng(7)
    eb = np.float32(2.0 ** -20)
    step = float(eb) * 63 / 32
    scale = np.repeat(2.0 ** rng.integers(0, 30, 4 * TILE // 32), 32)
    q = (rng.uniform(-1, 1, scale.size) * scale).astype(np.int64)
    x = (q * step).astype(np.float32)
    st_ref, s_ref, total_ref = zcref.compress(x, eb)
    st, s, total = u.gpu_compress(x, eb)
    assert st == st_ref and st in (ZC_OK, ZC_ERR_BOUND) and total == total_ref
    assert s.tobytes() == s_ref.tobytes(), u.first_diff(s, s_ref)
    assert zcref.inspect(s_ref)[2].max() >= 28
    st, y, n = u.gpu_decompress(s_ref, x.size)
    assert np.array_equal(y.view(np.uint32), zcref.decompress(s_ref)[1].view(np.uint32))
    # streams that only the encode-from-codes helper can make: every block at width 31
    q = np.tile(np.array([-(2 ** 30) + 1, 2 ** 30 - 1], np.int32), 16 * 300)
    q[::7] //= 3
    _, s31, _ = zcref.encode_codes(q, 1e-3)
    st, y, n = u.gpu_decompress(s31, q.size)
    assert st == ZC_OK and np.array_equal(y.view(np.uint32), zcref.decompress(s31)[1].view(np.uint32))
    # the status screen: values around 2^17 eb and 2^18 eb, inside and outside the domain
    eb2 = np.float32(8.8 * 2.0 ** -23)
    x2 = np.linspace(1.0, 2.0, 50000).astype(np.float32)
    st_ref, s_ref, _ = zcref.compress(x2, eb2)
    st, s, _ = u.gpu_compress(x2, eb2)
    assert st == st_ref == ZC_ERR_BOUND and s.tobytes() == s_ref.tobytes()
    for top in (2.0 ** 17, 2.0 ** 17 * 1.001, 2.0 ** 18, 2.0 ** 19):
        x3 = (np.linspace(-1, 1, 3 * TILE + 3) * top * 1e-3).astype(np.float32)
        st_ref, s_ref, _ = zcref.compress(x3, 1e-3)
        st, s, _ = u.gpu_compress(x3, 1e-3)
        assert st == st_ref and s.tobytes() == s_ref.tobytes()


def test_ties_and_signed_zero(zcref):
    u = _u()
    step = 0.5 * 63 / 32
    m = np.arange(-4000, 4001)
    x = ((m + 0.5) * step).astype(np.float32)
    x = np.concatenate([x, np.array([-0.0, 0.0, 1e-40, -1e-40], np.float32)])
    st_ref, s_ref, _ = zcref.compress(x, 0.5)
    st, s, _ = u.gpu_compress(x, 0.5)
    assert st == st_ref == ZC_OK and s.tobytes() == s_ref.tobytes()
    st, y, _ = u.gpu_decompress(s, x.size)
    assert np.array_equal(y.view(np.uint32), zcref.decompress(s_ref)[1].view(np.uint32))


def test_compress_error_paths(zcref):
    u = _u()
    x = np.linspace(0, 1, 3 * TILE).astype(np.float32)
    for bad in (0.0, -1.0, float("inf"), float("nan"), 2.0 ** -97):
        assert u.gpu_compress(x, bad)[0] == ZC_ERR_ARG
    y = x.copy(); y[TILE + 7] = np.nan
    assert u.gpu_compress(y, 1e-3)[0] == ZC_ERR_NONFINITE == zcref.compress(y, 1e-3)[0]
    y[TILE + 7] = -np.inf
    assert u.gpu_compress(y, 1e-3)[0] == ZC_ERR_NONFINITE
    y[TILE + 7] = 3e6
    assert u.gpu_compress(y, 1e-3)[0] == ZC_ERR_RANGE == zcref.compress(y, 1e-3)[0]
    y[9] = np.nan
    assert u.gpu_compress(y, 1e-3)[0] == ZC_ERR_NONFINITE
    st_ref, s_ref, total = zcref.compress(x, 1e-5)
    for cap in (total - 1, total - 4, 40, 0, 16):
        st, _, need = u.gpu_compress(x, 1e-5, out_cap=cap)
        assert st == ZC_ERR_CAPACITY and need == total
    # nothing is written past out_cap
    d_in = u.to_dev(x)
    d_out = torch.full((total + 64,), 0xA5, dtype=torch.uint8, device=u.DEV)
    cap = total - 4096
    st, need = zc.zc_compress(d_in, x.size, 1e-5, d_out[:cap], u.workspace(x.size))
    assert st == ZC_ERR_CAPACITY and need == total
    assert bool((d_out[cap:] == 0xA5).all())
    st, _, _ = u.gpu_compress(x, 1e-5, ws=torch.empty(64, dtype=torch.uint8, device=u.DEV))
    assert st == ZC_ERR_ARG                      # workspace too small


def test_decompress_error_paths(zcref):
    u = _u()
    x = np.linspace(0, 1, 2 * TILE + 100).astype(np.float32)
    _, s, total = zcref.compress(x, 1e-4)
    assert u.gpu_decompress(s[:16], x.size)[0] == ZC_ERR_FORMAT
    assert u.gpu_decompress(s[:-1], x.size)[0] == ZC_ERR_FORMAT == zcref.decompress(s[:-1])[0]
    for pos in (0, 4, 6, 7):
        t = s.copy(); t[pos] ^= 4
        assert u.gpu_decompress(t, x.size)[0] == ZC_ERR_FORMAT == zcref.decompress(t)[0]
    w0 = u.widths_begin((x.size + 31) // 32)
    t = s.copy(); t[w0 + 300] = 32
    assert u.gpu_decompress(t, x.size)[0] == ZC_ERR_FORMAT == zcref.decompress(t)[0]
    t = s.copy(); t[w0 + 300] ^= 1
    assert u.gpu_decompress(t, x.size)[0] == ZC_ERR_FORMAT == zcref.decompress(t)[0]
    t = s.copy(); t[20:24] = 0
    assert u.gpu_decompress(t, x.size)[0] == ZC_ERR_FORMAT
    t = s.copy(); t[16:20] = 0
    assert u.gpu_decompress(t, x.size)[0] == ZC_ERR_FORMAT
    st, _, n = u.gpu_decompress(s, x.size - 1)
    assert st == ZC_ERR_CAPACITY and n == x.size
    longer = np.concatenate([s, np.zeros(7, np.uint8)])
    st, y, n = u.gpu_decompress(longer, x.size + 1000)
    assert st == ZC_OK and n == x.size and np.array_equal(y, zcref.decompress(s)[1])
    st, h_n, h_eb, h_nsum, h_total, h_flags = zc.zc_peek_header(u.to_dev(s), s.size)
    assert (st, h_n, h_nsum, h_total) == (ZC_OK, x.size, 1, total) and h_eb == np.float32(1e-4)


def _rank_streams(zcref, k, n, rel, seed0):
    xs = [synth.power_law_field((n // 4096, 64, 64), seed=seed0 + i).numpy()[:n] for i in range(k)]
    eb = synth.abs_bound(torch.from_numpy(xs[0]), rel)
    streams = [zcref.compress(x, eb)[1] for x in xs]
    return xs, eb, streams


@pytest.mark.parametrize("k,n", [(1, 4096 * 4), (2, 4096 * 4 - 37), (3, 4096 * 9 + 1), (8, 4096 * 16), (17, 4096 * 3 + 5)])
def test_reduce_stream_matches_reference(zcref, k, n):
    u = _u()
    xs, eb, streams = _rank_streams(zcref, k, (n + 4095) // 4096 * 4096, 1e-4, seed0=20)
    xs = [x[:n] for x in xs]
    streams = [zcref.compress(x, eb)[1] for x in xs]
    st_ref, r_ref, total_ref = zcref.reduce(streams)
    st, r, total = u.gpu_reduce(streams, n)
    assert st == st_ref == ZC_OK and total == total_ref
    assert r.tobytes() == r_ref.tobytes(), u.first_diff(r, r_ref)
    st, y, _ = u.gpu_decompress(r, n)
    exact = np.sum([x.astype(np.float64) for x in xs], axis=0)
    assert np.max(np.abs(y.astype(np.float64) - exact)) <= k * eb
    assert int(r[20:24].view("<u4")[0]) == k
    # nested reduce on the GPU gives the flat result
    if k >= 3:
        _, a, _ = u.gpu_reduce(streams[:2], n)
        _, b, _ = u.gpu_reduce(streams[2:], n)
        _, ab, _ = u.gpu_reduce([a, b], n)
        assert ab.tobytes() == r_ref.tobytes()


def test_reduce_wide_and_cancelling_operands(zcref):
    u = _u()
    rng = np.random.default_rng(11)
    n = 3 * TILE + 77
    scale = np.repeat(2.0 ** rng.integers(0, 27, (n + 31) // 32), 32)[:n]
    qs = [(rng.uniform(-1, 1, n) * scale).astype(np.int32) for _ in range(5)]
    qs.append(-qs[0])                                 # exact cancellation with operand 0
    qs.append(np.zeros(n, np.int32))                  # all-constant operand
    streams = [zcref.encode_codes(q, 1e-3)[1] for q in qs]
    st_ref, r_ref, total_ref = zcref.reduce(streams)
    st, r, total = u.gpu_reduce(streams, n)
    assert st == st_ref == ZC_OK and total == total_ref
    assert r.tobytes() == r_ref.tobytes(), u.first_diff(r, r_ref)
    # everything cancels: all widths zero
    st, r, total = u.gpu_reduce([streams[0], streams[5]], n)
    assert st == ZC_OK and r.tobytes() == zcref.reduce([streams[0], streams[5]])[1].tobytes()
    assert not u.widths_of(r, (n + 31) // 32).any()


@pytest.mark.parametrize("k", [2, 9, 64])
def test_reduce_narrow_widths_all_classes(zcref, k):
    """Every block at most 15 bits wide (the staged kernel), widths 0..15 mixed inside each wave, up to 64 operands."""
    u = _u()
    rng = np.random.default_rng(100 + k)
    n = 5 * TILE + 45
    nb = (n + 31) // 32
    qs = []
    for i in range(k):
        scale = np.repeat(2.0 ** rng.integers(-2, 14, nb), 32)[:n]       # |code| < 2^13: |delta| < 2^14
        q = (rng.uniform(-1, 1, n) * scale).astype(np.int32)
        if i % 5 == 4:
            q[: n // 2] = 7                                              # long runs of constant blocks
        qs.append(q)
    qs[1] = -qs[0]                                                       # exact cancellation
    # extreme deltas of the class: +-(2^15 - 1) next to each other, all operands in phase
    for q in qs[2:]:
        q[64:96:2] = 2 ** 14 - 1
        q[65:96:2] = -(2 ** 14)
    streams = [zcref.encode_codes(q, 1e-3)[1] for q in qs]
    assert max(int(u.widths_of(s, nb).max()) for s in streams) <= 15
    st_ref, r_ref, total_ref = zcref.reduce(streams)
    st, r, total = u.gpu_reduce(streams, n)
    assert st == st_ref == ZC_OK and total == total_ref
    assert r.tobytes() == r_ref.tobytes(), u.first_diff(r, r_ref)


def test_reduce_error_paths(zcref):
    u = _u()
    xs, eb, streams = _rank_streams(zcref, 2, 4096 * 3, 1e-3, seed0=30)
    n = xs[0].size
    _, other, _ = zcref.compress(xs[0], eb * 2)
    assert u.gpu_reduce([streams[0], other], n)[0] == ZC_ERR_MISMATCH == zcref.reduce([streams[0], other])[0]
    _, short, _ = zcref.compress(xs[0][:-32], eb)
    assert u.gpu_reduce([streams[0], short], n)[0] == ZC_ERR_MISMATCH
    bad = streams[1].copy(); bad[0] ^= 1
    assert u.gpu_reduce([streams[0], bad], n)[0] == ZC_ERR_FORMAT
    assert u.gpu_reduce([streams[0], bad, other], n)[0] == ZC_ERR_FORMAT      # precedence
    big = np.full(TILE + 64, 2 ** 30 - 1, np.int32)
    big[TILE:] = 5
    _, sb, _ = zcref.encode_codes(big, eb)
    assert u.gpu_reduce([sb, sb], big.size)[0] == ZC_ERR_RANGE == zcref.reduce([sb, sb])[0]
    assert u.gpu_reduce([sb], big.size)[0] == ZC_OK
    # a block whose outlier is fine but whose chain runs out of range
    ramp = np.zeros(TILE, np.int32); ramp[40:] = 2 ** 29 + 5
    _, sr, _ = zcref.encode_codes(ramp, eb)
    assert u.gpu_reduce([sr, sr], ramp.size)[0] == ZC_ERR_RANGE == zcref.reduce([sr, sr])[0]
    # near the limit but inside: exact check must accept
    ok = np.zeros(TILE, np.int32); ok[40:] = 2 ** 29 - 1
    _, so, _ = zcref.encode_codes(ok, eb)
    st, r, _ = u.gpu_reduce([so, so], ok.size)
    assert st == ZC_OK and r.tobytes() == zcref.reduce([so, so])[1].tobytes()
    st_ref, r_ref, total = zcref.reduce(streams)
    st, _, need = u.gpu_reduce(streams, n, out_cap=total - 4)
    assert st == ZC_ERR_CAPACITY and need == total
    assert u.gpu_reduce([], n)[0] == ZC_ERR_ARG


# ---------------- k streams decompressed in one call ----------------
def test_decompress_many_matches_reference(zcref):
    """Streams of different lengths and bounds (one of them empty, one with wide blocks) in one
    call: every output equals the reference decompression of its stream, bit for bit."""
    u = _u()
    rng = np.random.default_rng(21)
    sizes = [4 * TILE + 5, 1, 0, 7 * TILE, 33, 2 * TILE - 1, 3 * TILE + 2048]
    rels = [1e-3, 1e-2, 1e-3, 1e-4, 1e-3, 1e-5, 1e-2]
    streams, wants = [], []
    for i, (n, rel) in enumerate(zip(sizes, rels)):
        x = synth.power_law_field((8, 64, 128), seed=80 + i).numpy().ravel()[:n]
        st, s, _ = zcref.compress(x, 2 * rel)               # the fields span about [-1, 1]
        assert st == ZC_OK
        streams.append(s); wants.append(zcref.decompress(s)[1])
    q = (rng.uniform(-1, 1, 2 * TILE) * 2.0 ** rng.integers(0, 29, 2 * TILE)).astype(np.int32)
    _, wide, _ = zcref.encode_codes(q, 1e-3)
    streams.append(wide); wants.append(zcref.decompress(wide)[1]); sizes.append(q.size)
    st, outs, ns = u.gpu_decompress_many(streams, sizes)
    assert st == ZC_OK and ns == sizes
    for i, (o, w) in enumerate(zip(outs, wants)):
        assert np.array_equal(o[: sizes[i]].view(np.uint32), w.view(np.uint32)), (i, u.first_diff(o[: sizes[i]], w))
    # one call with a single stream is zc_decompress
    st, outs, ns = u.gpu_decompress_many(streams[:1], sizes[:1])
    assert st == ZC_OK and np.array_equal(outs[0][: sizes[0]].view(np.uint32), wants[0].view(np.uint32))


def test_decompress_many_error_paths(zcref):
    u = _u()
    xs = [synth.power_law_field((2, 64, 64), seed=90 + i).numpy().ravel() for i in range(3)]
    streams = [zcref.compress(x, 1e-3)[1] for x in xs]
    n = xs[0].size
    # too little room for stream 1: CAPACITY, the others are decoded
    st, outs, ns = u.gpu_decompress_many(streams, [n, n - 1, n])
    assert st == ZC_ERR_CAPACITY and ns == [n, n, n]
    for i in (0, 2):
        assert np.array_equal(outs[i][:n].view(np.uint32), zcref.decompress(streams[i])[1].view(np.uint32))
    assert np.isnan(outs[1]).all()
    bad = streams[2].copy(); bad[4] ^= 4
    st, outs, _ = u.gpu_decompress_many([streams[0], bad], [n, n])
    assert st == ZC_ERR_FORMAT and np.isnan(outs[0]).all()
    ws = u.workspace(n, 3)
    d_chunks = [u.to_dev(s) for s in streams]
    d_outs = [torch.empty(n, dtype=torch.float32, device=u.DEV) for _ in streams]
    st, _ = zc.zc_decompress_many(d_chunks, [c.numel() for c in d_chunks], d_outs, ws, sync=False)
    assert st == ZC_OK
    st, total = zc.zc_finish(ws)
    assert st == ZC_OK and total == 3 * n
    for o, s in zip(d_outs, streams):
        assert np.array_equal(o.cpu().numpy().view(np.uint32), zcref.decompress(s)[1].view(np.uint32))


# ---------------- one ring round: received stream + local values -> stream of the sums ----------------
@pytest.mark.parametrize("n,rel", [(1, 1e-3), (31, 1e-3), (32, 1e-3), (33, 1e-3), (2048, 1e-2), (TILE, 1e-4), (TILE + 1, 1e-3),
                                   (3 * TILE + 777, 1e-3), (16 * TILE, 1e-4), (9 * TILE - 5, 1e-5)])
def test_reduce_step_stream_matches_reference(zcref, n, rel):
    u = _u()
    x = synth.power_law_field((max(1, (n + 4095) // 4096), 64, 64), seed=40).numpy().ravel()[:n]
    y = synth.power_law_field((max(1, (n + 4095) // 4096), 64, 64), seed=41).numpy().ravel()[:n]
    eb = synth.abs_bound(torch.from_numpy(np.concatenate([x, [1.0]]).astype(np.float32)), rel)
    _, received, _ = zcref.compress(x, eb)
    st_ref, s_ref, total_ref = zcref.reduce_step(received, y)
    st, s, total = u.gpu_reduce_step(received, y)
    assert st == st_ref == ZC_OK and total == total_ref
    assert s.tobytes() == s_ref.tobytes(), u.first_diff(s, s_ref)


def test_reduce_step_chain_and_special_cases(zcref):
    """N rounds in a row on the GPU against N rounds of the reference; adding zeros keeps the
    stream, adding to zeros compresses the local chunk."""
    u = _u()
    n = 5 * TILE + 321
    xs = [synth.power_law_field((8, 64, 128), seed=50 + i).numpy().ravel()[:n] for i in range(5)]
    eb = synth.abs_bound(torch.from_numpy(xs[0]), 1e-3)
    _, s_ref, _ = zcref.compress(xs[0], eb)
    s = s_ref
    for i in range(1, 5):
        _, s_ref, _ = zcref.reduce_step(s_ref, xs[i])
        st, s, _ = u.gpu_reduce_step(s, xs[i])
        assert st == ZC_OK and s.tobytes() == s_ref.tobytes(), (i, u.first_diff(s, s_ref))
    exact = np.sum([x.astype(np.float64) for x in xs], axis=0)
    _, yv, _ = u.gpu_decompress(s, n)
    assert np.abs(yv.astype(np.float64) - exact).max() <= 5 * eb
    st, same, _ = u.gpu_reduce_step(s, np.zeros(n, np.float32))
    want = s.copy(); want[20:24] = np.frombuffer(np.uint32(6).tobytes(), np.uint8)
    assert st == ZC_OK and same.tobytes() == want.tobytes()
    _, zeros, _ = zcref.compress(np.zeros(n, np.float32), eb)
    st, fresh, _ = u.gpu_reduce_step(zeros, xs[1])
    _, want, _ = zcref.compress(xs[1], eb)
    want = want.copy(); want[20:24] = np.frombuffer(np.uint32(2).tobytes(), np.uint8)
    assert st == ZC_OK and fresh.tobytes() == want.tobytes()


def test_reduce_step_wide_and_out_of_domain(zcref):
    """Received streams and sums with blocks wider than 15 bits, constant blocks, values that
    need the checked quantiser, and sums that leave the guaranteed domain (BOUND)."""
    u = _u()
    rng = np.random.default_rng(11)
    eb = np.float32(2.0 ** -20)
    step = float(eb) * 63 / 32
    n = 4 * TILE + 100
    scale = np.repeat(2.0 ** rng.integers(0, 28, (n + 31) // 32), 32)[:n]
    q = (rng.uniform(-1, 1, n) * scale).astype(np.int64)
    q[:TILE] = 7                                                   # constant blocks
    _, received, _ = zcref.encode_codes(q.astype(np.int32), eb)
    local = (rng.uniform(-1, 1, n) * np.roll(scale, 4096) * step).astype(np.float32)
    local[TILE // 2: TILE] = 0.0
    st_ref, s_ref, total_ref = zcref.reduce_step(received, local)
    st, s, total = u.gpu_reduce_step(received, local)
    assert st == st_ref and st in (ZC_OK, ZC_ERR_BOUND) and total == total_ref
    assert s.tobytes() == s_ref.tobytes(), u.first_diff(s, s_ref)
    assert zcref.inspect(s_ref)[2].max() >= 24
    # narrow received stream, wide sums
    x = synth.power_law_field((4, 64, 64), seed=60).numpy().ravel()
    eb2 = synth.abs_bound(torch.from_numpy(x), 1e-4)
    _, rec2, _ = zcref.compress(x, eb2)
    loc2 = (rng.standard_normal(x.size) * 3000).astype(np.float32)
    st_ref, s_ref, _ = zcref.reduce_step(rec2, loc2)
    st, s, _ = u.gpu_reduce_step(rec2, loc2)
    assert st == st_ref and s.tobytes() == s_ref.tobytes(), u.first_diff(s, s_ref)
    assert zcref.inspect(s_ref)[2].max() > 15


def test_reduce_step_error_paths(zcref):
    u = _u()
    x = synth.power_law_field((3, 64, 64), seed=70).numpy().ravel()
    n = x.size
    eb = synth.abs_bound(torch.from_numpy(x), 1e-3)
    _, s, _ = zcref.compress(x, eb)
    assert u.gpu_reduce_step(s, x[:-1])[0] == ZC_ERR_MISMATCH == zcref.reduce_step(s, x[:-1])[0]
    bad = s.copy(); bad[0] ^= 1
    assert u.gpu_reduce_step(bad, x)[0] == ZC_ERR_FORMAT
    y = x.copy(); y[5000] = np.inf
    assert u.gpu_reduce_step(s, y)[0] == ZC_ERR_NONFINITE == zcref.reduce_step(s, y)[0]
    y = x.copy(); y[5000] = np.float32(eb * 2.0 ** 32)
    assert u.gpu_reduce_step(s, y)[0] == ZC_ERR_RANGE == zcref.reduce_step(s, y)[0]
    y[77] = np.nan                                                  # precedence: NONFINITE before RANGE
    assert u.gpu_reduce_step(s, y)[0] == ZC_ERR_NONFINITE == zcref.reduce_step(s, y)[0]
    _, _, total = zcref.reduce_step(s, x)
    st, _, need = u.gpu_reduce_step(s, x, out_cap=total - 4)
    assert st == ZC_ERR_CAPACITY and need == total
    st, _, _ = u.gpu_reduce_step(s, x, out_cap=16)
    assert st == ZC_ERR_CAPACITY
    # empty input
    _, s0, _ = zcref.compress(np.zeros(0, np.float32), eb)
    st, r0, total0 = u.gpu_reduce_step(s0, np.zeros(0, np.float32))
    st_ref, r_ref, _ = zcref.reduce_step(s0, np.zeros(0, np.float32))
    assert st == st_ref == ZC_OK and r0.tobytes() == r_ref.tobytes()


def test_async_form_and_workspace_reuse(zcref):
    u = _u()
    x = synth.power_law_field((8, 64, 64), seed=5).numpy()
    eb = synth.abs_bound(torch.from_numpy(x), 1e-3)
    _, s_ref, total_ref = zcref.compress(x, eb)
    d_in = u.to_dev(x)
    d_out = torch.empty(zc.zc_compress_bound(x.size), dtype=torch.uint8, device=u.DEV)
    ws = u.workspace(x.size)
    ws.fill_(0xFF)                                     # stale workspace content must not matter
    for _ in range(3):
        st, none = zc.zc_compress(d_in, x.size, eb, d_out, ws, sync=False)
        assert st == ZC_OK and none is None
        st, total = zc.zc_finish(ws)
        assert st == ZC_OK and total == total_ref
        assert d_out[:total].cpu().numpy().tobytes() == s_ref.tobytes()
    d_y = torch.empty(x.size, dtype=torch.float32, device=u.DEV)
    st, _ = zc.zc_decompress(d_out, total_ref, d_y, ws, sync=False)
    st, n = zc.zc_finish(ws)
    assert st == ZC_OK and n == x.size
    assert np.array_equal(d_y.cpu().numpy(), zcref.decompress(s_ref)[1])


@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 1023, 1024, 4 * TILE + 3, (1 << 22) + 1])
def test_quality_sums_match_reference(zcref, n):
    """Max error, min and max are exact; the sum of squares is accumulated in binary64 in another
    order than the reference's, so it agrees to rounding (n * 2^-53 relative at worst)."""
    u = _u()
    rng = np.random.default_rng(n)
    ref = rng.uniform(-2, 3, n).astype(np.float32)
    test = (ref + rng.normal(0, 1e-3, n)).astype(np.float32)
    st_ref, want = zcref.quality(ref, test)
    d_ref = u.to_dev(ref) if n else torch.zeros(4, device=u.DEV)
    d_test = u.to_dev(test) if n else torch.zeros(4, device=u.DEV)
    st, got = zc.zc_quality(d_ref, d_test, n, u.workspace(max(n, 1)))
    assert st == st_ref == ZC_OK
    assert got[0] == want["max_err"] and got[2] == want["min"] and got[3] == want["max"]
    assert got[1] == want["sse"] or abs(got[1] / want["sse"] - 1) <= max(n, 1) * 2.0 ** -53
    st, again = zc.zc_quality(d_ref, d_test, n, u.workspace(max(n, 1)))
    assert again == got                                              # fixed order: same bits every run
    if n > 4:
        test[n // 2] = np.nan
        st, got = zc.zc_quality(d_ref, u.to_dev(test), n, u.workspace(n))
        assert st == ZC_OK and np.isnan(got[0]) and np.isnan(zcref.quality(ref, test)[1]["max_err"])
    assert zc.zc_quality(d_ref, None, 8, u.workspace(8))[0] == ZC_ERR_ARG


def test_hip_graph_replay(zcref):
    """The asynchronous forms only launch kernels (nothing is cleared with a memset, nothing
    synchronises), so a sequence of calls can be captured into a HIP graph.  Every replay, with
    eager calls and synchronisations in between, must reproduce the eager results bit for bit."""
    u = _u()
    k, n = 3, 6 * TILE + 123
    xs = [u.to_dev(synth.power_law_field((8, 64, 128), seed=110 + i).numpy().ravel()[:n]) for i in range(k)]
    eb = 2e-3
    cap = zc.zc_compress_bound(n)
    fixed, sizes = [], []
    ws0 = u.workspace(n, k)
    for x in xs:                                             # operand streams, made once
        buf = torch.empty(cap, dtype=torch.uint8, device=u.DEV)
        st, total = zc.zc_compress(x, n, eb, buf, ws0)
        assert st == ZC_OK
        fixed.append(buf); sizes.append(total)
    out_c = torch.empty(cap, dtype=torch.uint8, device=u.DEV)
    out_y = torch.empty(n, dtype=torch.float32, device=u.DEV)
    out_r = torch.empty(cap, dtype=torch.uint8, device=u.DEV)
    out_s = torch.empty(cap, dtype=torch.uint8, device=u.DEV)
    out_m = [torch.empty(n, dtype=torch.float32, device=u.DEV) for _ in range(k)]
    wss = [u.workspace(n, k) for _ in range(5)]

    def calls():
        zc.zc_compress(xs[0], n, eb, out_c, wss[0], sync=False)
        zc.zc_decompress(fixed[1], sizes[1], out_y, wss[1], sync=False)
        zc.zc_reduce_compressed(fixed, sizes, out_r, wss[2], sync=False)
        zc.zc_reduce_step(fixed[2], sizes[2], xs[0], n, out_s, wss[3], sync=False)
        zc.zc_decompress_many(fixed, sizes, out_m, wss[4], sync=False)

    def results():
        torch.cuda.synchronize()
        res = []
        for w in wss:
            st, r = zc.zc_finish(w)
            assert st == ZC_OK
            res.append(r)
        outs = [out_c[: res[0]], out_y, out_r[: res[2]], out_s[: res[3]]] + out_m
        return res, [o.clone() for o in outs]

    calls()
    want_res, want = results()
    assert want[0].cpu().numpy().tobytes() == zcref.compress(xs[0].cpu().numpy(), eb)[1].tobytes()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        calls()
    for rep in range(3):
        for o in [out_c, out_r, out_s]:
            o.fill_(0x11)
        for o in [out_y] + out_m:
            o.fill_(float("nan"))
        st, _ = zc.zc_compress(xs[1], n, eb, torch.empty(cap, dtype=torch.uint8, device=u.DEV), ws0)   # eager work in between
        assert st == ZC_OK
        torch.cuda.synchronize()
        g.replay()
        got_res, got = results()
        assert got_res == want_res, rep
        for i, (a, b) in enumerate(zip(got, want)):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), (rep, i)


def test_repeated_runs_are_identical():
    """The look-back scan is the only cross-workgroup protocol: many tiles, many runs, one answer."""
    u = _u()
    x = synth.hard_mix(1 << 22, seed=6, device=u.DEV)
    eb = synth.abs_bound(x, 1e-5)
    d_out = torch.empty(zc.zc_compress_bound(x.numel()), dtype=torch.uint8, device=u.DEV)
    ws = u.workspace(x.numel())
    first = None
    for _ in range(20):
        st, total = zc.zc_compress(x, x.numel(), eb, d_out, ws)
        assert st == ZC_OK
        got = d_out[:total].clone()
        if first is None:
            first = got
        assert torch.equal(first, got)


def test_kernel_timing_hook(zcref):
    """zc_profile_enable / zc_profile_collect: one positive time per main kernel, in call order."""
    u = _u()
    x = synth.power_law_field((16, 64, 64), seed=9).numpy()
    eb = synth.abs_bound(torch.from_numpy(x), 1e-3)
    zc.zc_profile_enable(True)
    st, s, total = u.gpu_compress(x, eb)
    st2, y, n = u.gpu_decompress(s, x.size)
    st3, r, _ = u.gpu_reduce([s, s], x.size)
    got = zc.zc_profile_collect()
    zc.zc_profile_enable(False)
    assert st == st2 == st3 == ZC_OK
    assert [name for name, _ in got] == ["compress", "decompress", "reduce"]
    assert all(0.0 < ms < 100.0 for _, ms in got)
    assert zc.zc_profile_collect() == []
    # a chosen kind only
    zc.zc_profile_enable(True, only=("reduce",))
    u.gpu_compress(x, eb)
    u.gpu_reduce([s, s], x.size)
    u.gpu_decompress(s, x.size)
    u.gpu_reduce([s, s, s], x.size)
    got = zc.zc_profile_collect()
    zc.zc_profile_enable(False)
    assert [name for name, _ in got] == ["reduce", "reduce"] and all(0.0 < ms < 100.0 for _, ms in got)
    u.gpu_reduce([s, s], x.size)
    assert zc.zc_profile_collect() == []


# ---------------- the index of indexed streams is checked by the kernels that use it ----------------
def _all_consumers(u, zcref, bad, good, x):
    """Status of every call that reads `bad` (a stream of x.size values), GPU and reference side by side."""
    n = x.size
    yield "decompress", u.gpu_decompress(bad, n)[0], zcref.decompress(bad)[0]
    yield "decompress_many", u.gpu_decompress_many([good, bad, good], [n, n, n])[0], zcref.decompress(bad)[0]
    yield "reduce operand 0", u.gpu_reduce([bad, good], n)[0], zcref.reduce([bad, good])[0]
    yield "reduce operand 2", u.gpu_reduce([good, good, bad], n)[0], zcref.reduce([good, good, bad])[0]
    yield "reduce_step", u.gpu_reduce_step(bad, x)[0], zcref.reduce_step(bad, x)[0]


def test_indexed_stream_index_is_validated(zcref, stream_variant):
    if stream_variant != "indexed":
        pytest.skip("plain streams have no index")
    u = _u()
    x = synth.power_law_field((5, 64, 64), seed=120).numpy().ravel()[:5 * 4096 - 37]
    eb = synth.abs_bound(torch.from_numpy(x), 1e-3)
    _, s, total = zcref.compress(x, eb)
    nseg = ((x.size + 31) // 32 + 63) // 64
    ix = s[32:32 + 4 * (nseg + 1)].view("<u4")
    assert nseg == 10 and ix[0] == 0 and np.all(np.diff(ix.astype(np.int64)) > 0)
    for name, st, st_ref in _all_consumers(u, zcref, s, s, x):
        assert st == st_ref == ZC_OK, name

    def broken(edit):
        t = s.copy()
        edit(t[32:32 + 4 * (nseg + 1)].view("<u4"))
        return t

    cases = {
        "first entry": lambda e: e.__setitem__(0, 4),
        "entry 1 up": lambda e: e.__setitem__(1, e[1] + 1),
        "entry 5 down": lambda e: e.__setitem__(5, e[5] - 4),
        "entry 7 far": lambda e: e.__setitem__(7, e[7] ^ 0x80000000),
        "last segment": lambda e: e.__setitem__(nseg - 1, e[nseg - 1] + 4),
        "closing entry": lambda e: e.__setitem__(nseg, e[nseg] + 4),
        "entries 3 and 4 shifted alike": lambda e: (e.__setitem__(3, e[3] + 4), e.__setitem__(4, e[4] + 4)),
        "all zero": lambda e: e.fill(0),
    }
    for what, edit in cases.items():
        t = broken(edit)
        for name, st, st_ref in _all_consumers(u, zcref, t, s, x):
            assert st == st_ref == ZC_ERR_FORMAT, f"{what}: {name}: {st} vs {st_ref}"
    # width bytes that do not fit the stream's promise
    nb = (x.size + 31) // 32
    w0 = u.widths_begin(nb)
    for pos, val in ((w0 + 70, 16), (w0 + 300, 32), (w0 + nb - 1, 255)):
        t = s.copy(); t[pos] = val
        for name, st, st_ref in _all_consumers(u, zcref, t, s, x):
            assert st == st_ref == ZC_ERR_FORMAT, f"width {val}: {name}: {st} vs {st_ref}"


def test_indexed_version_word(zcref, stream_variant):
    if stream_variant != "indexed":
        pytest.skip("plain streams are version 1")
    u = _u()
    n = 3 * TILE + 11
    rng = np.random.default_rng(121)
    q = np.cumsum(rng.integers(-40, 41, n)).astype(np.int32)
    _, narrow, _ = zcref.encode_codes(q, 1e-3)
    q2 = q.copy(); q2[2 * TILE + 5] += 1 << 20                   # one block of 21 bits in the last tile
    _, wide, _ = zcref.encode_codes(q2, 1e-3)
    assert narrow[4] == 2 and wide[4] == 3
    x = zcref.decompress(narrow)[1]
    # the GPU writes the same version words: a stream is wide iff one of its tiles is
    for qq, ref in ((q, narrow), (q2, wide)):
        xx = zcref.decompress(ref)[1]
        st, s, _ = u.gpu_compress(xx, 1e-3)
        assert st in (ZC_OK, ZC_ERR_BOUND) and s.tobytes() == ref.tobytes(), u.first_diff(s, ref)
    # "may hold wide blocks" without one is accepted, and what is written says what is in it
    t = narrow.copy(); t[4] = 3
    for name, st, st_ref in _all_consumers(u, zcref, t, narrow, x):
        assert st == st_ref == ZC_OK, name
    st, r, _ = u.gpu_reduce([t, narrow], n)
    assert r.tobytes() == zcref.reduce([t, narrow])[1].tobytes() and r[4] == 2
    st, r, _ = u.gpu_reduce_step(t, x)
    assert r.tobytes() == zcref.reduce_step(t, x)[1].tobytes()
    # "no wide block" with one is refused
    t = wide.copy(); t[4] = 2
    xw = zcref.decompress(wide)[1]
    for name, st, st_ref in _all_consumers(u, zcref, t, wide, xw):
        assert st == st_ref == ZC_ERR_FORMAT, name
    # a plain stream is refused, and the other way round
    u.set_variant(zcref, False)
    _, plain, _ = zcref.encode_codes(q, 1e-3)
    assert u.gpu_decompress(narrow, n)[0] == ZC_ERR_FORMAT == zcref.decompress(narrow)[0]
    u.set_variant(zcref, True)
    assert u.gpu_decompress(plain, n)[0] == ZC_ERR_FORMAT == zcref.decompress(plain)[0]
    assert u.gpu_reduce([narrow, plain], n)[0] == ZC_ERR_FORMAT == zcref.reduce([narrow, plain])[0]


@pytest.mark.parametrize("tail", [1, 11, 31])
def test_wide_block_in_the_ragged_last_tile(zcref, tail):
    """The last block's padding repeats its last code, also in a tile that holds a block wider than 15 bits."""
    u = _u()
    n = 2 * TILE + 5 * 32 + tail
    rng = np.random.default_rng(122 + tail)
    q = np.cumsum(rng.integers(-40, 41, n)).astype(np.int32)
    q[2 * TILE + 40] += 1 << 20
    _, ref, _ = zcref.encode_codes(q, 1e-3)
    x = zcref.decompress(ref)[1]
    assert zcref.compress(x, 1e-3)[1].tobytes() == ref.tobytes()
    st, s, _ = u.gpu_compress(x, 1e-3)
    assert st == zcref.compress(x, 1e-3)[0] and s.tobytes() == ref.tobytes(), u.first_diff(s, ref)


# ---------------- the other aggregation functions: Max, Min (ring round) and Average (decompress) ----------------
@pytest.mark.parametrize("n,rel", [(1, 1e-3), (33, 1e-3), (TILE, 1e-4), (5 * TILE + 77, 1e-3), (16 * TILE - 5, 1e-2)])
def test_reduce_step_max_min_match_reference(zcref, n, rel):
    u = _u()
    x = synth.power_law_field((n // 4096 + 1, 64, 64), seed=400).numpy().ravel()[:n]
    loc = synth.power_law_field((n // 4096 + 1, 64, 64), seed=401).numpy().ravel()[:n]
    eb = synth.abs_bound(torch.from_numpy(x), rel) if n > 1 else 1e-3
    _, s, _ = zcref.compress(x, eb)
    for op in (zcref.OP_SUM, zcref.OP_MAX, zcref.OP_MIN):
        st_ref, r_ref, total_ref = zcref.reduce_step(s, loc, op=op)
        st, r, total = u.gpu_reduce_step(s, loc, op=op)
        assert st == st_ref == ZC_OK and total == total_ref
        assert r.tobytes() == r_ref.tobytes(), f"op {op}: " + u.first_diff(r, r_ref)


def test_ring_of_max_rounds_is_the_elementwise_maximum(zcref):
    u = _u()
    n = 3 * TILE + 123
    xs = [synth.power_law_field((4, 64, 64), seed=410 + i).numpy().ravel()[:n] for i in range(5)]
    eb = synth.abs_bound(torch.from_numpy(xs[0]), 1e-3)
    for op, extreme in ((zcref.OP_MAX, np.maximum), (zcref.OP_MIN, np.minimum)):
        st, s, _ = u.gpu_compress(xs[0], eb)
        for x in xs[1:]:
            st, s, _ = u.gpu_reduce_step(s, x, op=op)
            assert st == ZC_OK
        want = zcref.compress(extreme.reduce(xs), eb)[1].copy()
        want[20:24] = np.array([len(xs)], "<u4").view(np.uint8)
        assert s.tobytes() == want.tobytes(), u.first_diff(s, want)


def test_reduce_step_op_error_paths_and_wide(zcref):
    u = _u()
    x = synth.power_law_field((3, 64, 64), seed=420).numpy().ravel()
    loc = synth.power_law_field((3, 64, 64), seed=421).numpy().ravel()
    eb = synth.abs_bound(torch.from_numpy(x), 1e-3)
    _, s, _ = zcref.compress(x, eb)
    for op in (zcref.OP_MAX, zcref.OP_MIN):
        for bad in (np.nan, np.inf, -np.inf):
            l2 = loc.copy(); l2[7000] = bad
            assert u.gpu_reduce_step(s, l2, op=op)[0] == ZC_ERR_NONFINITE == zcref.reduce_step(s, l2, op=op)[0]
        l2 = loc.copy(); l2[5000] = np.float32(eb * 2.0 ** 32) * (1 if op == zcref.OP_MAX else -1)
        assert u.gpu_reduce_step(s, l2, op=op)[0] == ZC_ERR_RANGE == zcref.reduce_step(s, l2, op=op)[0]
        assert u.gpu_reduce_step(s, loc[:-1], op=op)[0] == ZC_ERR_MISMATCH == zcref.reduce_step(s, loc[:-1], op=op)[0]
        # values far outside the guaranteed domain: wide blocks, BOUND status, stream still identical
        l3 = loc.copy(); l3[::97] *= np.float32(3e5) * (1 if op == zcref.OP_MAX else -1)
        st_ref, r_ref, _ = zcref.reduce_step(s, l3, op=op)
        st, r, _ = u.gpu_reduce_step(s, l3, op=op)
        assert st == st_ref and r.tobytes() == r_ref.tobytes(), u.first_diff(r, r_ref)
        assert zcref.inspect(r_ref)[2].max() > 15
    assert u.gpu_reduce_step(s, loc, op=3)[0] == ZC_ERR_ARG == zcref.reduce_step(s, loc, op=3)[0]


@pytest.mark.parametrize("k,n", [(1, TILE + 5), (3, 4 * TILE + 1), (8, 16 * TILE), (64, 2 * TILE - 9)])
def test_decompress_average_matches_reference(zcref, k, n):
    u = _u()
    xs, eb, streams = _rank_streams(zcref, k, 4096 * ((n + 4095) // 4096), 1e-3, seed0=430)
    streams = [zcref.compress(x[:n], eb)[1] for x in xs]
    st, red, _ = u.gpu_reduce(streams, n)
    assert st == ZC_OK and red.tobytes() == zcref.reduce(streams)[1].tobytes()
    st, y, m = u.gpu_decompress(red, n, average=True)
    st_ref, y_ref, _ = zcref.decompress(red, average=True)
    assert st == st_ref == ZC_OK and m == n
    assert np.array_equal(y.view(np.uint32), y_ref.view(np.uint32)), u.first_diff(y, y_ref)
    mean = np.mean(np.stack([x[:n].astype(np.float64) for x in xs]), axis=0)
    assert np.abs(y.astype(np.float64) - mean).max() <= eb * (1 + 1e-6)
    assert u.gpu_decompress(red, n - 1, average=True)[0] == ZC_ERR_CAPACITY
    assert u.gpu_decompress(red[:-1], n, average=True)[0] == ZC_ERR_FORMAT


# ---------------- one chunk of a stream on its own ----------------
def _gpu_range(u, s, first, count, cap=None, ws_n=None):
    d_in = u.to_dev(s)
    cap = count if cap is None else cap
    d_out = torch.full((max(min(cap, 1 << 22), 4) + 8,), float("nan"), dtype=torch.float32, device=u.DEV)
    ws = u.workspace(ws_n)
    st, n = zc.zc_decompress_range(d_in, d_in.numel(), first, count, d_out, ws, out_cap_elems=min(cap, 1 << 22))
    torch.cuda.synchronize()
    if st == ZC_OK:
        assert bool(torch.isnan(d_out[n:]).all()), "wrote past the part"
    return st, (d_out[:n].cpu().numpy() if st == ZC_OK else None), n


def test_decompress_range_matches_reference(zcref):
    u = _u()
    n = 9 * TILE + 2048 + 77
    x = synth.power_law_field((n // 4096 + 1, 64, 64), seed=600).numpy().ravel()[:n]
    eb = synth.abs_bound(torch.from_numpy(x), 1e-3)
    _, s, _ = zcref.compress(x, eb)
    whole = zcref.decompress(s)[1]
    cases = [(0, 2048), (2048, 2048), (2048, 3 * TILE), (6144, 5000), (4 * TILE, 1), (9 * TILE, 1 << 30), (9 * TILE + 2048, 77),
             (9 * TILE + 2048, 78), (0, n), (0, 0), (TILE + 4096, 10 * TILE)]
    for first, count in cases:
        st_ref, ref, m_ref = zcref.decompress_range(s, first, count, out_cap_elems=n)
        st, got, m = _gpu_range(u, s, first, count, ws_n=n)
        assert st == st_ref == ZC_OK and m == m_ref, (first, count, st, st_ref, m, m_ref)
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), (first, count)
        assert np.array_equal(ref, whole[first:first + count])
    # chunks decompressed one by one, each on a HIP stream and a workspace of its own, give the whole
    d_in = u.to_dev(s)
    out = torch.empty(n, dtype=torch.float32, device=u.DEV)
    chunk = 2 * TILE + 2048
    jobs = []
    torch.cuda.synchronize()
    for first in range(0, n, chunk):
        hs = torch.cuda.Stream()
        ws = u.workspace(n)
        with torch.cuda.stream(hs):
            st, _ = zc.zc_decompress_range(d_in, d_in.numel(), first, chunk, out[first:first + chunk], ws, sync=False,
                                           stream=hs)
        assert st == ZC_OK
        jobs.append((hs, ws, min(chunk, n - first)))
    for hs, ws, want in jobs:
        st, m = zc.zc_finish(ws, stream=hs)
        assert st == ZC_OK and m == want
    assert np.array_equal(out.cpu().numpy().view(np.uint32), whole.view(np.uint32))
    # errors
    assert _gpu_range(u, s, 100, 10, ws_n=n)[0] == ZC_ERR_ARG == zcref.decompress_range(s, 100, 10)[0]
    assert _gpu_range(u, s, 10 * TILE, 10, ws_n=n)[0] == ZC_ERR_ARG == zcref.decompress_range(s, 10 * TILE, 10)[0]
    assert _gpu_range(u, s, 2048, 100, cap=99, ws_n=n)[0] == ZC_ERR_CAPACITY == zcref.decompress_range(s, 2048, 100, out_cap_elems=99)[0]
    bad = s.copy(); bad[0] ^= 1
    assert _gpu_range(u, bad, 0, 10, ws_n=n)[0] == ZC_ERR_FORMAT


# ---------------- random mixtures of block widths, constant, narrow and wide side by side ----------------
def _random_codes(rng, n, p_const=0.4, p_wide=0.2):
    """Codes whose blocks have widths drawn per block: 0, 1..15 or 16..27, signs chosen so the codes stay small."""
    nb = (n + 31) // 32
    q = np.zeros(nb * 32, np.int64)
    kind = rng.random(nb)
    for b in range(nb):
        if kind[b] < p_const:
            w = 0
        elif kind[b] < 1 - p_wide:
            w = int(rng.integers(1, 16))
        else:
            w = int(rng.integers(16, 28))
        cur = int(rng.integers(-1000, 1001))
        q[32 * b] = cur
        if w == 0:
            q[32 * b:32 * b + 32] = cur
            continue
        mags = rng.integers(0, 1 << w, 32)
        mags[int(rng.integers(1, 32))] = (1 << w) - 1 if rng.random() < 0.5 else 1 << (w - 1)     # the block's width is exactly w
        for j in range(1, 32):
            cur += int(mags[j]) * (-1 if cur > 0 else 1)
            q[32 * b + j] = cur
    return q[:n].astype(np.int32)


@pytest.mark.parametrize("seed,n,p_wide", [(1, 3 * TILE + 100, 0.2), (2, 7 * TILE - 31, 0.0), (3, TILE + 2048 + 1, 0.6), (4, 12 * TILE, 0.02)])
def test_random_width_mixtures(zcref, seed, n, p_wide):
    u = _u()
    rng = np.random.default_rng(1000 + seed)
    eb = 1e-3
    qs = [_random_codes(rng, n, p_wide=p_wide) for _ in range(3)]
    streams = [zcref.encode_codes(q, eb)[1] for q in qs]
    for s in streams:
        st, y, m = u.gpu_decompress(s, n)
        st_ref, y_ref, _ = zcref.decompress(s)
        assert st == st_ref == ZC_OK and m == n and np.array_equal(y.view(np.uint32), y_ref.view(np.uint32))
        # back through the compressor: the values are grid points, the stream comes back unchanged
        st, s2, _ = u.gpu_compress(y_ref, eb)
        st_ref, s2_ref, _ = zcref.compress(y_ref, eb)
        assert st == st_ref and s2.tobytes() == s2_ref.tobytes(), u.first_diff(s2, s2_ref)
    st_ref, r_ref, total_ref = zcref.reduce(streams)
    st, r, total = u.gpu_reduce(streams, n)
    assert st == st_ref == ZC_OK and r.tobytes() == r_ref.tobytes(), u.first_diff(r, r_ref)
    local = zcref.decompress(streams[1])[1]
    for op in (zcref.OP_SUM, zcref.OP_MAX, zcref.OP_MIN):
        st_ref, t_ref, _ = zcref.reduce_step(streams[0], local, op=op)
        st, t, _ = u.gpu_reduce_step(streams[0], local, op=op)
        assert st == st_ref and st in (ZC_OK, ZC_ERR_BOUND) and t.tobytes() == t_ref.tobytes(), u.first_diff(t, t_ref)
    st, outs, ns = u.gpu_decompress_many(streams, [n, n, n])
    assert st == ZC_OK
    for o, s in zip(outs, streams):
        assert np.array_equal(o[:n].view(np.uint32), zcref.decompress(s)[1].view(np.uint32))
    first = 2048 * int(rng.integers(0, n // 2048 + 1))
    st_ref, part_ref, m_ref = zcref.decompress_range(streams[2], first, 5000, out_cap_elems=5000)
    st, part, m = _gpu_range(u, streams[2], first, 5000, ws_n=n)
    assert st == st_ref == ZC_OK and m == m_ref and np.array_equal(part.view(np.uint32), part_ref.view(np.uint32))


# ---------------- a stream produced in parts ----------------
PACK = 16384          # values of a tile of the compression kernel


def test_compress_in_parts_matches_reference(zcref, stream_variant):
    u = _u()
    n = 5 * PACK + 1000
    x = synth.power_law_field((n // 4096 + 1, 64, 64), seed=700).numpy().ravel()[:n]
    eb = synth.abs_bound(torch.from_numpy(x), 1e-3)
    st_ref, s_ref, total_ref = zcref.compress(x, eb)
    _, _, _, off = zcref.inspect(s_ref)
    nb = (n + 31) // 32
    d_in = u.to_dev(x)
    cap = zc.zc_compress_bound(n)
    d_out = torch.full((cap + 64,), 0xA5, dtype=torch.uint8, device=u.DEV)
    ws = u.workspace(n)
    parts = [(0, PACK), (PACK, 2 * PACK), (3 * PACK, n - 3 * PACK)]
    for first, count in parts:
        st, so_far = zc.zc_compress_part(d_in, n, eb, first, count, d_out, ws, out_cap=cap)
        assert st == ZC_OK
        end_block = (first + count + 31) // 32
        want = u.tables_end(nb) + (int(off[end_block]) if end_block < nb else total_ref - u.tables_end(nb))
        assert so_far == want, (first, count, so_far, want)
        if stream_variant == "indexed" and first + count < n:
            # what exists so far can be read: the first part alone, then a range that ends with the part
            part = torch.full((first + count,), float("nan"), dtype=torch.float32, device=u.DEV)
            st, m = zc.zc_decompress_range(d_out, so_far, 0, first + count, part, u.workspace(n))
            assert st == ZC_OK and m == first + count
            assert np.array_equal(part.cpu().numpy().view(np.uint32), zcref.decompress(s_ref)[1][:first + count].view(np.uint32))
            big = torch.empty(n, dtype=torch.float32, device=u.DEV)
            st, m = zc.zc_decompress_range(d_out, so_far, first + count - 2048, 10 ** 6, big, u.workspace(n))
            assert st == ZC_ERR_FORMAT          # ... and not beyond
    got = d_out[:total_ref].cpu().numpy()
    assert so_far == total_ref and got.tobytes() == s_ref.tobytes(), u.first_diff(got, s_ref)
    assert bool((d_out[cap:] == 0xA5).all())
    # one part that is everything; a part of nothing; the asynchronous form
    d_out.fill_(0x5A)
    st, total = zc.zc_compress_part(d_in, n, eb, 0, n, d_out, ws, out_cap=cap)
    assert st == ZC_OK and d_out[:total].cpu().numpy().tobytes() == s_ref.tobytes()
    d_out.fill_(0x5A)
    for first, count in parts:
        st, _ = zc.zc_compress_part(d_in, n, eb, first, count, d_out, ws, sync=False, out_cap=cap)
        assert st == ZC_OK
    st, total = zc.zc_finish(ws)
    assert st == ZC_OK and d_out[:total].cpu().numpy().tobytes() == s_ref.tobytes()
    st, total = zc.zc_compress_part(d_in[:0], 0, eb, 0, 0, d_out, ws, out_cap=cap)
    assert st == ZC_OK and d_out[:total].cpu().numpy().tobytes() == zcref.compress(x[:0], eb)[1].tobytes()
    # errors of a part show at the end, and parts that do not fit the rules are refused
    bad = x.copy(); bad[PACK + 5] = np.nan
    d_bad = u.to_dev(bad)
    assert zc.zc_compress_part(d_bad, n, eb, 0, PACK, d_out, ws, out_cap=cap)[0] == ZC_OK
    assert zc.zc_compress_part(d_bad, n, eb, PACK, PACK, d_out, ws, out_cap=cap)[0] == ZC_ERR_NONFINITE
    assert zc.zc_compress_part(d_bad, n, eb, 2 * PACK, n - 2 * PACK, d_out, ws, out_cap=cap)[0] == ZC_ERR_NONFINITE
    assert zc.zc_compress_part(d_in, n, eb, 100, PACK, d_out, ws, out_cap=cap)[0] == ZC_ERR_ARG
    assert zc.zc_compress_part(d_in, n, eb, 0, 100, d_out, ws, out_cap=cap)[0] == ZC_ERR_ARG
    assert zc.zc_compress_part(d_in, n, eb, 5 * PACK, 1001, d_out, ws, out_cap=cap)[0] == ZC_ERR_ARG
    assert zc.zc_compress_part(d_in, n, eb, 6 * PACK, 0, d_out, ws, out_cap=cap)[0] == ZC_ERR_ARG
    st, need = zc.zc_compress_part(d_in, n, eb, 0, n, d_out, ws, out_cap=total_ref - 4)
    assert st == ZC_ERR_CAPACITY and need == total_ref


# ---------------- corrupted streams: the same verdict as the reference, whatever the bytes ----------------
@pytest.mark.parametrize("seed", [0, 1])
def test_corrupted_streams_get_the_reference_verdict(zcref, seed):
    """Random edits of header, index, width table and payload, and truncations: every consuming call ends
    with the status the reference gives (every access of the kernels is fenced by sizes the host passed or
    the header proved), and where both accept the stream the results are the reference's."""
    u = _u()
    rng = np.random.default_rng(900 + seed)
    n = 3 * TILE + 2048 * int(rng.integers(0, 4)) + int(rng.integers(0, 2048))
    x = synth.power_law_field((n // 4096 + 1, 64, 64), seed=900 + seed).numpy().ravel()[:n]
    x[:: 997] *= np.float32(300.0)                                   # a few wide blocks
    eb = 1e-3
    st, good, total = zcref.compress(x, eb)
    assert st in (ZC_OK, ZC_ERR_BOUND)
    nb = (n + 31) // 32
    tables = u.tables_end(nb)
    verdicts = {}
    for trial in range(40):
        s = good.copy()
        kind = trial % 4
        if kind == 0:                                                # header
            s[int(rng.integers(0, 32))] ^= np.uint8(1 << int(rng.integers(0, 8)))
        elif kind == 1:                                              # index and tables
            for _ in range(int(rng.integers(1, 4))):
                s[int(rng.integers(32, tables))] = np.uint8(rng.integers(0, 256))
        elif kind == 2:                                              # payload: still a valid stream
            s[int(rng.integers(tables, total))] ^= np.uint8(1 << int(rng.integers(0, 8)))
        else:                                                        # truncated
            s = s[: int(rng.integers(0, total))]
        if s.size < 16:
            continue
        ref = zcref.decompress(s, out_cap_elems=n)
        st, y, m = u.gpu_decompress(s, n)
        assert st == ref[0], (trial, kind, "decompress", st, ref[0])
        if st == ZC_OK:
            assert np.array_equal(y.view(np.uint32), ref[1].view(np.uint32))
        ref = zcref.reduce([good, s])
        st, r, _ = u.gpu_reduce([good, s], n)
        assert st == ref[0], (trial, kind, "reduce", st, ref[0])
        if st == ZC_OK:
            assert r.tobytes() == ref[1].tobytes()
        ref = zcref.reduce_step(s, x)
        st, r, _ = u.gpu_reduce_step(s, x)
        assert st == ref[0], (trial, kind, "reduce_step", st, ref[0])
        if st in (ZC_OK, ZC_ERR_BOUND):
            assert r.tobytes() == ref[1].tobytes()
        verdicts[ref[0]] = verdicts.get(ref[0], 0) + 1
    assert len(verdicts) >= 2                                        # some accepted, some refused


def test_both_stream_variants_in_one_process_without_any_setting(zcref):
    """The variant is an argument of each call: plain and indexed streams are written and read side by
    side, by the library called directly (no test-side defaults), and the other variant's flag is FORMAT."""
    import paper_2502_18554_amd as lib
    from paper_2502_18554_amd.binding import ZC_STREAM_PLAIN
    u = _u()
    n = 3 * TILE + 123
    xs = [synth.power_law_field((8, 64, 64), seed=60 + i).numpy()[:n] for i in range(3)]
    eb = synth.abs_bound(torch.from_numpy(xs[0]), 1e-3)
    ws = u.workspace(n, 3)
    streams = {}
    for flags in (0, ZC_STREAM_PLAIN, 0, ZC_STREAM_PLAIN):          # interleaved on one workspace
        zcref.set_indexed(flags == 0)
        got = []
        for x in xs:
            out = torch.empty(lib.zc_compress_bound(n, flags), dtype=torch.uint8, device=u.DEV)
            st, total = lib.zc_compress(u.to_dev(x), n, eb, out, ws, flags=flags)
            assert st == ZC_OK and out[:total].cpu().numpy().tobytes() == zcref.compress(x, eb)[1].tobytes()
            got.append((out, total))
        streams[flags] = got
    y = torch.empty(n, dtype=torch.float32, device=u.DEV)
    red = torch.empty(lib.zc_compress_bound(n), dtype=torch.uint8, device=u.DEV)
    for flags, other in ((0, ZC_STREAM_PLAIN), (ZC_STREAM_PLAIN, 0)):
        zcref.set_indexed(flags == 0)
        s, total = streams[flags][0]
        st, m = lib.zc_decompress(s, total, y, ws, flags=flags)
        assert st == ZC_OK and m == n
        assert np.array_equal(y.cpu().numpy(), zcref.decompress(s[:total].cpu().numpy())[1])
        assert lib.zc_decompress(s, total, y, ws, flags=other)[0] == ZC_ERR_FORMAT
        assert lib.zc_peek_header(s, total)[5] == flags
        st, rt = lib.zc_reduce_compressed([a for a, _ in streams[flags]], [b for _, b in streams[flags]], red, ws, flags=flags)
        ref = zcref.reduce([a[:b].cpu().numpy() for a, b in streams[flags]])[1]
        assert st == ZC_OK and red[:rt].cpu().numpy().tobytes() == ref.tobytes()
        mixed = [streams[flags][0], streams[other][1], streams[flags][2]]
        assert lib.zc_reduce_compressed([a for a, _ in mixed], [b for _, b in mixed], red, ws, flags=flags)[0] == ZC_ERR_FORMAT
    zcref.set_indexed(u.INDEXED)


def test_workspace_content_is_irrelevant(zcref):
    """Nothing in a workspace is ever cleared: a call must not care what it finds there: noise, all ones,
    or what an earlier call left behind, seen at another offset (a workspace carved out of recycled memory)."""
    u = _u()
    n = 5 * TILE + 1000
    xs = [synth.power_law_field((11, 64, 64), seed=70 + i).numpy()[:n] for i in range(3)]
    eb = synth.abs_bound(torch.from_numpy(xs[0]), 1e-3)
    refs = [zcref.compress(x, eb)[1] for x in xs]
    red_ref = zcref.reduce(refs)[1]
    step_ref = zcref.reduce_step(refs[0], xs[1])[1]
    size = zc.zc_workspace_bytes(n, 3) + 16
    arena = torch.empty(size + 4096, dtype=torch.uint8, device=u.DEV)
    gen = torch.Generator(device=u.DEV)
    gen.manual_seed(7)
    for fill in ("noise", "ones", "used", "shifted", "shifted again"):
        shift = {"shifted": 128, "shifted again": 1152}.get(fill, 0)
        ws = arena[shift:shift + size]
        if fill == "noise":
            arena.copy_(torch.randint(0, 256, arena.shape, dtype=torch.uint8, device=u.DEV, generator=gen))
        elif fill == "ones":
            arena.fill_(0xFF)
        st, s, _ = u.gpu_compress(xs[0], eb, ws=ws)
        assert st == ZC_OK and s.tobytes() == refs[0].tobytes(), fill
        st, r, _ = u.gpu_reduce(refs, n, ws=ws)
        assert st == ZC_OK and r.tobytes() == red_ref.tobytes(), fill
        st, t, _ = u.gpu_reduce_step(refs[0], xs[1], ws=ws)
        assert st == ZC_OK and t.tobytes() == step_ref.tobytes(), fill
        st, y, m = u.gpu_decompress(refs[0], n, ws=ws)
        assert st == ZC_OK and np.array_equal(y, zcref.decompress(refs[0])[1]), fill
        # an error of one call must not show in the next
        assert u.gpu_decompress(refs[0], n - 1, ws=ws)[0] == ZC_ERR_CAPACITY
        st, s, _ = u.gpu_compress(xs[2], eb, ws=ws)
        assert st == ZC_OK and s.tobytes() == refs[2].tobytes(), fill


def test_concurrent_calls_on_several_streams(zcref):
    """Calls that write streams (compress, k-way reduce, ring round) run at the same time on three HIP
    streams with a workspace each, while a long elementwise kernel keeps a fourth stream busy; every output
    is the reference's, byte for byte.  All waits inside the kernels are bounded."""
    u = _u()
    n = 48 * TILE + 77
    xs = [synth.power_law_field((97, 64, 64), seed=80 + i).numpy()[:n] for i in range(4)]
    eb = synth.abs_bound(torch.from_numpy(xs[0]), 1e-3)
    refs = [zcref.compress(x, eb)[1] for x in xs]
    want = {"compress": refs[3], "reduce": zcref.reduce(refs[:3])[1], "round": zcref.reduce_step(refs[0], xs[1])[1]}
    d_x = [u.to_dev(x) for x in xs]
    d_s = [u.to_dev(s) for s in refs]
    cap = zc.zc_compress_bound(n)
    outs = {k: torch.empty(cap, dtype=torch.uint8, device=u.DEV) for k in want}
    wss = {k: u.workspace(n, 3) for k in want}
    streams = {k: torch.cuda.Stream() for k in want}
    busy_stream = torch.cuda.Stream()
    big = torch.ones(1 << 28, dtype=torch.float32, device=u.DEV)
    torch.cuda.synchronize()
    for rep in range(6):
        for o in outs.values():
            o.fill_(0x11)
        torch.cuda.synchronize()
        with torch.cuda.stream(busy_stream):
            for _ in range(4):
                big.mul_(1.0000001).add_(1e-9)
        for _ in range(3):                         # several rounds of the three calls in flight together
            assert zc.zc_compress(d_x[3], n, eb, outs["compress"], wss["compress"], sync=False, stream=streams["compress"])[0] == ZC_OK
            assert zc.zc_reduce_compressed(d_s[:3], [s.numel() for s in d_s[:3]], outs["reduce"], wss["reduce"], sync=False,
                                           stream=streams["reduce"])[0] == ZC_OK
            assert zc.zc_reduce_step(d_s[0], d_s[0].numel(), d_x[1], n, outs["round"], wss["round"], sync=False,
                                     stream=streams["round"])[0] == ZC_OK
        for k in want:
            st, total = zc.zc_finish(wss[k], stream=streams[k])
            assert st == ZC_OK and total == want[k].size, (k, rep, st)
            assert outs[k][:total].cpu().numpy().tobytes() == want[k].tobytes(), (k, rep)
        torch.cuda.synchronize()


@pytest.mark.parametrize("short_by", ["all", "more than an index span"])
def test_output_too_small_by_a_lot_is_capacity(zcref, short_by):
    """A stream that is in order and an output buffer that is much too small: CAPACITY and the stream's n,
    also when the buffer is short by more than the 2^20 values that one workgroup of the index kernel covers."""
    u = _u()
    n = (1 << 21) + 4097
    x = synth.sinusoids(n, seed=9).numpy()
    eb = synth.abs_bound(torch.from_numpy(x), 1e-3)
    _, s, _ = zcref.compress(x, eb)
    cap = 0 if short_by == "all" else n - (1 << 20) - 1
    ws = u.workspace(n, 2)
    ws.fill_(0x5A)
    st, _, m = u.gpu_decompress(s, cap, ws=ws)
    assert (st, m) == (ZC_ERR_CAPACITY, n)
    assert zcref.decompress(s, out_cap_elems=cap)[0] == ZC_ERR_CAPACITY
    st, _, ns = u.gpu_decompress_many([s, s], [cap, n], ws=ws)
    assert st == ZC_ERR_CAPACITY and ns == [n, n]
    st, outs, ns = u.gpu_decompress_many([s, s], [n, n], ws=ws)
    assert st == ZC_OK and np.array_equal(outs[1][:n], zcref.decompress(s)[1])


def test_infinity_under_a_huge_bound_is_nonfinite(zcref):
    """With a bound above 2^111 the quantiser's screen 2^17 eb is no binary32 number any more; an infinite
    input must still end as NONFINITE, in the compression, the staged quantiser and the ring round."""
    u = _u()
    eb = np.float32(1e34)
    x = np.zeros(2 * TILE + 5, np.float32)
    x[TILE + 3] = np.inf
    assert zcref.compress(x, eb)[0] == ZC_ERR_NONFINITE
    assert u.gpu_compress(x, eb)[0] == ZC_ERR_NONFINITE
    d_q = torch.empty(x.size, dtype=torch.int32, device=u.DEV)
    assert zc.zc_debug_quantize(u.to_dev(x), x.size, float(eb), d_q, u.workspace(x.size)) == ZC_ERR_NONFINITE
    zeros = np.zeros_like(x)
    _, s0, _ = zcref.compress(zeros, eb)
    assert zcref.reduce_step(s0, x)[0] == ZC_ERR_NONFINITE
    assert u.gpu_reduce_step(s0, x)[0] == ZC_ERR_NONFINITE
    x[TILE + 3] = np.float32(3e38)             # finite, and inside the bound's domain: nothing to report
    st, s, _ = u.gpu_compress(x, eb)
    st_ref, s_ref, _ = zcref.compress(x, eb)
    assert st == st_ref and (s is None or s.tobytes() == s_ref.tobytes())


@pytest.mark.parametrize("k,n,rel", [(1, TILE + 5, 1e-3), (2, 4 * TILE - 37, 1e-2), (3, 9 * 4096 + 1, 1e-4), (8, 16 * 4096, 1e-4),
                                     (17, 3 * 4096 + 5, 1e-3), (64, 2 * TILE - 9, 1e-3)])
def test_reduce_max_min_stream_matches_reference(zcref, k, n, rel):
    """The k-way Max and Min of compressed operands, byte for byte; also against numpy's extreme compressed
    once and against the ring of Max rounds, both on the GPU."""
    u = _u()
    xs, eb, _ = _rank_streams(zcref, k, (n + 4095) // 4096 * 4096, rel, seed0=90)
    xs = [x[:n] for x in xs]
    streams = [zcref.compress(x, eb)[1] for x in xs]
    for op, extreme in ((zc.binding.ZC_OP_MAX, np.maximum), (zc.binding.ZC_OP_MIN, np.minimum)):
        st_ref, r_ref, total_ref = zcref.reduce(streams, op=op)
        st, r, total = u.gpu_reduce(streams, n, op=op)
        assert st == st_ref == ZC_OK and total == total_ref
        assert r.tobytes() == r_ref.tobytes(), u.first_diff(r, r_ref)
        st, y, _ = u.gpu_decompress(r, n)
        assert np.max(np.abs(y.astype(np.float64) - extreme.reduce(xs))) <= eb
        if k <= 8:
            ring = streams[0]
            for x in xs[1:]:
                st, ring, _ = u.gpu_reduce_step(ring, x, op=op)
                assert st == ZC_OK
            assert ring.tobytes() == r.tobytes()
    # Sum through the same entry point is zc_reduce_compressed
    st, r, _ = u.gpu_reduce(streams, n, op=zc.binding.ZC_OP_SUM)
    assert st == ZC_OK and r.tobytes() == zcref.reduce(streams)[1].tobytes()


def test_reduce_max_min_wide_blocks_and_errors(zcref):
    u = _u()
    rng = np.random.default_rng(12)
    n = 3 * TILE + 77
    scale = np.repeat(2.0 ** rng.integers(0, 27, (n + 31) // 32), 32)[:n]
    qs = [(rng.uniform(-1, 1, n) * scale).astype(np.int32) for _ in range(4)]
    qs.append(np.zeros(n, np.int32))                  # an all-constant operand
    qs.append(qs[1].copy())                           # an operand twice
    streams = [zcref.encode_codes(q, 1e-3)[1] for q in qs]
    narrow = [zcref.encode_codes((q >> 14).astype(np.int32), 1e-3)[1] for q in qs]
    for op in (zc.binding.ZC_OP_MAX, zc.binding.ZC_OP_MIN):
        for ss in (streams, narrow, [streams[0]] + narrow[1:]):
            st_ref, r_ref, total_ref = zcref.reduce(ss, op=op)
            st, r, total = u.gpu_reduce(ss, n, op=op)
            assert st == st_ref == ZC_OK and total == total_ref
            assert r.tobytes() == r_ref.tobytes(), u.first_diff(r, r_ref)
    # error paths follow the reference
    op = zc.binding.ZC_OP_MAX
    other = zcref.encode_codes(qs[0], 2e-3)[1]
    assert u.gpu_reduce([streams[0], other], n, op=op)[0] == ZC_ERR_MISMATCH == zcref.reduce([streams[0], other], op=op)[0]
    shorter = zcref.encode_codes(qs[0][:n - 1], 1e-3)[1]
    assert u.gpu_reduce([streams[0], shorter], n, op=op)[0] == ZC_ERR_MISMATCH
    bad = streams[1].copy(); bad[0] ^= 1
    assert u.gpu_reduce([streams[0], bad], n, op=op)[0] == ZC_ERR_FORMAT == zcref.reduce([streams[0], bad], op=op)[0]
    st, _, total = u.gpu_reduce(narrow, n, out_cap=4096, op=op)
    assert st == ZC_ERR_CAPACITY and total == zcref.reduce(narrow, op=op)[2]
    assert u.gpu_reduce(narrow, n, op=7)[0] == ZC_ERR_ARG
    empty = [zcref.encode_codes(np.zeros(0, np.int32), 1e-3)[1]] * 3
    st, r, _ = u.gpu_reduce(empty, 0, op=op)
    assert st == ZC_OK and r.tobytes() == zcref.reduce(empty, op=op)[1].tobytes()


def _poison_beyond(stream, nb, end_block, off):
    """A copy of an indexed stream in which everything that describes blocks from end_block on (index entries,
    width bytes, outliers, payload) is overwritten: what a part that ends there must not look at."""
    import gpuutil as u
    s = stream.copy()
    if end_block >= nb:
        return s
    nseg = (nb + 63) // 64
    wb, te = u.widths_begin(nb), u.tables_end(nb)
    ob = wb + u.pad16(nb)
    first_seg = (end_block + 63) // 64 + 1          # the entry at the part's end is the end of its last segment
    s[32 + 4 * first_seg:32 + 4 * (nseg + 1)] = 0xEE
    s[wb + end_block:wb + nb] = 0xEE
    s[ob + 4 * end_block:ob + 4 * nb] = 0xEE
    s[te + int(off[end_block]):] = 0xEE
    return s


def test_reduce_and_ring_round_in_parts_match_reference(zcref, stream_variant):
    """zc_reduce_compressed_part and zc_reduce_step_part: the parts add up, byte for byte, to the stream of the
    call in one piece (the reference's), each part leaves a stream that can be read up to its end, and a part
    looks at nothing of its operands beyond its own segments."""
    u = _u()
    n = 5 * TILE + 1000
    k = 3
    xs = [synth.power_law_field((n // 4096 + 1, 64, 64), seed=710 + i).numpy().ravel()[:n] for i in range(k)]
    eb = synth.abs_bound(torch.from_numpy(xs[0]), 1e-3)
    streams = [zcref.compress(x, eb)[1] for x in xs]
    nb = (n + 31) // 32
    cap = zc.zc_compress_bound(n)
    d_out = torch.full((cap + 64,), 0xA5, dtype=torch.uint8, device=u.DEV)
    ws = u.workspace(n, k)
    d_streams = [u.to_dev(s) for s in streams]
    sizes = [s.size for s in streams]
    parts = [(0, TILE), (TILE, 2 * TILE), (3 * TILE, n - 3 * TILE)]
    if stream_variant == "plain":              # plain streams cannot be taken up in parts
        assert zc.zc_reduce_compressed_part(d_streams, sizes, n, 0, TILE, d_out, ws, out_cap=cap)[0] == ZC_ERR_ARG
        assert zc.zc_reduce_step_part(d_streams[0], sizes[0], u.to_dev(xs[1]), n, 0, 0, TILE, d_out, ws, out_cap=cap)[0] == ZC_ERR_ARG
        return
    offs = [zcref.inspect(s)[3] for s in streams]
    cases = [("sum", lambda: zcref.reduce(streams), None)]
    for op in (zc.binding.ZC_OP_SUM, zc.binding.ZC_OP_MAX):
        cases.append((f"round {op}", (lambda op=op: zcref.reduce_step(streams[0], xs[1], op=op)), op))
    for name, reference, op in cases:
        st_ref, r_ref, total_ref = reference()
        assert st_ref == ZC_OK
        off_r = zcref.inspect(r_ref)[3]
        d_out.fill_(0xA5)
        d_loc = u.to_dev(xs[1])
        for first, count in parts:
            end_block = (first + count + 31) // 32
            poisoned = [u.to_dev(_poison_beyond(s, nb, end_block, o)) for s, o in zip(streams, offs)]
            if op is None:
                st, so_far = zc.zc_reduce_compressed_part(poisoned, sizes, n, first, count, d_out, ws, out_cap=cap)
            else:
                st, so_far = zc.zc_reduce_step_part(poisoned[0], sizes[0], d_loc, n, op, first, count, d_out, ws, out_cap=cap)
            assert st == ZC_OK, (name, first)
            want = u.tables_end(nb) + (int(off_r[end_block]) if end_block < nb else total_ref - u.tables_end(nb))
            assert so_far == want, (name, first, so_far, want)
            if first + count < n:                 # what exists so far can be read
                part = torch.full((first + count,), float("nan"), dtype=torch.float32, device=u.DEV)
                st, m = zc.zc_decompress_range(d_out, so_far, 0, first + count, part, u.workspace(n))
                assert st == ZC_OK and m == first + count
                assert np.array_equal(part.cpu().numpy().view(np.uint32), zcref.decompress(r_ref)[1][:first + count].view(np.uint32))
        got = d_out[:total_ref].cpu().numpy()
        assert so_far == total_ref and got.tobytes() == r_ref.tobytes(), (name, u.first_diff(got, r_ref))
        assert bool((d_out[cap:] == 0xA5).all())
    # the asynchronous form, one part that is everything, and parts that do not fit the rules
    d_out.fill_(0x5A)
    for first, count in parts:
        assert zc.zc_reduce_compressed_part(d_streams, sizes, n, first, count, d_out, ws, sync=False, out_cap=cap)[0] == ZC_OK
    st, total = zc.zc_finish(ws)
    assert st == ZC_OK and d_out[:total].cpu().numpy().tobytes() == zcref.reduce(streams)[1].tobytes()
    st, total = zc.zc_reduce_compressed_part(d_streams, sizes, n, 0, n, d_out, ws, out_cap=cap)
    assert st == ZC_OK and d_out[:total].cpu().numpy().tobytes() == zcref.reduce(streams)[1].tobytes()
    assert zc.zc_reduce_compressed_part(d_streams, sizes, n, 100, TILE, d_out, ws, out_cap=cap)[0] == ZC_ERR_ARG
    assert zc.zc_reduce_compressed_part(d_streams, sizes, n, 0, 100, d_out, ws, out_cap=cap)[0] == ZC_ERR_ARG
    assert zc.zc_reduce_compressed_part(d_streams, sizes, n, 6 * TILE, TILE, d_out, ws, out_cap=cap)[0] == ZC_ERR_ARG
    assert zc.zc_reduce_compressed_part(d_streams, sizes, n + 32, 0, TILE, d_out, ws, out_cap=cap)[0] == ZC_ERR_MISMATCH
    # (workgroups ask for their tables where the n they are told puts them, before they know the headers: a
    #  wrong n, far too large or too small, must neither read outside the streams nor pass)
    big_ws = u.workspace(64 * n, len(d_streams))
    assert zc.zc_reduce_compressed_part(d_streams, sizes, 64 * n, 0, TILE, d_out, big_ws, out_cap=cap)[0] == ZC_ERR_MISMATCH
    assert zc.zc_reduce_compressed_part(d_streams, sizes, 64 * n, 32 * n // TILE * TILE, TILE, d_out, big_ws, out_cap=cap)[0] == ZC_ERR_MISMATCH
    assert zc.zc_reduce_compressed_part(d_streams, sizes, TILE, 0, TILE, d_out, ws, out_cap=cap)[0] == ZC_ERR_MISMATCH
    assert zc.zc_reduce_step_part(d_streams[0], sizes[0], d_loc, n, 0, 0, 100, d_out, ws, out_cap=cap)[0] == ZC_ERR_ARG
    # an error in a middle part shows at the end
    bad = xs[1].copy(); bad[TILE + 5] = np.nan
    d_bad = u.to_dev(bad)
    assert zc.zc_reduce_step_part(d_streams[0], sizes[0], d_bad, n, 0, 0, TILE, d_out, ws, out_cap=cap)[0] == ZC_OK
    assert zc.zc_reduce_step_part(d_streams[0], sizes[0], d_bad, n, 0, TILE, TILE, d_out, ws, out_cap=cap)[0] == ZC_ERR_NONFINITE
    assert zc.zc_reduce_step_part(d_streams[0], sizes[0], d_bad, n, 0, 2 * TILE, n - 2 * TILE, d_out, ws, out_cap=cap)[0] == ZC_ERR_NONFINITE


@pytest.mark.parametrize("lead_width", [0, 1, 2, 3, 6])
def test_staging_corners_full_width_waves_off_the_grid(zcref, lead_width):
    """The copy of a wave's payload into LDS moves whole 16-byte pieces and fetches what is left separately:
    waves whose 64 blocks are all 15 bits wide (1024 words) starting 0..3 words off the 16-byte grid (up to three
    words beyond the four pieces), and streams whose payload ends inside a piece.  Decompression, the k-way Sum,
    Max and the ring round, against the reference."""
    u = _u()
    rng = np.random.default_rng(900 + lead_width)
    nseg = 9
    n = 2048 * nseg - 5                                   # the last block is ragged
    q = np.zeros(n, np.int64)
    # block 0 decides how far off the grid everything behind it starts: 1 + lead_width payload words, or none
    if lead_width:
        q[1:32:2] = 2 ** (lead_width - 1)
    sign = np.where(np.arange(n - 32) % 2 == 0, 1, -1)
    q[32:] = sign * (2 ** 13 + rng.integers(0, 2 ** 13 - 1, n - 32))      # deltas of magnitude 2^14 .. 2^15 - 1
    q = q.astype(np.int32)
    eb = 1e-3
    st, s, total = zcref.encode_codes(q, eb)
    assert st == ZC_OK
    nb = (n + 31) // 32
    w = u.widths_of(s, nb)
    assert w[0] == lead_width and (w[1:] == 15).all()
    st, y, m = u.gpu_decompress(s, n)
    st_ref, y_ref, _ = zcref.decompress(s)
    assert st == st_ref == ZC_OK and m == n and np.array_equal(y.view(np.uint32), y_ref.view(np.uint32))
    # a second operand with small codes keeps the sums inside 15 bits where it matters less: widths stay mixed
    q2 = rng.integers(-3, 4, n).astype(np.int32)
    s2 = zcref.encode_codes(q2, eb)[1]
    for op in (None, 1):
        st_ref, r_ref, t_ref = zcref.reduce([s, s2]) if op is None else zcref.reduce([s, s2], op=op)
        st, r, t = u.gpu_reduce([s, s2], n, op=op)
        assert st == st_ref and t == t_ref and r.tobytes() == r_ref.tobytes(), (op, u.first_diff(r, r_ref))
    local = (rng.uniform(-1, 1, n) * eb).astype(np.float32)
    st_ref, t_ref, b_ref = zcref.reduce_step(s, local)
    st, t, b = u.gpu_reduce_step(s, local)
    assert st == st_ref and b == b_ref and t.tobytes() == t_ref.tobytes()
    # every length of the payload modulo four words, by cutting blocks off the end
    for cut in (1, 2, 3, 4, 5):
        qc = q[: n - 32 * cut]
        sc = zcref.encode_codes(qc, eb)[1]
        st, y, m = u.gpu_decompress(sc, qc.size)
        assert st == ZC_OK and np.array_equal(y.view(np.uint32), zcref.decompress(sc)[1].view(np.uint32)), cut
