"""The local steps of the paper's compressed Allreduce, chained on one GPU.

N ranks are emulated by N buffers on the same device; "sending" is handing the stream to the
next call.  Two forms are run and compared with the exact float64 sum:
 * the ring of Section 3.1.2 / 3.5: N - 1 rounds of reduce-scatter, each round one
   zc_reduce_step per rank (received compressed chunk + local uncompressed chunk), then the
   Allgather tail, where every rank decompresses the N reduced chunks with one
   zc_decompress_many;
 * the direct form: every chunk compressed once, the N streams of a chunk summed by one
   zc_reduce_compressed.
Both stay within N * eb (Section 3.2: one bounded error per compression in the chain), and
every rank ends with the same bits.
"""
import numpy as np
import pytest
import torch

from gpuutil import zc
from paper_2502_18554_amd import synth
from paper_2502_18554_amd.binding import ZC_OK

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("stream_variant")]
DEV = "cuda:0"


def _compress(x, eb, ws):
    out = torch.empty(zc.zc_compress_bound(x.numel()), dtype=torch.uint8, device=DEV)
    st, total = zc.zc_compress(x, x.numel(), eb, out, ws)
    assert st == ZC_OK
    return out, total


@pytest.mark.parametrize("nranks,chunk", [(4, 3 * 8192 + 517), (8, 8192)])
def test_ring_allreduce_and_direct_form(nranks, chunk):
    N = nranks
    n = N * chunk
    eb = 1e-3
    bufs = [synth.power_law_field((N, 64, (chunk + 63) // 64 + 1), seed=200 + r, device=DEV).ravel()[:n].contiguous()
            for r in range(N)]
    exact = torch.zeros(n, dtype=torch.float64, device=DEV)
    for b in bufs:
        exact += b.double()
    ws = torch.empty(zc.zc_workspace_bytes(chunk, N) + 16, dtype=torch.uint8, device=DEV)
    # chunk views need 16-byte alignment: copy the chunks out
    local = [[b[c * chunk:(c + 1) * chunk].clone() for c in range(N)] for b in bufs]

    # ---- ring reduce-scatter: in round t rank r sends chunk (r - t) mod N to rank r + 1 ----
    carried = [None] * N                                     # the stream each rank sends next
    for r in range(N):
        carried[r] = _compress(local[r][r], eb, ws)
    for t in range(1, N):
        received = [carried[(r - 1) % N] for r in range(N)]
        for r in range(N):
            c = (r - t) % N
            out = torch.empty(zc.zc_compress_bound(chunk), dtype=torch.uint8, device=DEV)
            st, total = zc.zc_reduce_step(received[r][0], received[r][1], local[r][c], chunk, out, ws)
            assert st == ZC_OK
            carried[r] = (out, total)
    # rank r now owns the fully reduced chunk (r + 1) mod N, compressed
    owned = {(r + 1) % N: carried[r] for r in range(N)}
    st, nsum = zc.zc_peek_header(owned[0][0], owned[0][1])[0], zc.zc_peek_header(owned[0][0], owned[0][1])[3]
    assert st == ZC_OK and nsum == N
    # ---- Allgather tail: every rank decompresses the N chunks it has gathered, in one call ----
    results = []
    for r in range(N):
        outs = [torch.empty(chunk, dtype=torch.float32, device=DEV) for _ in range(N)]
        st, ns = zc.zc_decompress_many([owned[c][0] for c in range(N)], [owned[c][1] for c in range(N)], outs, ws)
        assert st == ZC_OK and ns == [chunk] * N
        results.append(torch.cat(outs))
    for r in range(1, N):
        assert torch.equal(results[0].view(torch.int32), results[r].view(torch.int32))
    err = (results[0].double() - exact).abs().max().item()
    assert err <= N * eb, (err, N * eb)

    # ---- direct form: every chunk compressed once, N streams summed on the codes ----
    direct = []
    for c in range(N):
        streams = [_compress(local[r][c], eb, ws) for r in range(N)]
        out = torch.empty(zc.zc_compress_bound(chunk), dtype=torch.uint8, device=DEV)
        st, total = zc.zc_reduce_compressed([s for s, _ in streams], [t for _, t in streams], out, ws)
        assert st == ZC_OK
        direct.append((out, total))
    outs = [torch.empty(chunk, dtype=torch.float32, device=DEV) for _ in range(N)]
    st, _ = zc.zc_decompress_many([d[0] for d in direct], [d[1] for d in direct], outs, ws)
    assert st == ZC_OK
    err_direct = (torch.cat(outs).double() - exact).abs().max().item()
    assert err_direct <= N * eb
    # the direct form adds exact codes: its error is a sum of N independent quantisation errors,
    # the ring adds one more rounding per round on top of the carried error; both are well inside
    # the worst case, and neither is biased
    assert abs((torch.cat(outs).double() - exact).mean().item()) < eb / 50
    assert abs((results[0].double() - exact).mean().item()) < eb / 50


@pytest.mark.parametrize("nranks,chunk", [(4, 2 * 8192 + 99)])
def test_ring_allreduce_max_min_and_average(nranks, chunk):
    """The other aggregation functions of Section 3.2 through the same ring: Max and Min by rounds of
    zc_reduce_step_op (the result is within eb of the exact extreme however long the ring), Average by
    summing on the codes and dividing on the way out (within eb of the exact mean)."""
    N = nranks
    eb = 1e-3
    ws = torch.empty(zc.zc_workspace_bytes(chunk, N) + 16, dtype=torch.uint8, device=DEV)
    local = [synth.power_law_field((N, 64, (chunk + 63) // 64 + 1), seed=300 + r, device=DEV).ravel()[:chunk].clone()
             for r in range(N)]
    stacked = torch.stack([x.double() for x in local])
    for op, exact in ((zc.binding.ZC_OP_MAX, stacked.max(0).values), (zc.binding.ZC_OP_MIN, stacked.min(0).values)):
        carried = _compress(local[0], eb, ws)
        for r in range(1, N):
            out = torch.empty(zc.zc_compress_bound(chunk), dtype=torch.uint8, device=DEV)
            st, total = zc.zc_reduce_step_op(carried[0], carried[1], local[r], chunk, op, out, ws)
            assert st == ZC_OK
            carried = (out, total)
        y = torch.empty(chunk, dtype=torch.float32, device=DEV)
        st, n = zc.zc_decompress(carried[0], carried[1], y, ws)
        assert st == ZC_OK and n == chunk
        assert (y.double() - exact).abs().max().item() <= eb
        # the ring's result is the stream of the exact extreme, compressed once
        direct = _compress(exact.float(), eb, ws)
        y2 = torch.empty(chunk, dtype=torch.float32, device=DEV)
        zc.zc_decompress(direct[0], direct[1], y2, ws)
        assert torch.equal(y.view(torch.int32), y2.view(torch.int32))
    streams = [_compress(x, eb, ws) for x in local]
    out = torch.empty(zc.zc_compress_bound(chunk), dtype=torch.uint8, device=DEV)
    st, total = zc.zc_reduce_compressed([s for s, _ in streams], [t for _, t in streams], out, ws)
    assert st == ZC_OK
    y = torch.empty(chunk, dtype=torch.float32, device=DEV)
    st, n = zc.zc_decompress_average(out, total, y, ws)
    assert st == ZC_OK and n == chunk
    err = y.double() - stacked.mean(0)
    assert err.abs().max().item() <= eb * (1 + 1e-6)
    sigma = eb * 63 / 32 / 12 ** 0.5
    assert abs(err.pow(2).mean().sqrt().item() / (sigma / N ** 0.5) - 1) < 0.1        # Corollary 1
