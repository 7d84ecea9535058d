"""zc_compress_noalloc (the entry point for callers that cannot allocate: its workspace is a static
device array of the library) against zc_compress on a caller's workspace, through the C ABI: the
streams must agree byte for byte, on two calls in a row, the second on a smaller input, which finds the
array as the first call left it."""
import numpy as np
import pytest
import torch

import paper_2502_18554_amd as zc
from paper_2502_18554_amd import synth
from paper_2502_18554_amd.binding import ZC_ERR_ARG, ZC_ERR_CAPACITY, ZC_NOALLOC_MAX_N, ZC_OK

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TILE = 16384          # values of one tile of the compression kernel


def _with_workspace(x, eb, flags=0):
    n = x.numel()
    out = torch.full((zc.zc_compress_bound(n) + 64,), 0xA5, dtype=torch.uint8, device=DEV)
    ws = torch.empty(zc.zc_workspace_bytes(n, 1) + 16, dtype=torch.uint8, device=DEV)
    st, total = zc.zc_compress(x, n, eb, out, ws, out_cap=out.numel() - 64, flags=flags)
    assert st == ZC_OK
    return out[:total].cpu().numpy()


def _no_alloc(x, eb, sync=True):
    n = x.numel()
    cap = zc.zc_compress_bound(n)
    out = torch.full((cap + 64,), 0xA5, dtype=torch.uint8, device=DEV)
    st, total = zc.zc_compress_noalloc(x, n, eb, out, sync=sync, out_cap=cap)
    if not sync:
        assert st == ZC_OK
        st, total = zc.zc_finish(None)
    assert st == ZC_OK, zc.zc_strerror(st)
    assert bool((out[cap:] == 0xA5).all()), "wrote past out_cap"
    return out[:total].cpu().numpy()


@pytest.mark.parametrize("hand_out", [0, zc.binding.ZC_TILES_BY_TICKET], ids=["dispatch_order", "tickets"])
def test_two_calls_in_a_row_match_the_workspace_form(hand_out):
    """The entry point takes no flags (the default stream variant and tile hand-out); the stream it is compared
    with comes from zc_compress on a workspace of the caller, in either hand-out mode."""
    if True:
        big = synth.power_law_field((40, 64, 64), seed=11, device=DEV)[: 9 * TILE + 4321].contiguous()
        small = synth.sinusoids(2 * TILE + 77, seed=5).to(DEV)
        eb_big, eb_small = synth.abs_bound(big, 1e-3), synth.abs_bound(small, 1e-4)
        want_big, want_small = _with_workspace(big, eb_big, hand_out), _with_workspace(small, eb_small, hand_out)
        # first call, then a smaller input on the array as the first call left it, then both again in the
        # asynchronous form (completed by zc_finish with a null workspace)
        for sync in (True, False):
            got_big = _no_alloc(big, eb_big, sync)
            got_small = _no_alloc(small, eb_small, sync)
            assert got_big.tobytes() == want_big.tobytes()
            assert got_small.tobytes() == want_small.tobytes()
        # the empty input and a single value find the array used as well
        for n in (0, 1):
            x = small[:n].contiguous() if n else torch.zeros(4, device=DEV)[:0]
            want = _with_workspace(small[:max(n, 1)][:n], eb_small) if n else None
            got = _no_alloc(small[:n], eb_small)
            if want is not None:
                assert got.tobytes() == want.tobytes()
            else:
                assert got.size == zc.zc_compress_bound(0)


def test_size_limit_and_errors():
    x = torch.zeros(64, device=DEV)
    out = torch.empty(4096, dtype=torch.uint8, device=DEV)
    # beyond the static workspace: refused before anything is launched (the input is never touched)
    st, _ = zc.zc_compress_noalloc(x, ZC_NOALLOC_MAX_N + 1, 1e-3, out)
    assert st == ZC_ERR_ARG
    st, _ = zc.zc_compress_noalloc(x, 64, float("nan"), out)
    assert st == ZC_ERR_ARG
    st, total = zc.zc_compress_noalloc(x, 64, 1e-3, out, out_cap=16)
    assert st == ZC_ERR_CAPACITY
    # and the call after an error is as good as any
    want = _with_workspace(x, 1e-3)
    assert _no_alloc(x, 1e-3).tobytes() == want.tobytes()


def test_largest_size_allowed():
    n = ZC_NOALLOC_MAX_N
    x = synth.sinusoids(1 << 20, seed=2).to(DEV).repeat(n >> 20)
    eb = synth.abs_bound(x[: 1 << 20], 1e-3)
    got = _no_alloc(x, eb)
    want = _with_workspace(x, eb)
    assert np.array_equal(got, want)
