"""The look-back's other way of reading a tile's own chain (ZC_CHAINS_COHERENT: device-coherent vector
loads instead of scalar loads through the XCD's L2) is the path a tile also takes by itself when the scalar
loads find nothing new; results must not depend on it.  Streams of many tiles, so that chains are deep."""
import numpy as np
import pytest
import torch

import gpuutil
from paper_2502_18554_amd import synth
from paper_2502_18554_amd.binding import ZC_OK

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("stream_variant")]

TILE = 8192


@pytest.fixture(params=["dispatch_order", "tickets"], autouse=True)
def coherent_chains(request):
    gpuutil.set_tickets(request.param == "tickets")
    gpuutil.set_coherent(True)
    yield request.param
    gpuutil.set_coherent(False)
    gpuutil.set_tickets(False)


def _fields(count, n):
    return [synth.power_law_field((40, 128, 128), seed=300 + i).numpy()[:n] for i in range(count)]


def test_compress_and_reduce_with_coherent_chains(zcref):
    u = gpuutil
    n = 75 * TILE + 4321                         # 38 tiles of the compressor, 76 of the others, a ragged end
    xs = _fields(3, n)
    eb = synth.abs_bound(torch.from_numpy(xs[0]), 1e-3)
    refs = [zcref.compress(x, eb)[1] for x in xs]
    for x, ref in zip(xs, refs):
        st, s, total = u.gpu_compress(x, eb)
        assert st == ZC_OK and total == ref.size and s.tobytes() == ref.tobytes(), u.first_diff(s, ref)
    for op in (None, 1, 2):
        st_ref, red_ref = zcref.reduce(refs, op=op or 0)[:2]
        st, red, total = u.gpu_reduce(refs, n, op=op)
        assert st == st_ref == ZC_OK and red.tobytes() == red_ref.tobytes(), u.first_diff(red, red_ref)
    for op in (None, 1, 2):
        st_ref, step_ref = zcref.reduce_step(refs[0], xs[1], op=op or 0)[:2]
        st, step, total = u.gpu_reduce_step(refs[0], xs[1], op=op)
        assert st == st_ref == ZC_OK and step.tobytes() == step_ref.tobytes(), u.first_diff(step, step_ref)


def test_wide_tiles_with_coherent_chains(zcref):
    """Blocks wider than 15 bits take the kernels' other paths, which look back the same way."""
    u = gpuutil
    n = 20 * TILE
    x = synth.hard_mix(n, seed=9).numpy()
    eb = synth.abs_bound(torch.from_numpy(x), 1e-5)
    st_ref, ref = zcref.compress(x, eb)[:2]
    st, s, total = u.gpu_compress(x, eb)
    assert st == st_ref
    if st == ZC_OK:
        assert s.tobytes() == ref.tobytes(), u.first_diff(s, ref)
        st_r, red_ref = zcref.reduce([ref, ref])[:2]
        st_g, red, _ = u.gpu_reduce([ref, ref], n)
        assert st_g == st_r and (st_r != ZC_OK or red.tobytes() == red_ref.tobytes())


def test_streaming_probe_moves_what_it_says():
    """zc_debug_stream: every 16-byte store holds the exclusive-or of the lane's loads (and of the lane's and the
    workgroup's numbers); nothing outside the two ranges is touched."""
    import paper_2502_18554_amd as lib
    dev = gpuutil.DEV
    gen = torch.Generator(device=dev)
    gen.manual_seed(11)
    for tiles, loads, stores in ((3, 1, 1), (5, 8, 3), (2, 16, 16), (4, 0, 2), (4, 3, 0)):
        words = 512 * 4                                   # 32-bit words of one 8 KiB access
        src = torch.randint(0, 2**31 - 1, (tiles * max(loads, 1) * words + 4,), dtype=torch.int32, device=dev, generator=gen)
        dst = torch.full((tiles * max(stores, 1) * words + 4,), 0x5A5A5A5A, dtype=torch.int32, device=dev)
        before = dst.clone()
        assert lib.zc_debug_stream(src if loads else None, dst if stores else None, tiles, loads, stores) == ZC_OK
        torch.cuda.synchronize()
        if not stores:
            assert torch.equal(dst, before)
            continue
        got = dst[: tiles * stores * words].view(tiles, stores, 512, 4).cpu().numpy()
        want = np.zeros((tiles, 512, 4), dtype=np.int32)
        want[:, :, 0] = np.arange(512)[None, :]
        want[:, :, 1] = np.arange(tiles)[:, None]
        if loads:
            x = src[: tiles * loads * words].view(tiles, loads, 512, 4).cpu().numpy()
            for i in range(loads):
                want ^= x[:, i]
        for j in range(stores):
            assert np.array_equal(got[:, j], want), (tiles, loads, stores, j)
        assert torch.equal(dst[tiles * stores * words:], before[tiles * stores * words:])
