"""Helpers for the GPU parity tests: run the HIP library through its C ABI on torch buffers
and hand back numpy arrays that can be compared with the reference CPU codec."""
import numpy as np
import torch

import paper_2502_18554_amd as _zc
from paper_2502_18554_amd.binding import ZC_CHAINS_COHERENT, ZC_STREAM_PLAIN, ZC_TILES_BY_TICKET

DEV = "cuda:0"

INDEXED = False          # the stream variant the tests are run on (the reference is set to the same; it starts out plain)
TICKETS = False          # tiles handed out by tickets
COHERENT = False         # the look-back reads every descriptor with device-coherent loads

# calls that take the stream variant only, and calls that also take the way tiles are handed out
_READERS = {"zc_compress_bound", "zc_decompress", "zc_decompress_average", "zc_decompress_range", "zc_decompress_many",
            "zc_debug_block_offsets"}
_WRITERS = {"zc_compress", "zc_compress_part", "zc_reduce_compressed", "zc_reduce_compressed_op", "zc_reduce_step",
            "zc_reduce_step_op", "zc_reduce_compressed_part", "zc_reduce_step_part"}


def flags(writer=True):
    """The flags argument for the stream variant (and tile hand-out) the tests are running under."""
    return ((0 if INDEXED else ZC_STREAM_PLAIN) | (ZC_TILES_BY_TICKET if writer and TICKETS else 0)
            | (ZC_CHAINS_COHERENT if writer and COHERENT else 0))


class _Library:
    """The package, with the flags of the variant under test filled in wherever a call takes flags: the
    library itself has no setting for them."""

    def __getattr__(self, name):
        f = getattr(_zc, name)
        if name not in _READERS and name not in _WRITERS:
            return f

        def call(*args, **kwargs):
            kwargs.setdefault("flags", flags(name in _WRITERS))
            return f(*args, **kwargs)
        return call


zc = _Library()


def set_variant(zcref, indexed):
    """The library calls made through `zc` and the reference codec write and accept plain (False) or
    indexed (True) streams from here on."""
    global INDEXED
    INDEXED = bool(indexed)
    if zcref is not None:
        zcref.set_indexed(INDEXED)


def set_tickets(on):
    global TICKETS
    TICKETS = bool(on)


def set_coherent(on):
    global COHERENT
    COHERENT = bool(on)


def pad16(v):
    return (v + 15) // 16 * 16


def index_bytes(nb):
    return pad16(4 * ((nb + 63) // 64 + 1)) if INDEXED else 0


def widths_begin(nb):
    return 32 + index_bytes(nb)


def tables_end(nb):
    return widths_begin(nb) + pad16(nb) + pad16(4 * nb)


def widths_of(s, nb):
    return s[widths_begin(nb):widths_begin(nb) + nb]


def to_dev(x):
    if isinstance(x, np.ndarray):
        x = torch.from_numpy(np.ascontiguousarray(x))
    return x.to(DEV).contiguous()


def workspace(n, k=1):
    return torch.empty(zc.zc_workspace_bytes(n, k) + 16, dtype=torch.uint8, device=DEV)


def gpu_compress(x, eb, out_cap=None, ws=None):
    """-> (status, stream bytes (numpy uint8), total_bytes)"""
    d_in = to_dev(x)
    n = d_in.numel()
    cap = zc.zc_compress_bound(n) if out_cap is None else out_cap
    d_out = torch.full((cap + 64,), 0xA5, dtype=torch.uint8, device=DEV)
    ws = workspace(n) if ws is None else ws
    st, total = zc.zc_compress(d_in, n, float(eb), d_out, ws, out_cap=cap)
    assert bool((d_out[cap:] == 0xA5).all()), "wrote past out_cap"
    torch.cuda.synchronize()
    out = d_out[: min(total, cap)].cpu().numpy() if st in (_zc.binding.ZC_OK, _zc.binding.ZC_ERR_BOUND) else None
    return st, out, total


def gpu_decompress(stream, n_cap, in_bytes=None, ws=None, average=False):
    """-> (status, float32 numpy array of n values, n)"""
    d_in = to_dev(stream)
    in_bytes = d_in.numel() if in_bytes is None else in_bytes
    d_out = torch.full((max(n_cap, 4),), float("nan"), dtype=torch.float32, device=DEV)
    ws = workspace(max(n_cap, 1)) if ws is None else ws
    fn = zc.zc_decompress_average if average else zc.zc_decompress
    st, n = fn(d_in, in_bytes, d_out, ws, out_cap_elems=n_cap)
    torch.cuda.synchronize()
    return st, (d_out[:n].cpu().numpy() if st == _zc.binding.ZC_OK else None), n


def gpu_reduce(streams, n, out_cap=None, ws=None, op=None):
    """-> (status, stream bytes, total_bytes)"""
    d_chunks = [to_dev(s) for s in streams]
    cap = zc.zc_compress_bound(n) if out_cap is None else out_cap
    d_out = torch.full((cap + 64,), 0x5A, dtype=torch.uint8, device=DEV)
    ws = workspace(max(n, 1), len(streams)) if ws is None else ws
    if op is None:
        st, total = zc.zc_reduce_compressed(d_chunks, [c.numel() for c in d_chunks], d_out, ws, out_cap=cap)
    else:
        st, total = zc.zc_reduce_compressed_op(d_chunks, [c.numel() for c in d_chunks], op, d_out, ws, out_cap=cap)
    assert bool((d_out[cap:] == 0x5A).all()), "wrote past out_cap"
    torch.cuda.synchronize()
    return st, (d_out[: min(total, cap)].cpu().numpy() if st == _zc.binding.ZC_OK else None), total


def gpu_decompress_many(streams, n_caps, ws=None):
    """-> (status, [float32 arrays], [n])"""
    d_chunks = [to_dev(s) for s in streams]
    d_outs = [torch.full((max(c, 4) + 4,), float("nan"), dtype=torch.float32, device=DEV) for c in n_caps]
    ws = workspace(max(max(n_caps), 1), len(streams)) if ws is None else ws
    st, ns = zc.zc_decompress_many(d_chunks, [c.numel() for c in d_chunks], d_outs, ws, out_cap_elems=n_caps)
    torch.cuda.synchronize()
    for o, c in zip(d_outs, n_caps):
        assert bool(torch.isnan(o[max(c, 4):]).all()), "wrote past out_cap_elems"
    return st, [o.cpu().numpy() for o in d_outs], ns


def gpu_reduce_step(stream, local, out_cap=None, ws=None, n_local=None, op=None):
    """-> (status, stream bytes, total_bytes)"""
    d_in = to_dev(stream)
    d_loc = to_dev(np.ascontiguousarray(local, dtype=np.float32)) if len(local) else torch.zeros(4, device=DEV)
    n = len(local) if n_local is None else n_local
    cap = zc.zc_compress_bound(n) if out_cap is None else out_cap
    d_out = torch.full((cap + 64,), 0x3C, dtype=torch.uint8, device=DEV)
    ws = workspace(max(n, 1)) if ws is None else ws
    if op is None:
        st, total = zc.zc_reduce_step(d_in, d_in.numel(), d_loc, n, d_out, ws, out_cap=cap)
    else:
        st, total = zc.zc_reduce_step_op(d_in, d_in.numel(), d_loc, n, op, d_out, ws, out_cap=cap)
    assert bool((d_out[cap:] == 0x3C).all()), "wrote past out_cap"
    torch.cuda.synchronize()
    ok = st in (_zc.binding.ZC_OK, _zc.binding.ZC_ERR_BOUND)
    return st, (d_out[: min(total, cap)].cpu().numpy() if ok else None), total


def first_diff(a, b):
    a = np.asarray(a); b = np.asarray(b)
    if a.shape != b.shape:
        return f"shape {a.shape} vs {b.shape}"
    d = np.nonzero(a != b)[0]
    return "equal" if d.size == 0 else f"{d.size} differ, first at {d[0]}: {a[d[0]]} vs {b[d[0]]}"
