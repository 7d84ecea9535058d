"""Stream pieces rebuilt from library routines, used only to pin the reference CPU codec.

Each piece of the fZ-light definition (Section 3.3 of the paper) reduces to a textbook or
library routine: the mid-tread uniform quantiser is numpy.rint on float64, the code length
is Python's int.bit_length, block positions are numpy.cumsum, plane words are
numpy.packbits(bitorder="little").  The reference codec must agree with every one of them.
"""
import struct

import numpy as np


def step(abs_eb):
    return float(np.float32(abs_eb)) * 63.0 / 32.0


def codes(x, abs_eb):
    inv = 1.0 / step(abs_eb)
    return np.rint(np.asarray(x, np.float32).astype(np.float64) * inv).astype(np.int64)


def recon(q, abs_eb):
    return (np.asarray(q, np.int64).astype(np.float64) * step(abs_eb)).astype(np.float32)


def pad16(v):
    return (v + 15) // 16 * 16


def blocks_of(q):
    q = np.asarray(q, np.int64)
    n = q.size
    nb = (n + 31) // 32
    if n == 0:
        return np.zeros((0, 32), np.int64)
    qp = np.concatenate([q, np.full(nb * 32 - n, q[-1], np.int64)]).reshape(nb, 32)
    return qp


def stream_from_codes(q, abs_eb, nsum=1, indexed=False):
    q = np.asarray(q, np.int64)
    n = q.size
    qp = blocks_of(q)
    nb = qp.shape[0]
    d = np.diff(qp, axis=1, prepend=qp[:, :1])          # first delta is 0
    mag = np.abs(d)
    widths = np.array([int(m).bit_length() for m in mag.max(axis=1)] if nb else [], np.int64)
    sizes = np.where(widths > 0, 4 * (1 + widths), 0)
    offsets = np.concatenate([[0], np.cumsum(sizes)])[:-1] if nb else np.zeros(0, np.int64)
    payload = bytearray()
    for b in range(nb):
        w = int(widths[b])
        if w == 0:
            continue
        assert len(payload) == offsets[b]
        payload += np.packbits((d[b] < 0).astype(np.uint8), bitorder="little").tobytes()
        for p in range(w):
            payload += np.packbits(((mag[b] >> p) & 1).astype(np.uint8), bitorder="little").tobytes()
    # indexed variant: the payload word offset of every 64th block, from the same cumsum
    ix = b""
    version = 1
    if indexed:
        nseg = (nb + 63) // 64
        entries = np.concatenate([offsets[::64], [len(payload)]]) // 4          # nseg starts and the payload size
        ix = entries.astype("<u4").tobytes().ljust(pad16(4 * (nseg + 1)), b"\0")
        version = 3 if nb and widths.max() > 15 else 2
    total = 32 + pad16(nb) + pad16(4 * nb) + len(ix) + len(payload)
    eb_bits = int(np.float32(abs_eb).view(np.uint32))
    head = struct.pack("<IHBBQIIQ", 0x314C435A, version, 5, 6, n, eb_bits, nsum, total)
    wt = widths.astype(np.uint8).tobytes().ljust(pad16(nb), b"\0")
    ot = qp[:, 0].astype("<i4").tobytes().ljust(pad16(4 * nb), b"\0") if nb else b""
    return np.frombuffer(head + ix + wt + ot + bytes(payload), np.uint8), widths, offsets
