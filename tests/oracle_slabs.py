"""The unchanged single-threaded oracle run over a whole workload, slab by slab in a thread pool.

Lanes are independent streams (pinned on the CPU: a batch's payload is the concatenation of its
lanes' bytes, the offset table their running sum), so a slab of whole images that starts and ends
on a lane boundary gives exactly that part of the whole container's payload.  The header and the
offset table of the whole container are written here from the format's definition, not taken from
any implementation."""
import os
import struct
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from oracle import pilc_oracle as orc


def _slab_images(wl, threads):
    """Image ranges [a, b) that start and end on lane boundaries, about `threads` x 4 of them."""
    n, h, w, m, mode, la, lb = wl.geom
    unit = max(1, la // (h * w)) if mode == 0 else 1      # images per lane when lanes span images
    units = -(-n // unit)
    per = max(1, -(-units // (threads * 4))) * unit
    return [(a, min(a + per, n)) for a in range(0, n, per)]


def whole_container(wl, threads=None):
    """Container bytes (uint8 array) the oracle gives for the whole workload."""
    n, h, w, m, mode, la, lb = wl.geom
    threads = threads or max(1, min(16, os.cpu_count() or 1))
    orc.lib()

    def one(ab):
        a, b = ab
        sl = slice(a, b)
        g = orc.make_geom(b - a, h, w, m, mode, la, lb)
        rc, coded = orc.encode(g, wl.img[sl], wl.mu[sl], wl.log_scale[sl], wl.chan_coef[sl])
        assert rc == orc.OK, "oracle encode of images %d..%d: rc %d" % (a, b, rc)
        lanes = struct.unpack_from("<I", coded, 40)[0]
        offs = np.frombuffer(coded, dtype="<u4", count=lanes + 1, offset=64)
        return np.diff(offs.astype(np.int64)), coded[64 + 4 * (lanes + 1):]

    with ThreadPoolExecutor(max_workers=threads) as pool:
        parts = list(pool.map(one, _slab_images(wl, threads)))
    sizes = np.concatenate([p[0] for p in parts])
    lanes = sizes.size
    payload = int(sizes.sum())
    assert payload < (1 << 32)
    offs = np.zeros(lanes + 1, dtype="<u4")
    offs[1:] = np.cumsum(sizes)
    head = struct.pack("<4s11IQQ", b"PILC", 1, n, h, w, 3, m, mode, la, lb, lanes, 0, payload, 0)
    assert len(head) == 64
    return np.concatenate([np.frombuffer(head, dtype=np.uint8), offs.view(np.uint8)] + [p[1] for p in parts])


def whole_mix_container(wl, threads=None):
    """As whole_container for a mixture workload (magic "PMIX", K in header word 11)."""
    from oracle import mix_oracle as mx

    n, h, w, m, mode, la, lb = wl.geom
    assert mode == 1 or (h * w) % la == 0, "lanes must not span images here"
    threads = threads or max(1, min(16, os.cpu_count() or 1))
    per = max(1, -(-n // (threads * 4)))
    mx.lib()

    def one(a):
        b = min(a + per, n)
        sl = slice(a, b)
        g = orc.make_geom(b - a, h, w, m, mode, la, lb)
        rc, coded = mx.encode(g, wl.num_comp, wl.img[sl], wl.mu[sl], wl.log_scale[sl], wl.weight[sl],
                              wl.chan_coef[sl])
        assert rc == mx.OK, "mixture oracle encode of images %d..%d: rc %d" % (a, b, rc)
        lanes = struct.unpack_from("<I", coded, 40)[0]
        offs = np.frombuffer(coded, dtype="<u4", count=lanes + 1, offset=64)
        return np.diff(offs.astype(np.int64)), coded[64 + 4 * (lanes + 1):]

    with ThreadPoolExecutor(max_workers=threads) as pool:
        parts = list(pool.map(one, range(0, n, per)))
    sizes = np.concatenate([p[0] for p in parts])
    lanes, payload = sizes.size, int(sizes.sum())
    offs = np.zeros(lanes + 1, dtype="<u4")
    offs[1:] = np.cumsum(sizes)
    head = struct.pack("<4s11IQQ", b"PMIX", 1, n, h, w, 3, m, mode, la, lb, lanes, wl.num_comp, payload, 0)
    return np.concatenate([np.frombuffer(head, dtype=np.uint8), offs.view(np.uint8)] + [p[1] for p in parts])


def whole_piece_container(wl, threads=None):
    """Container of the table-driven coder for a whole piece workload: pieces are independent, so
    slabs of pieces are encoded by the reference in a thread pool and their records concatenated."""
    from oracle import ansai_oracle as ao

    threads = threads or max(1, min(16, os.cpu_count() or 1))
    pieces, count = wl.sym.shape
    d, x = wl.mass.shape
    per = max(1, -(-pieces // (threads * 4)))
    ao.lib()

    def one(a):
        b = min(a + per, pieces)
        rc, coded = ao.encode(wl.prec_bits, wl.mass, wl.sym[a:b], wl.dist[a:b])
        assert rc == ao.OK, "piece oracle encode of %d..%d: rc %d" % (a, b, rc)
        offs = np.frombuffer(coded, dtype="<u4", count=b - a + 1, offset=64)
        return np.diff(offs.astype(np.int64)), coded[64 + 4 * (b - a + 1):]

    with ThreadPoolExecutor(max_workers=threads) as pool:
        parts = list(pool.map(one, range(0, pieces, per)))
    sizes = np.concatenate([p[0] for p in parts])
    payload = int(sizes.sum())
    offs = np.zeros(pieces + 1, dtype="<u4")
    offs[1:] = np.cumsum(sizes)
    head = struct.pack("<4s6I20xQQ", b"PANS", 1, pieces, count, wl.prec_bits, d, x, payload, 0)
    assert len(head) == 64
    return np.concatenate([np.frombuffer(head, dtype=np.uint8), offs.view(np.uint8)] + [p[1] for p in parts])
