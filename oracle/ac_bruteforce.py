"""Exact arithmetic coding with unbounded integers.  TEST INFRASTRUCTURE ONLY.

A brute-force yardstick for the rANS core on tiny inputs: the interval
[low, low+width) / den is narrowed symbol by symbol with no renormalisation and
no rounding, and the message is the shortest bit string all of whose continuations
stay inside the final interval (a dyadic interval [b, b+1) / 2^bits contained in
it).  Its length is ceil(-log2 prod_t(f_t / 2^M)) or one bit more, which is
the code length that an entropy coder approaches (Sec. 2, eq. (1), and the
source-coding bound used in App. A, eq. (13) of arXiv 2206.05279).

The tables are supplied by the caller: ``cdf_fn(t, decoded_prefix)`` returns the
257 cumulative counts C_t(0..256) of position t, which may depend on the symbols
already decoded (the channel conditioning does).
"""
from __future__ import annotations

from typing import Callable, List, Sequence, Tuple

CdfFn = Callable[[int, Sequence[int]], Sequence[int]]


def encode(symbols: Sequence[int], cdf_fn: CdfFn, prec_bits: int) -> Tuple[int, int]:
    """Returns (bits, value): the message is the `bits`-bit binary fraction value / 2^bits."""
    low, width, den = 0, 1, 1
    for t, x in enumerate(symbols):
        cdf = cdf_fn(t, symbols[:t])
        c, f = int(cdf[x]), int(cdf[x + 1]) - int(cdf[x])
        assert f > 0
        low = (low << prec_bits) + width * c
        width = width * f
        den <<= prec_bits
    bits = 0
    while True:
        # smallest b with b / 2^bits >= low / den
        b = -((-low << bits) // den)
        if (b + 1) * den <= (low + width) << bits:
            return bits, b
        bits += 1


def decode(bits: int, value: int, count: int, cdf_fn: CdfFn, prec_bits: int) -> List[int]:
    low, width, den = 0, 1, 1
    out: List[int] = []
    for t in range(count):
        cdf = cdf_fn(t, out)
        # position of the message inside the current interval, in units of 1/2^M of it
        num = (value * den << prec_bits) - (low << prec_bits << bits)
        slot = num // (width << bits)
        assert 0 <= slot < (1 << prec_bits)
        x = 0
        while int(cdf[x + 1]) <= slot:
            x += 1
        out.append(x)
        c, f = int(cdf[x]), int(cdf[x + 1]) - int(cdf[x])
        low = (low << prec_bits) + width * c
        width = width * f
        den <<= prec_bits
    return out
