"""Seeded synthetic inputs for the table-driven coder: integer probability masses for D
distributions and, per piece, symbols with the index of the distribution each was drawn from.

This module holds NO arithmetic of the coding method.  The recipe is the one the paper states
for its coder measurements (arXiv 2206.05279, Sec. 4.3 and the table comparing rANS with ANS-AI
in the appendix): fix D logistic laws, pick one uniformly at random for every symbol, sample the
symbol from it; pieces of 1000 symbols in 0..255 with the index in 0..7.  The laws are centred
at 128 (Sec. 3.3 codes residuals re-centred there), their scales spread geometrically.

Pieces are drawn in fixed blocks, each from its own seed, so the first k pieces of a workload
do not depend on how many are requested.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

BASE_SEED = 20220605 + 100
BLOCK_PIECES = 4096


@dataclass
class PieceWorkload:
    name: str
    prec_bits: int
    mass: np.ndarray  # uint32 [D, X], rows sum to 2^prec_bits, every entry >= 1
    sym: np.ndarray   # uint8 [pieces, count]
    dist: np.ndarray  # uint8 [pieces, count]

    @property
    def pieces(self) -> int:
        return self.sym.shape[0]

    @property
    def count(self) -> int:
        return self.sym.shape[1]

    @property
    def symbols(self) -> int:
        return self.sym.size


def logistic_masses(prec_bits: int, num_dist: int, num_sym: int = 256, s_min: float = 0.7,
                    s_max: float = 16.0) -> np.ndarray:
    """Integer masses of num_dist logistic laws centred at num_sym/2, cut to [0, num_sym):
    one count for every symbol plus a share of the remaining 2^M - X counts given by the
    logistic CDF at the half-integer edges (largest peak stays below one half)."""
    top = 1 << prec_bits
    assert top >= 2 * num_sym, "need room for one count per symbol"
    if num_dist == 1:
        scales = np.array([np.sqrt(s_min * s_max)])
    else:
        scales = s_min * (s_max / s_min) ** (np.arange(num_dist) / (num_dist - 1))
    edges = np.arange(num_sym + 1, dtype=np.float64) - 0.5 - num_sym / 2
    out = np.zeros((num_dist, num_sym), dtype=np.uint32)
    for d, s in enumerate(scales):
        cdf = 1.0 / (1.0 + np.exp(-edges / s))
        cdf[0], cdf[-1] = 0.0, 1.0
        cut = np.rint(cdf * (top - num_sym)).astype(np.int64)
        out[d] = 1 + np.diff(cut)
    assert (out.sum(axis=1) == top).all() and out.min() >= 1
    return out


def random_masses(rng: np.random.Generator, prec_bits: int, num_dist: int, num_sym: int,
                  concentration: float = 0.3) -> np.ndarray:
    """Arbitrary masses (Dirichlet shares of the counts left after one per symbol); small
    concentrations give rows dominated by one symbol."""
    top = 1 << prec_bits
    assert top >= num_sym
    out = np.zeros((num_dist, num_sym), dtype=np.uint32)
    for d in range(num_dist):
        share = rng.dirichlet(np.full(num_sym, concentration))
        out[d] = 1 + rng.multinomial(top - num_sym, share)
    return out


def index_stream_masses(prec_bits: int, num_sym: int = 256, exponent: float = 1.0, seed: int = 7) -> np.ndarray:
    """One static law over num_sym codebook indices, for the stream of vector indices (Sec. 3.1:
    the indices go through the same coder; the paper does not give their distribution): Zipf-like
    shares over a seeded permutation of the indices, one count per index plus a share of the rest."""
    top = 1 << prec_bits
    assert top >= 2 * num_sym
    rng = np.random.Generator(np.random.PCG64(seed))
    share = 1.0 / (1.0 + np.arange(num_sym)) ** exponent
    share = share[rng.permutation(num_sym)]
    cut = np.rint(np.concatenate([[0.0], np.cumsum(share / share.sum())]) * (top - num_sym)).astype(np.int64)
    out = (1 + np.diff(cut)).astype(np.uint32)[None, :]
    assert out.sum() == top and out.min() >= 1
    return out


def _inverse_table(mass: np.ndarray) -> np.ndarray:
    """[D, 2^M] symbol whose count interval holds u (inverse-CDF sampling)."""
    return np.stack([np.repeat(np.arange(mass.shape[1], dtype=np.uint8), row) for row in mass])


def _draw_block(seed: int, block: int, rows: int, count: int, inv: np.ndarray, uniform_sym: bool):
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, block])))
    num_dist, top = inv.shape
    dist = rng.integers(0, num_dist, size=(BLOCK_PIECES, count), dtype=np.uint8)[:rows]
    u = rng.integers(0, top, size=(BLOCK_PIECES, count), dtype=np.uint16)[:rows]
    if uniform_sym:
        x = int(inv.max()) + 1
        sym = (u.astype(np.uint32) * x // top).astype(np.uint8)
    else:
        sym = inv.reshape(-1)[dist.astype(np.intp) * top + u]
    return sym, dist


def draw_pieces(mass: np.ndarray, prec_bits: int, pieces: int, count: int, seed: int = BASE_SEED,
                uniform_sym: bool = False, threads: int = 8):
    """sym, dist uint8 [pieces, count].  uniform_sym draws the symbols uniformly instead of
    from their law (the coder must stay lossless on data its model does not fit)."""
    inv = _inverse_table(mass)
    assert inv.shape[1] == 1 << prec_bits
    blocks = (pieces + BLOCK_PIECES - 1) // BLOCK_PIECES
    sym = np.empty((pieces, count), dtype=np.uint8)
    dist = np.empty((pieces, count), dtype=np.uint8)

    def job(b):
        lo = b * BLOCK_PIECES
        rows = min(BLOCK_PIECES, pieces - lo)
        s, d = _draw_block(seed, b, rows, count, inv, uniform_sym)
        sym[lo:lo + rows], dist[lo:lo + rows] = s, d

    if blocks <= 1 or threads <= 1:
        for b in range(blocks):
            job(b)
    else:
        with ThreadPoolExecutor(max_workers=threads) as pool:
            list(pool.map(job, range(blocks)))
    return sym, dist


# The paper's coder measurement (Sec. 4.3): 10^6 pieces of 1000 symbols, 8 distributions.
PIECE_CONFIGS = {
    0: dict(name="pieces0: 4096 x 1000, D=8, M=12", pieces=4096, count=1000, num_dist=8, prec_bits=12),
    1: dict(name="pieces1: 1,000,000 x 1000, D=8, M=12", pieces=1000000, count=1000, num_dist=8, prec_bits=12),
    # The stream of vector indices (Sec. 3.1; the "Coder Decode" phase of the per-phase table): one
    # piece per 32x32 image = its 16x16 codebook indices, one static law, as many images as that table.
    2: dict(name="index stream: 1,000,000 x 256 indices, K=256, D=1, M=12", pieces=1000000, count=256,
            num_dist=1, prec_bits=12),
}


def make_piece_workload(cfg: int, pieces: int | None = None, threads: int = 8) -> PieceWorkload:
    c = PIECE_CONFIGS[cfg]
    n = c["pieces"] if pieces is None else int(pieces)
    mass = index_stream_masses(c["prec_bits"]) if cfg == 2 else logistic_masses(c["prec_bits"], c["num_dist"])
    sym, dist = draw_pieces(mass, c["prec_bits"], n, c["count"], seed=BASE_SEED + cfg, threads=threads)
    return PieceWorkload(c["name"], c["prec_bits"], mass, sym, dist)
