"""Seeded synthetic inputs for the mixture-of-logistics coder.

Serves the oracle, the tests and the benchmark alike and holds none of the method's arithmetic:
it only draws images and parameter arrays.  The images are those of `synth.make_workload`; the
mixture parameters stand in for the output of a PixelCNN++-style head, which Sec. 2 of
arXiv 2206.05279 names (a mixture of ten logistic laws per symbol) without giving one:

* component 0 of a subpixel is the single-law parameter set of the base workload (mean near the
  true value);
* the other K - 1 components have means at the true value plus N(0, 24^2) (in pixel units,
  clipped to [0, 255.996]) and log-scales uniform in [0, 3];
* a pixel's K weights are a flat Dirichlet draw with component 0 boosted by 1, quantised to
  Q0.15 so that they sum to 2^15 exactly (the rounding remainder goes to the largest weight).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

from . import synth


@dataclass
class MixWorkload:
    name: str
    n: int
    h: int
    w: int
    prec_bits: int
    lane_mode: int
    lane_a: int
    lane_b: int
    num_comp: int
    img: np.ndarray        # [n,h,w,3]   u8
    mu: np.ndarray         # [n,h,w,3,K] u16 Q8.8
    log_scale: np.ndarray  # [n,h,w,3,K] i16 Q4.12
    weight: np.ndarray     # [n,h,w,K]   u16 Q0.15, sums to 32768 per pixel
    chan_coef: np.ndarray  # [n,3]       i16 Q2.14

    @property
    def geom(self) -> Tuple[int, int, int, int, int, int, int]:
        return (self.n, self.h, self.w, self.prec_bits, self.lane_mode, self.lane_a, self.lane_b)

    @property
    def subpixels(self) -> int:
        return self.n * self.h * self.w * 3


def quantise_weights(p: np.ndarray) -> np.ndarray:
    """Rows of non-negative reals summing to 1 -> u16 rows summing to 32768."""
    q = np.floor(p * 32768.0).astype(np.int64)
    rest = 32768 - q.sum(axis=-1)
    top = np.argmax(q, axis=-1)
    flat = q.reshape(-1, q.shape[-1])
    flat[np.arange(flat.shape[0]), top.reshape(-1)] += rest.reshape(-1)
    assert q.min() >= 0 and q.max() <= 32768 and np.all(q.sum(axis=-1) == 32768)
    return q.astype(np.uint16)


def _params_block(rng: np.random.Generator, img, base_mu, base_ls, k: int, mu, ls, weight) -> None:
    shape = img.shape
    mu[..., 0] = base_mu
    ls[..., 0] = base_ls
    if k > 1:
        # float32 draws: the values only have to be seeded and plausible
        m = rng.standard_normal(size=shape + (k - 1,), dtype=np.float32)
        m *= np.float32(24.0)
        m += img.astype(np.float32)[..., None]
        np.clip(m, 0.0, 255.996, out=m)
        m *= np.float32(256.0)
        mu[..., 1:] = np.rint(m).astype(np.uint16)
        u = rng.random(size=shape + (k - 1,), dtype=np.float32)
        u *= np.float32(3.0 * 4096.0)
        ls[..., 1:] = np.rint(u).astype(np.int16)
    g = rng.standard_exponential(size=shape[:3] + (k,), dtype=np.float32).astype(np.float64)
    g[..., 0] += 1.0
    weight[...] = quantise_weights(g / g.sum(axis=-1, keepdims=True))


_BLOCK = 64  # images per independently seeded block


def mixture_params(seed_seq: np.random.SeedSequence, base: synth.Workload, num_comp: int,
                   threads: int = 8):
    """Blocks of 64 images, each from its own child seed, drawn in a thread pool: the result does
    not depend on the number of threads."""
    k = int(num_comp)
    shape = base.img.shape
    mu = np.empty(shape + (k,), dtype=np.uint16)
    ls = np.empty(shape + (k,), dtype=np.int16)
    weight = np.empty(shape[:3] + (k,), dtype=np.uint16)
    starts = list(range(0, shape[0], _BLOCK))
    children = seed_seq.spawn(len(starts))

    def work(i):
        sl = slice(starts[i], min(starts[i] + _BLOCK, shape[0]))
        rng = np.random.Generator(np.random.PCG64(children[i]))
        _params_block(rng, base.img[sl], base.mu[sl], base.log_scale[sl], k, mu[sl], ls[sl], weight[sl])

    if threads > 1 and len(starts) > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=threads) as pool:
            list(pool.map(work, range(len(starts))))
    else:
        for i in range(len(starts)):
            work(i)
    return mu, ls, weight


def make_mix_workload(cfg: int, n: int, num_comp: int, *, seed: Optional[int] = None,
                      h: Optional[int] = None, w: Optional[int] = None,
                      prec_bits: Optional[int] = None, lanes_per_image: int = 64) -> MixWorkload:
    """Base workload `cfg` of `synth.make_workload` (first n images) with K-component parameters."""
    base = synth.make_workload(cfg, n, seed=seed, h=h, w=w, prec_bits=prec_bits,
                               lanes_per_image=lanes_per_image)
    mu, ls, weight = mixture_params(
        np.random.SeedSequence([20220605 if seed is None else seed, 77, cfg, num_comp]), base, num_comp)
    return MixWorkload(base.name + "-mix%d" % num_comp, base.n, base.h, base.w, base.prec_bits,
                       base.lane_mode, base.lane_a, base.lane_b, int(num_comp), base.img, mu, ls,
                       weight, base.chan_coef)


def from_base(base: synth.Workload, num_comp: int, seed: int) -> MixWorkload:
    """Mixture parameters around any base workload (edge-case shapes of the tests)."""
    mu, ls, weight = mixture_params(np.random.SeedSequence([seed, 78, num_comp]), base, num_comp)
    return MixWorkload(base.name + "-mix%d" % num_comp, base.n, base.h, base.w, base.prec_bits,
                       base.lane_mode, base.lane_a, base.lane_b, int(num_comp), base.img, mu, ls,
                       weight, base.chan_coef)
