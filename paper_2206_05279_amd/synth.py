"""Seeded synthetic workloads, shaped like the image suites the paper measures on.

This module holds NO arithmetic of the coding method: it only draws images and
distribution parameters.  Both the CPU oracle's tests and the GPU path consume
the arrays it returns, so its details influence bits/subpixel only, never
parity.

The five workloads stand in for CIFAR-sized, ImageNet64-sized and 1080p inputs
(Sec. 4 of arXiv 2206.05279 measures on such suites); their content is
procedural noise, not dataset items.  Images are drawn in fixed blocks, each
from its own seed, so the first k images of a workload do not depend on how
many images are requested.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 20220605


@dataclass
class Workload:
    name: str
    n: int
    h: int
    w: int
    prec_bits: int
    lane_mode: int
    lane_a: int
    lane_b: int
    img: np.ndarray        # uint8  [n,h,w,3]
    mu: np.ndarray         # uint16 [n,h,w,3]  Q8.8
    log_scale: np.ndarray  # int16  [n,h,w,3]  Q4.12
    chan_coef: np.ndarray  # int16  [n,3]      Q2.14

    @property
    def geom(self) -> Tuple[int, int, int, int, int, int, int]:
        return (self.n, self.h, self.w, self.prec_bits, self.lane_mode, self.lane_a, self.lane_b)

    @property
    def subpixels(self) -> int:
        return self.n * self.h * self.w * 3


def _rng(cfg: int, block: int, seed: Optional[int]) -> np.random.Generator:
    base = BASE_SEED + cfg if seed is None else seed
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([base, block])))


def _upsample_axis(n_in: int, n_out: int):
    """Bilinear taps with half-pixel centres and edge clamp."""
    src = (np.arange(n_out) + 0.5) * (n_in / n_out) - 0.5
    i0 = np.floor(src).astype(np.int64)
    frac = src - i0
    return np.clip(i0, 0, n_in - 1), np.clip(i0 + 1, 0, n_in - 1), frac


def _upsample(field: np.ndarray, h: int, w: int) -> np.ndarray:
    """field [b, fh, fw, c] -> [b, h, w, c]."""
    y0, y1, fy = _upsample_axis(field.shape[1], h)
    x0, x1, fx = _upsample_axis(field.shape[2], w)
    fy = fy[None, :, None, None]
    fx = fx[None, None, :, None]
    rows = field[:, y0] * (1.0 - fy) + field[:, y1] * fy
    return rows[:, :, x0] * (1.0 - fx) + rows[:, :, x1] * fx


def _to_u8(x: np.ndarray) -> np.ndarray:
    return np.clip(np.rint(x), 0, 255).astype(np.uint8)


def _params(rng, img: np.ndarray, sigma_mu: float, ls_lo: float, ls_hi: float):
    mu = np.clip(np.rint((img.astype(np.float64) + sigma_mu * rng.standard_normal(img.shape)) * 256.0),
                 0, 65535).astype(np.uint16)
    ls = np.rint(rng.uniform(ls_lo, ls_hi, size=img.shape) * 4096.0).astype(np.int16)
    coef = np.rint(rng.uniform(0.0, 1.0, size=(img.shape[0], 3)) * 16384.0).astype(np.int16)
    return mu, ls, coef


def _block_smooth32(rng, b: int, per_image_sigma: bool):
    field = rng.uniform(0.0, 255.0, size=(b, 8, 8, 3))
    sigma = rng.uniform(2.0, 12.0, size=(b, 1, 1, 1)) if per_image_sigma else 6.0
    img = _to_u8(_upsample(field, 32, 32) + sigma * rng.standard_normal((b, 32, 32, 3)))
    return (img,) + _params(rng, img, 4.0, -1.0, 3.0)


def _block_octaves64(rng, b: int):
    o0 = _upsample(rng.uniform(0.0, 255.0, size=(b, 4, 4, 3)), 64, 64)
    o1 = _upsample(rng.uniform(0.0, 255.0, size=(b, 16, 16, 3)), 64, 64)
    o2 = rng.uniform(0.0, 255.0, size=(b, 64, 64, 3))
    img = _to_u8(0.6 * o0 + 0.3 * o1 + 0.1 * o2 + 5.0 * rng.standard_normal((b, 64, 64, 3)))
    return (img,) + _params(rng, img, 3.0, -1.5, 2.5)


def _block_frames(rng, b: int, h: int, w: int):
    yy = (np.arange(h) / max(h - 1, 1))[None, :, None, None]
    xx = (np.arange(w) / max(w - 1, 1))[None, None, :, None]
    theta = rng.uniform(0.0, 2.0 * np.pi, size=(b, 1, 1, 3))
    v0 = rng.uniform(0.0, 255.0, size=(b, 1, 1, 3))
    v1 = rng.uniform(0.0, 255.0, size=(b, 1, 1, 3))
    # position along the gradient direction, normalised to [0,1]
    proj = np.cos(theta) * xx + np.sin(theta) * yy
    lo = np.minimum(0.0, np.cos(theta)) + np.minimum(0.0, np.sin(theta))
    hi = np.maximum(0.0, np.cos(theta)) + np.maximum(0.0, np.sin(theta))
    base = v0 + (v1 - v0) * (proj - lo) / np.maximum(hi - lo, 1e-9)
    for i in range(b):
        for _ in range(5):
            y0, y1 = np.sort(rng.integers(0, h + 1, size=2))
            x0, x1 = np.sort(rng.integers(0, w + 1, size=2))
            base[i, y0:y1, x0:x1, :] = rng.uniform(0.0, 255.0, size=3)
    img = _to_u8(base + 3.0 * rng.standard_normal((b, h, w, 3)))
    return (img,) + _params(rng, img, 2.0, -2.0, 2.0)


def _block_extreme(rng, b: int, h: int, w: int, random_half: bool):
    coef = np.rint(rng.uniform(0.0, 1.0, size=(b, 3)) * 16384.0).astype(np.int16)
    if random_half:
        img = rng.integers(0, 256, size=(b, h, w, 3), dtype=np.uint8)
        mu = np.full(img.shape, 128 * 256, dtype=np.uint16)
        ls = np.full(img.shape, 4 * 4096, dtype=np.int16)
    else:
        colour = rng.integers(0, 256, size=(b, 1, 1, 3), dtype=np.uint8)
        img = np.broadcast_to(colour, (b, h, w, 3)).copy()
        mu = img.astype(np.uint16) * 256
        ls = np.full(img.shape, -3 * 4096, dtype=np.int16)
    return img, mu, ls, coef


_FULL_N = {0: 64, 1: 50000, 2: 16384, 3: 30, 4: 8192}
_BLOCK = {0: 64, 1: 1024, 2: 256, 3: 1, 4: 16}


def full_size(cfg: int) -> int:
    return _FULL_N[cfg]


def make_workload(cfg: int, n: Optional[int] = None, *, seed: Optional[int] = None,
                  h: Optional[int] = None, w: Optional[int] = None,
                  prec_bits: Optional[int] = None, lanes_per_image: int = 64) -> Workload:
    """Build workload `cfg` (0..4) with its first n images (default: all).

    cfg 3 accepts a reduced frame size (h, w); cfg 4 accepts a reduced image size,
    the frequency precision (12 or 16) and the lanes per image of its sweep.
    For cfg 4 the n images are the first n/2 of the random half followed by the
    first n/2 of the constant half.
    """
    if cfg not in _FULL_N:
        raise ValueError("unknown workload %r" % (cfg,))
    n = _FULL_N[cfg] if n is None else int(n)
    if n <= 0:
        raise ValueError("n must be positive")
    blk = _BLOCK[cfg]
    parts = []
    if cfg == 4:
        hh, ww = h or 256, w or 256
        half = (n + 1) // 2
        for random_half, count, tag in ((True, half, 0), (False, n - half, 1 << 20)):
            for b0 in range(0, count, blk):
                b = min(blk, count - b0)
                parts.append(_block_extreme(_rng(cfg, tag + b0 // blk, seed), blk, hh, ww,
                                            random_half)[0:4])
                parts[-1] = tuple(a[:b] for a in parts[-1])
    else:
        for b0 in range(0, n, blk):
            b = min(blk, n - b0)
            rng = _rng(cfg, b0 // blk, seed)
            if cfg == 0:
                out = _block_smooth32(rng, blk, False)
            elif cfg == 1:
                out = _block_smooth32(rng, blk, True)
            elif cfg == 2:
                out = _block_octaves64(rng, blk)
            else:
                out = _block_frames(rng, blk, h or 1080, w or 1920)
            parts.append(tuple(a[:b] for a in out))
    img, mu, ls, coef = (np.ascontiguousarray(np.concatenate([p[i] for p in parts], axis=0))
                         for i in range(4))
    hh, ww = img.shape[1], img.shape[2]
    if cfg == 0:
        name, m, mode, la, lb = "tiny-smoke-32x32", 14, 0, 32, 0
    elif cfg == 1:
        name, m, mode, la, lb = "cifar-shaped-32x32", 14, 0, 16384, 0
    elif cfg == 2:
        name, m, mode, la, lb = "imagenet64-shaped", 15, 0, 64, 0
    elif cfg == 3:
        name, m, mode, la, lb = "video-1080p-tiles16", 15, 1, 16, 16
    else:
        m = prec_bits or 12
        if (hh * ww) % lanes_per_image:
            raise ValueError("lanes_per_image must divide h*w")
        name, mode, la, lb = "entropy-extreme-M%d-L%d" % (m, lanes_per_image), 0, hh * ww // lanes_per_image, 0
    if prec_bits is not None and cfg != 4:
        m = prec_bits
    return Workload(name, n, hh, ww, m, mode, la, lb, img, mu, ls, coef)


def make_random_case(seed: int, n: int, h: int, w: int, prec_bits: int, lane_mode: int, lane_a: int,
                     lane_b: int = 0, *, wild: bool = False) -> Workload:
    """Small free-form case for edge tests.  `wild` draws parameters over their whole
    16-bit ranges (means at 0/65535, log-scales beyond both clamps, coefficients up
    to +-2) instead of a plausible model output."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, n, h, w])))
    img = rng.integers(0, 256, size=(n, h, w, 3), dtype=np.uint8)
    if wild:
        mu = rng.integers(0, 65536, size=img.shape, dtype=np.uint16)
        mu[rng.random(img.shape) < 0.1] = 0
        mu[rng.random(img.shape) < 0.1] = 65535
        ls = rng.integers(-32768, 32768, size=img.shape).astype(np.int16)
        coef = rng.integers(-32768, 32768, size=(n, 3)).astype(np.int16)
    else:
        mu, ls, coef = _params(rng, img, 6.0, -2.0, 3.0)
    return Workload("random-case", n, h, w, prec_bits, lane_mode, lane_a, lane_b,
                    img, mu, ls, coef)
