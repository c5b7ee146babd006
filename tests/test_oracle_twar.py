"""Pins of the Three-Way AR transform's CPU reference (arXiv 2206.05279, Sec. 3.1 eqs. (2)-(4)):
a hand-worked example, closed forms for special weights (the plane predictor, the PNG "Sub"
filter, G - R), exact invertibility, and an independent vectorised forward pass."""
import os

import numpy as np
import pytest

from oracle import twar_oracle as to

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "twar_worked_example.txt")
ONE = 1 << 14


def q(values):
    return [[int(round(float(v) * ONE)) for v in row] for row in values]


def params(weights, bias=(0, 0, 0)):
    return to.make_params(q(weights), [int(round(float(b) * ONE)) for b in bias])


def read_golden():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        out[key] = [float(v) for v in vals]
    return out


def test_worked_example():
    g = read_golden()
    img = np.array(g["image"], dtype=np.uint8).reshape(1, 2, 2, 3)
    for case in "ab":
        p = params(np.array(g["weights_" + case]).reshape(3, 3), g["bias_" + case])
        res = to.forward(p, img)
        assert res.reshape(-1).tolist() == [int(v) for v in g["residual_" + case]], case
        assert np.array_equal(to.inverse(p, res), img)
    pb_ = params(np.array(g["weights_b"]).reshape(3, 3), g["bias_b"])
    assert to.predict(pb_, 0, 0, 12, 15) == 15
    assert to.predict(params([[-1, 0, 0], [0, 0, 0], [0, 0, 0]]), 0, 5, 0, 0) == 0
    assert to.predict(params([[1, 1, 1], [0, 0, 0], [0, 0, 0]]), 0, 255, 255, 255) == 255


def test_zero_weights_leave_the_image():
    rng = np.random.default_rng(1)
    img = rng.integers(0, 256, (3, 5, 7, 3), dtype=np.uint8)
    p = params(np.zeros((3, 3)))
    assert np.array_equal(to.forward(p, img), img)
    assert np.array_equal(to.inverse(p, img), img)
    # a bias alone shifts every subpixel by the same amount (mod 256)
    p = params(np.zeros((3, 3)), (3, 100, 255))
    assert np.array_equal(to.forward(p, img), (img.astype(np.int64) - np.array([3, 100, 255])).astype(np.uint8))


def test_plane_predictor_cancels_an_affine_image():
    """up + left - upleft reproduces a + b*u + c*v exactly: the residual is zero off the border,
    the column step on the first row, the row step on the first column."""
    h, w = 9, 11
    u, v = np.meshgrid(np.arange(h), np.arange(w), indexing="ij")
    plane = (7 + 5 * u + 3 * v).astype(np.uint8)                # stays below 256
    img = np.stack([plane, plane, plane], axis=-1)[None]
    p = params([[-1, 1, 1], [0, 0, 0], [0, 0, 0]])
    r = to.forward(p, img)[0, :, :, 0].astype(np.int64)
    assert (r[1:, 1:] == 0).all()
    assert r[0, 0] == 7 and (r[0, 1:] == 3).all() and (r[1:, 0] == 5).all()


def test_left_difference_and_channel_difference():
    rng = np.random.default_rng(2)
    img = rng.integers(0, 256, (2, 6, 8, 3), dtype=np.uint8)
    x = img.astype(np.int64)
    p = params([[0, 0, 1], [0, 0, 1], [1, 0, 0]])               # R - left R, G - R, B - left B
    r = to.forward(p, img).astype(np.int64)
    left = np.concatenate([np.zeros_like(x[:, :, :1]), x[:, :, :-1]], axis=2)
    assert np.array_equal(r[..., 0], (x[..., 0] - left[..., 0]) % 256)
    assert np.array_equal(r[..., 1], (x[..., 1] - x[..., 0]) % 256)
    assert np.array_equal(r[..., 2], (x[..., 2] - left[..., 2]) % 256)
    p = params([[0, 1, 0], [0, 1, 0], [0, 1, 0]])               # R - up R, G - left R, B - left G
    r = to.forward(p, img).astype(np.int64)
    up = np.concatenate([np.zeros_like(x[:, :1]), x[:, :-1]], axis=1)
    assert np.array_equal(r[..., 0], (x[..., 0] - up[..., 0]) % 256)
    assert np.array_equal(r[..., 1], (x[..., 1] - left[..., 0]) % 256)
    assert np.array_equal(r[..., 2], (x[..., 2] - left[..., 1]) % 256)


def vector_forward(weights_q, bias_q, img):
    """Forward pass from shifted copies of the image (no loops over pixels)."""
    x = img.astype(np.int64)
    pad = np.pad(x, ((0, 0), (1, 0), (1, 0), (0, 0)))
    ul, up, left, cur = pad[:, :-1, :-1], pad[:, :-1, 1:], pad[:, 1:, :-1], pad[:, 1:, 1:]
    ctx = [(ul[..., 0], up[..., 0], left[..., 0]), (left[..., 1], left[..., 0], cur[..., 0]),
           (left[..., 2], left[..., 1], cur[..., 1])]
    out = np.zeros_like(x)
    for c in range(3):
        acc = sum(int(weights_q[c][k]) * ctx[c][k] for k in range(3)) + int(bias_q[c]) + (1 << 13)
        out[..., c] = (cur[..., c] - np.clip(acc >> 14, 0, 255)) % 256
    return out.astype(np.uint8)


@pytest.mark.parametrize("seed", range(6))
def test_random_weights_forward_and_round_trip(seed):
    rng = np.random.default_rng(100 + seed)
    wq = rng.integers(-ONE, ONE + 1, (3, 3)) if seed else np.full((3, 3), 32767)
    bq = rng.integers(-64 * ONE, 64 * ONE, 3)
    n, h, w = [(1, 1, 1), (2, 1, 9), (2, 9, 1), (3, 32, 32), (1, 17, 40), (2, 5, 5)][seed]
    img = rng.integers(0, 256, (n, h, w, 3), dtype=np.uint8)
    p = to.make_params(wq.tolist(), bq.tolist())
    res = to.forward(p, img)
    assert np.array_equal(res, vector_forward(wq, bq, img))
    assert np.array_equal(to.inverse(p, res), img)


def test_residual_of_a_smooth_image_is_cheaper():
    """What the transform is for: on a smooth image the residual's entropy is far below the image's."""
    h = w = 64
    u, v = np.meshgrid(np.arange(h), np.arange(w), indexing="ij")
    rng = np.random.default_rng(3)
    base = 128 + 60 * np.sin(u / 9.0) + 50 * np.cos(v / 7.0)
    img = np.clip(np.stack([base, base * 0.9 + 10, base * 0.8 + 30], -1) + rng.normal(0, 1.5, (h, w, 3)), 0, 255)
    img = img.astype(np.uint8)[None]
    p = params([[-1, 1, 1], [0.5, -0.5, 1], [0.5, -0.5, 1]])
    res = to.forward(p, img)

    def entropy(a):
        c = np.bincount(a.reshape(-1), minlength=256) / a.size
        c = c[c > 0]
        return float(-(c * np.log2(c)).sum())
    assert entropy(res) < entropy(img) - 2.0
