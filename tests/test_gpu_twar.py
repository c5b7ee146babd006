"""GPU parity of the Three-Way AR residual transform (Sec. 3.1 eqs. (2)-(4)) against the CPU
reference, through the C ABI: residuals and recovered images byte for byte, on shapes that
cover several images per wavefront, bands of 64 rows, the LDS-tile and the in-place path, and
the workgroup-per-image path for tall images."""
import numpy as np
import pytest
import torch

from oracle import twar_oracle as to
from paper_2206_05279_amd import binding as pb

pytestmark = pytest.mark.gpu

ONE = 1 << 14
SHAPES = [(1, 1, 1), (3, 32, 32), (5, 7, 9), (2, 64, 64), (7, 16, 16), (2, 33, 5), (1, 100, 37),
          (1, 130, 300), (2, 3, 700), (513, 32, 32), (1, 200, 64),
          # taller than a wavefront with rows of whole 16-pixel chunks: a workgroup per image with all
          # bands under way at once; one band and a bit, a band boundary at the last row, three
          # rounds of a workgroup, a full-size frame
          (3, 65, 16), (2, 128, 48), (1, 1600, 32), (2, 1080, 1920),
          # few images taller than 256 rows: bands of an image in workgroups of their own that follow
          # each other through counters in global memory (three bands of 234 rows; nine of 234; two
          # of 193 and two of 129, whose last wavefront has a single row; two full bands of 256)
          (2, 700, 64), (1, 2100, 160), (3, 385, 32), (3, 257, 32), (2, 512, 48),
          # many images with more rows than a workgroup has threads: rounds within a workgroup
          (256, 800, 16),
          # more groups of small images: eight images a group, rows of 27 dwords, an odd number of
          # groups, 17-row images (13 idle threads), many groups with a single-image group at the end
          (9, 8, 8), (40, 32, 36), (11, 64, 64), (100, 17, 16), (24577, 32, 32),
          # tiles copied a byte, 4 bytes or 16 bytes at a time (image sizes 105, 36 and 3960 bytes,
          # the last with 33-row images), each with many groups and a short last one
          (4001, 5, 7), (7001, 3, 4), (1300, 33, 40)]


def models(rng):
    yield "plane", [[-ONE, ONE, ONE], [ONE // 2, -ONE // 2, ONE], [ONE // 2, -ONE // 2, ONE]], [0, 0, 0]
    yield "random", rng.integers(-ONE, ONE + 1, (3, 3)).tolist(), rng.integers(-64 * ONE, 64 * ONE, 3).tolist()
    yield "extreme", [[32767] * 3, [-32768] * 3, [32767, -32768, 1]], [1 << 30, -(1 << 30), 12345]


@pytest.mark.parametrize("shape", SHAPES, ids=["x".join(map(str, s)) for s in SHAPES])
def test_forward_and_inverse_match_the_reference(shape):
    rng = np.random.default_rng(sum(shape))
    img = rng.integers(0, 256, shape + (3,), dtype=np.uint8)
    if shape[1] >= 16:  # some structure, so that predictions matter
        img = (img // 8 + np.linspace(0, 200, shape[2]).astype(np.uint8)[None, None, :, None]).astype(np.uint8)
    d_img = torch.from_numpy(img).cuda()
    for name, wq, bq in models(rng):
        print("shape", shape, "model", name, flush=True)
        ref = to.forward(to.make_params(wq, bq), img)
        p = pb.make_twar_params(wq, bq)
        d_res = torch.full_like(d_img, 0x5A)
        pb.pilc_twar_forward(p, d_img, d_res)
        assert np.array_equal(d_res.cpu().numpy(), ref), name
        d_back = torch.full_like(d_img, 0xA5)
        pb.pilc_twar_inverse(p, d_res, d_back)
        assert np.array_equal(d_back.cpu().numpy(), img), name
        # and the reference's own inverse agrees on a residual that is not a forward image
        noise = rng.integers(0, 256, img.shape, dtype=np.uint8)
        d_noise = torch.from_numpy(noise).cuda()
        pb.pilc_twar_inverse(p, d_noise, d_back)
        assert np.array_equal(d_back.cpu().numpy(), to.inverse(to.make_params(wq, bq), noise)), name


def test_thirty_frames_come_back_every_time():
    """The workload bench.py times (30 frames of 1080 x 1920, five bands each, 150 workgroups that
    follow each other through the image itself): the inverse of the forward transform is the
    image, on five calls in a row into a buffer poisoned before each, compared on the device.  A
    band that read a row of the band above before it was there would pick up the poison."""
    g = torch.Generator().manual_seed(11)
    img = torch.randint(0, 256, (30, 1080, 1920, 3), dtype=torch.uint8, generator=g).cuda()
    p = pb.make_twar_params([[-ONE, ONE, ONE], [ONE // 2, -ONE // 2, ONE], [ONE // 2, -ONE // 2, ONE]], [0, 0, 0])
    res = torch.empty_like(img)
    back = torch.empty_like(img)
    pb.pilc_twar_forward(p, img, res)
    # two frames of the residual against the CPU reference
    assert np.array_equal(res[:2].cpu().numpy(), to.forward(to.make_params(
        [[-ONE, ONE, ONE], [ONE // 2, -ONE // 2, ONE], [ONE // 2, -ONE // 2, ONE]], [0, 0, 0]), img[:2].cpu().numpy()))
    for turn in range(5):
        back.fill_(0xA5 ^ turn)
        pb.pilc_twar_inverse(p, res, back)
        assert torch.equal(back, img), turn


def test_bands_give_up_a_wait_that_is_never_answered():
    """A band of a tall image waits for the last row of the band above.  With that row made to
    publish nothing (a switch that exists for this test) and a bound of 20 microseconds the band
    below must give up, every kernel must end, and the call must say PILC_E_TIMEOUT; the next
    ordinary call works."""
    rng = np.random.default_rng(5)
    img = rng.integers(0, 256, (2, 700, 64, 3), dtype=np.uint8)
    wq, bq = [[ONE // 2, ONE // 4, ONE // 4]] * 3, [0, 0, 0]
    p = pb.make_twar_params(wq, bq)
    d_res = torch.from_numpy(to.forward(to.make_params(wq, bq), img)).cuda()
    d_back = torch.zeros_like(d_res)
    try:
        pb.pilc_set_one_pass_wait(2000, True)
        assert pb.pilc_twar_inverse(p, d_res, d_back, check=False) == pb.PILC_E_TIMEOUT
    finally:
        pb.pilc_set_one_pass_wait(0, False)
    assert pb.pilc_twar_inverse(p, d_res, d_back, check=False) == pb.PILC_OK
    assert np.array_equal(d_back.cpu().numpy(), img)


def test_bad_arguments():
    img = torch.zeros((2, 4, 4, 3), dtype=torch.uint8, device="cuda:0")
    out = torch.zeros_like(img)
    p = pb.make_twar_params([[0] * 3] * 3, [0] * 3)
    assert pb.pilc_twar_forward(p, img, img, check=False) == pb.PILC_E_ARG      # in place is not allowed
    assert pb.pilc_twar_inverse(p, img, img, check=False) == pb.PILC_E_ARG
    bad = pb.make_twar_params([[0] * 3] * 3, [(1 << 30) + 1, 0, 0])
    assert pb.pilc_twar_forward(bad, img, out, check=False) == pb.PILC_E_ARG
    empty = torch.zeros((0, 4, 4, 3), dtype=torch.uint8, device="cuda:0")
    assert pb.lib().pilc_twar_forward(0, 4, 4, img.data_ptr(), None, out.data_ptr(), None) == pb.PILC_E_ARG
    del empty
