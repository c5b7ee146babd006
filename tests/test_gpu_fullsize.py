"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.  The oracle
cannot afford whole 150-200 MB sets inside a test, so: (i) lanes are independent streams (pinned
on the CPU), hence sampled lanes are encoded one by one by the oracle and compared byte for byte
with the GPU container; (ii) offsets must be the exclusive scan of lane sizes; (iii) the GPU
decode must return the original image exactly."""
import numpy as np
import pytest
import torch

from oracle import pilc_oracle as orc
from paper_2206_05279_amd import binding as pb
from paper_2206_05279_amd import synth

pytestmark = pytest.mark.gpu

from gpu_util import DeviceWorkload, parse_container  # noqa: E402


def _oracle_lane_bytes(wl, lane):
    """Container bytes of one lane, from the oracle run on that lane's pixels alone."""
    n, h, w, m, mode, la, lb = wl.geom
    hw = h * w
    if mode == 0 and la % hw == 0:            # lane = whole images
        k = la // hw
        i0, i1 = lane * k, min((lane + 1) * k, n)
        g = orc.make_geom(i1 - i0, h, w, m, 0, la, 0)
        sl = slice(i0, i1)
        rc, coded = orc.encode(g, wl.img[sl].copy(), wl.mu[sl].copy(), wl.log_scale[sl].copy(),
                               wl.chan_coef[sl].copy())
        assert rc == orc.OK
        return parse_container(coded)[3]
    if mode == 0:                             # lane inside one image: encode the image, pick the lane
        per = hw // la
        i = lane // per
        g = orc.make_geom(1, h, w, m, 0, la, 0)
    else:
        per = -(-h // la) * -(-w // lb)
        i = lane // per
        g = orc.make_geom(1, h, w, m, 1, la, lb)
    sl = slice(i, i + 1)
    rc, coded = orc.encode(g, wl.img[sl].copy(), wl.mu[sl].copy(), wl.log_scale[sl].copy(),
                           wl.chan_coef[sl].copy())
    assert rc == orc.OK
    _, _, offs, body = parse_container(coded)
    j = lane - i * per
    return body[offs[j]:offs[j + 1]]


FULL = [
    ("cfg1-full", lambda: synth.make_workload(1), 12),
    ("cfg2-full", lambda: synth.make_workload(2), 6),
    ("cfg3-full", lambda: synth.make_workload(3), 2),
    ("cfg4-full-M12-L64", lambda: synth.make_workload(4, prec_bits=12, lanes_per_image=64), 6),
    ("cfg4-full-M16-L64", lambda: synth.make_workload(4, prec_bits=16, lanes_per_image=64), 6),
]
# the rest of the stress workload's sweep (lanes per image 1..1024, M = 12 and 16) on a subset of
# 256 of its 256x256 images: 128 of the random half and 128 of the constant half
FULL += [("cfg4-256img-M%d-L%d" % (m, lpi),
          (lambda m=m, lpi=lpi: synth.make_workload(4, 256, prec_bits=m, lanes_per_image=lpi)), 3)
         for m in (12, 16) for lpi in (1, 2, 4, 8, 16, 32, 128, 256, 512, 1024)]


@pytest.mark.parametrize("name,make,samples", FULL, ids=[c[0] for c in FULL])
def test_full_size_sampled_parity(name, make, samples):
    print("generating", name, flush=True)
    wl = make()
    d = DeviceWorkload(wl)
    print("encoding", name, wl.geom, flush=True)
    _, nbytes = d.encode()
    coded = d.coded_numpy()
    lanes, payload, offs, body = parse_container(coded)
    assert lanes == pb.pilc_lane_count(d.geom) and nbytes == 64 + 4 * (lanes + 1) + payload
    sizes = np.diff(offs.astype(np.int64))
    assert offs[0] == 0 and offs[-1] == payload and sizes.min() >= 4 and not np.any(sizes & 1)
    rng = np.random.default_rng(99)
    picks = sorted(set([0, lanes - 1] + [int(v) for v in rng.integers(0, lanes, size=samples)]))
    for lane in picks:
        want = _oracle_lane_bytes(wl, lane)
        got = body[offs[lane]:offs[lane + 1]]
        assert np.array_equal(got, want), "lane %d differs" % lane
    print("decoding", name, flush=True)
    assert d.decode() == pb.PILC_OK
    assert torch.equal(d.out, d.img)
    print("bits/subpixel %.4f" % (8.0 * nbytes / wl.subpixels), flush=True)


def test_table_coder_full_size_sampled_parity():
    """The table-driven coder (Sec. 3.2 Algs. 3-4) on the 10^6 x 1000 recipe of Sec. 4.3, in the
    launch configuration bench.py times: pieces are independent, so sampled pieces are encoded by
    the reference one by one and compared with their records; offsets must be the exclusive scan
    of the record sizes; decode must return the symbols."""
    import struct

    from oracle import ansai_oracle as ao
    from paper_2206_05279_amd import synth_pieces as sp

    from gpu_util import DevicePieces

    print("generating pieces1", flush=True)
    wl = sp.make_piece_workload(1, threads=16)
    dp = DevicePieces(wl.prec_bits, wl.mass, wl.sym, wl.dist)
    print("encoding", flush=True)
    _, nbytes = dp.encode()
    coded = dp.coded_numpy()
    pieces = wl.pieces
    assert coded[:4].tobytes() == b"PANS"
    assert struct.unpack_from("<6I", coded, 4) == (1, pieces, wl.count, wl.prec_bits, 8, 256)
    payload = struct.unpack_from("<Q", coded, 48)[0]
    offs = np.frombuffer(coded, dtype="<u4", count=pieces + 1, offset=64)
    body = coded[64 + 4 * (pieces + 1):]
    assert nbytes == 64 + 4 * (pieces + 1) + payload and offs[0] == 0 and offs[-1] == payload
    # every record's size follows from its own bit count, and the offsets are their running sum
    bits = np.frombuffer(body, dtype="<u4")[(offs[:-1] // 4 + 1).astype(np.int64)]
    sizes = 8 + 4 * ((bits.astype(np.int64) + 31) // 32)
    assert np.array_equal(np.diff(offs.astype(np.int64)), sizes)
    rng = np.random.default_rng(11)
    sample = np.unique(np.concatenate([[0, 63, 64, pieces - 65, pieces - 1], rng.integers(0, pieces, 200)]))
    rc, ref = ao.encode(wl.prec_bits, wl.mass, wl.sym[sample], wl.dist[sample])
    assert rc == ao.OK
    roffs = np.frombuffer(ref, dtype="<u4", count=sample.size + 1, offset=64)
    rbody = ref[64 + 4 * (sample.size + 1):]
    for i, p in enumerate(sample):
        assert np.array_equal(body[offs[p]:offs[p + 1]], rbody[roffs[i]:roffs[i + 1]]), "piece %d" % p
    print("decoding", flush=True)
    dp.decode()
    assert torch.equal(dp.out, dp.sym)


def test_twar_full_size_parity():
    """The Three-Way AR transform on all 50,000 images of the CIFAR-shaped workload: the whole
    residual against the reference, and the inverse back to the images."""
    from oracle import twar_oracle as to

    wl = synth.make_workload(1)
    weights, bias = [[-16384, 16384, 16384], [8192, -8192, 16384], [8192, -8192, 16384]], [0, 0, 0]
    print("reference forward", flush=True)
    ref = to.forward(to.make_params(weights, bias), wl.img)
    img = torch.from_numpy(wl.img).cuda()
    res, back = torch.empty_like(img), torch.empty_like(img)
    p = pb.make_twar_params(weights, bias)
    pb.pilc_twar_forward(p, img, res)
    assert np.array_equal(res.cpu().numpy(), ref)
    pb.pilc_twar_inverse(p, res, back)
    assert torch.equal(back, img)


def test_mixture_full_size_sampled_parity():
    """The mixture workload bench.py times (2048 images of cfg 2, K = 10, one lane per row):
    sampled images are encoded by the mixture oracle on their own and their 64 lanes compared byte
    for byte with the GPU container; offsets are the scan of lane sizes; the GPU decode returns
    the images."""
    from oracle import mix_oracle as mx
    from paper_2206_05279_amd import synth_mix
    from gpu_util import DeviceMix

    print("generating mixture workload", flush=True)
    wl = synth_mix.make_mix_workload(2, 2048, 10)
    d = DeviceMix(wl)
    print("encoding", wl.geom, flush=True)
    _, nbytes = d.encode()
    coded = d.coded_numpy()
    assert coded[:4].tobytes() == b"PMIX" and int(np.frombuffer(coded.tobytes(), "<u4", 1, 44)[0]) == 10
    lanes = pb.pilc_lane_count(d.geom)
    offs = np.frombuffer(coded.tobytes(), dtype="<u4", count=lanes + 1, offset=64)
    body = coded[64 + 4 * (lanes + 1):]
    sizes = np.diff(offs.astype(np.int64))
    assert offs[0] == 0 and offs[-1] == body.size and sizes.min() >= 4 and not np.any(sizes & 1)
    n, h, w, m, mode, la, lb = wl.geom
    per = h * w // la
    rng = np.random.default_rng(98)
    for i in sorted(set([0, n - 1] + [int(v) for v in rng.integers(0, n, size=6)])):
        sl = slice(i, i + 1)
        g = orc.make_geom(1, h, w, m, mode, la, lb)
        rc, one = mx.encode(g, 10, wl.img[sl], wl.mu[sl], wl.log_scale[sl], wl.weight[sl], wl.chan_coef[sl])
        assert rc == mx.OK
        want = one[64 + 4 * (per + 1):]
        got = body[offs[i * per]:offs[(i + 1) * per]]
        assert np.array_equal(got, want), "image %d differs" % i
        o1 = np.frombuffer(one.tobytes(), dtype="<u4", count=per + 1, offset=64)
        assert np.array_equal(np.diff(o1.astype(np.int64)), sizes[i * per:(i + 1) * per])
    print("decoding", flush=True)
    assert d.decode() == pb.PILC_OK
    assert torch.equal(d.out, d.img)
    print("bits/subpixel %.4f" % (8.0 * nbytes / wl.subpixels), flush=True)
