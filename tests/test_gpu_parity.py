"""GPU <-> oracle parity through the C ABI: per-symbol tables, container bytes, decoded images,
error paths.  Integer work: the bar is bit-exact."""
import numpy as np
import pytest
import torch

from oracle import pilc_oracle as orc
from paper_2206_05279_amd import binding as pb
from paper_2206_05279_amd import synth

pytestmark = pytest.mark.gpu

from gpu_util import DeviceWorkload, first_difference  # noqa: E402


def _ogeom(wl):
    return orc.make_geom(*wl.geom)


@pytest.fixture(params=[1, 2, 3], ids=["thread-per-lane", "few-lane", "thread-per-lane-one-pass"])
def policy(request):
    """Runs a test once with each lane-kernel family forced (thread per lane: with the scan and
    pack kernels, and with the encoder placing its lanes itself)."""
    pb.pilc_set_kernel_policy(request.param)
    yield request.param
    pb.pilc_set_kernel_policy(0)


def _alternating_fit():
    """CIFAR-shaped lanes of 16 images in which every other run of 4 images is uniformly random
    while the parameters still describe the smooth images: the few-lane decoder has to go from
    its windows to the search and back several times inside a lane."""
    wl = synth.make_workload(1, 16 * 9)
    rng = np.random.default_rng(5)
    for i0 in range(4, wl.n, 8):
        wl.img[i0:i0 + 4] = rng.integers(0, 256, size=wl.img[i0:i0 + 4].shape, dtype=np.uint8)
    return wl


SMALL_CASES = [
    ("cfg0-full", lambda: synth.make_workload(0)),
    ("cfg1-70-lanes", lambda: synth.make_workload(1, 16 * 70)),
    ("cfg1-ragged-last-lane", lambda: synth.make_workload(1, 16 * 5 + 3)),
    ("cfg2-64-images", lambda: synth.make_workload(2, 64)),
    ("cfg3-clipped-tiles", lambda: synth.make_workload(3, 2, h=88, w=200)),
    ("cfg4-M12-L1", lambda: synth.make_workload(4, 8, h=64, w=64, prec_bits=12, lanes_per_image=1)),
    ("cfg4-M16-L16", lambda: synth.make_workload(4, 8, h=64, w=64, prec_bits=16, lanes_per_image=16)),
    ("cfg4-M16-L1-mixed-wavefront", lambda: synth.make_workload(4, 6, h=64, w=64, prec_bits=16, lanes_per_image=1)),
    ("cfg1-fit-and-random-runs", _alternating_fit),
    ("cfg4-M12-L1024", lambda: synth.make_workload(4, 8, h=64, w=64, prec_bits=12, lanes_per_image=1024)),
    ("cfg4-M16-L1024", lambda: synth.make_workload(4, 6, h=64, w=64, prec_bits=16, lanes_per_image=1024)),
    ("wild-flat-M10", lambda: synth.make_random_case(1, 37, 12, 10, 10, 0, 40, wild=True)),
    ("wild-flat-span-M16", lambda: synth.make_random_case(2, 37, 12, 10, 16, 0, 360, wild=True)),
    ("wild-tiles-M13", lambda: synth.make_random_case(3, 5, 37, 41, 13, 1, 8, 16, wild=True)),
    ("wild-tiles-1xw", lambda: synth.make_random_case(4, 3, 9, 70, 11, 1, 1, 70, wild=True)),
    ("wild-single-pixel-lanes", lambda: synth.make_random_case(5, 2, 7, 9, 14, 0, 1, wild=True)),
    ("one-pixel", lambda: synth.make_random_case(6, 1, 1, 1, 12, 0, 1, wild=True)),
    ("one-lane-whole-batch", lambda: synth.make_random_case(7, 4, 16, 16, 15, 0, 4 * 256)),
    # more lanes than one workgroup of the few-lane decoder per compute unit can hold, of uneven length:
    # the form of that decoder whose wavefronts stage their own batches
    ("wild-5720-clipped-tile-lanes", lambda: synth.make_random_case(8, 40, 37, 41, 13, 1, 3, 4, wild=True)),
]


@pytest.mark.parametrize("name,make", SMALL_CASES, ids=[c[0] for c in SMALL_CASES])
def test_symbol_tables_match_oracle(name, make):
    wl = make()
    print("case", name, wl.geom, flush=True)
    d = DeviceWorkload(wl)
    cum = torch.zeros(wl.subpixels, dtype=torch.uint32, device="cuda:0")
    freq = torch.zeros_like(cum)
    pb.pilc_symbol_tables(d.geom, d.img, d.mu, d.log_scale, d.chan_coef, cum, freq)
    o_cum, o_freq = orc.symbol_tables(_ogeom(wl), wl.img, wl.mu, wl.log_scale, wl.chan_coef)
    assert np.array_equal(cum.cpu().numpy(), o_cum)
    assert np.array_equal(freq.cpu().numpy(), o_freq)


@pytest.mark.parametrize("name,make", SMALL_CASES, ids=[c[0] for c in SMALL_CASES])
def test_container_and_image_match_oracle(name, make, policy):
    wl = make()
    print("case", name, wl.geom, "policy", policy, flush=True)
    d = DeviceWorkload(wl)
    rc, nbytes = d.encode()
    o_rc, o_coded = orc.encode(_ogeom(wl), wl.img, wl.mu, wl.log_scale, wl.chan_coef)
    assert o_rc == orc.OK
    got = d.coded_numpy()
    assert nbytes == o_coded.size and np.array_equal(got, o_coded), first_difference(got, o_coded)
    # decode the GPU's own container, and the oracle's
    assert d.decode() == pb.PILC_OK
    assert np.array_equal(d.decoded_numpy(), wl.img)
    o_rc, o_img = orc.decode(_ogeom(wl), got, wl.mu, wl.log_scale, wl.chan_coef)
    assert o_rc == orc.OK and np.array_equal(o_img, wl.img)
    # encode is deterministic
    d.coded.zero_()
    d.encode()
    assert np.array_equal(d.coded_numpy(), o_coded)


def test_exact_capacity_is_enough_and_one_byte_less_is_not():
    wl = synth.make_workload(0, 8)
    d = DeviceWorkload(wl)
    _, nbytes = d.encode()
    ref = d.coded_numpy().copy()
    d.coded.zero_()
    rc, nb2 = d.encode(capacity=nbytes)
    assert rc == pb.PILC_OK and nb2 == nbytes and np.array_equal(d.coded_numpy(), ref)
    rc, _ = d.encode(check=False, capacity=nbytes - 1)
    assert rc == pb.PILC_E_CAPACITY
    rc, _ = d.encode(check=False, capacity=64 + 4 * 256)  # not even the offset table
    assert rc == pb.PILC_E_CAPACITY
    # a workspace that is too small is refused on the host
    small = torch.empty(1024, dtype=torch.uint8, device="cuda:0")
    rc, _ = pb.pilc_encode(d.geom, d.img, d.mu, d.log_scale, d.chan_coef, small, d.coded, check=False)
    assert rc == pb.PILC_E_WORKSPACE


def test_one_pass_encoder_gives_up_a_wait_that_is_never_answered():
    """The one-pass encoder's workgroups wait for the byte counts of the workgroups before
    them.  The wait is bounded: with the first workgroup made to publish nothing (a switch that
    exists for this test) and a bound of 20 microseconds, every other workgroup must give up, every
    kernel must end, and the call must say PILC_E_TIMEOUT; the next ordinary call works."""
    wl = synth.make_workload(2, 64)           # 4096 row lanes: 64 workgroups of 64
    d = DeviceWorkload(wl)
    pb.pilc_set_kernel_policy(3)
    try:
        _, nbytes = d.encode()
        ref = d.coded_numpy()[:nbytes].copy()
        pb.pilc_set_one_pass_wait(2000, True)
        rc, _ = d.encode(check=False)
        assert rc == pb.PILC_E_TIMEOUT
        pb.pilc_set_one_pass_wait(0, False)
        d.coded.zero_()
        rc, nb2 = d.encode()
        assert rc == pb.PILC_OK and nb2 == nbytes and np.array_equal(d.coded_numpy()[:nbytes], ref)
    finally:
        pb.pilc_set_one_pass_wait(0, False)
        pb.pilc_set_kernel_policy(0)


def test_few_lane_decoder_gives_up_a_wait_that_is_never_answered():
    """A decoding wavefront of the few-lane decoder waits for its stager to say that a batch is
    ready.  With the stagers made silent (a switch that exists for this test) and a bound of 20
    microseconds every decoding wavefront must give up, the kernel must end, and the call must say
    PILC_E_TIMEOUT; the next ordinary call works."""
    wl = synth.make_workload(1, 16 * 9)
    d = DeviceWorkload(wl)
    rc, _ = d.encode()
    assert rc == pb.PILC_OK
    pb.pilc_set_kernel_policy(2)
    try:
        pb.pilc_set_one_pass_wait(2000, True)
        assert d.decode(check=False) == pb.PILC_E_TIMEOUT
        pb.pilc_set_one_pass_wait(0, False)
        assert d.decode() == pb.PILC_OK
        assert np.array_equal(d.decoded_numpy(), wl.img)
    finally:
        pb.pilc_set_one_pass_wait(0, False)
        pb.pilc_set_kernel_policy(0)


def test_damaged_containers_give_error_codes_never_faults(policy):
    wl = synth.make_workload(0, 4)
    d = DeviceWorkload(wl)
    _, nbytes = d.encode()
    good = d.coded.clone()
    lanes = pb.pilc_lane_count(d.geom)
    table_end = 64 + 4 * (lanes + 1)

    def run(mutate, nb=nbytes):
        bad = good.clone()
        mutate(bad)
        return d.decode(coded=bad, nbytes=nb, check=False)

    def flip(pos, bit=1):
        def m(t):
            t[pos] ^= bit
        return m

    assert run(flip(0)) == pb.PILC_E_FORMAT                      # magic
    assert run(flip(4)) == pb.PILC_E_FORMAT                      # version
    assert run(flip(24)) == pb.PILC_E_FORMAT                     # M
    assert run(flip(40)) == pb.PILC_E_FORMAT                     # lanes
    assert run(flip(48, 2)) == pb.PILC_E_FORMAT                  # payload size vs container size
    assert run(lambda t: None, nb=nbytes - 2) == pb.PILC_E_FORMAT  # truncated
    assert run(lambda t: None, nb=16) == pb.PILC_E_FORMAT
    assert run(flip(64, 2)) == pb.PILC_E_CORRUPT                 # offsets[0] != 0
    assert run(flip(64 + 4 * 7, 2)) == pb.PILC_E_CORRUPT         # lane 6 longer, lane 7 shorter
    assert run(flip(64 + 4 * 9 + 3, 0x80)) == pb.PILC_E_CORRUPT  # offset far out of bounds
    assert run(flip(64 + 4 * 9, 1)) == pb.PILC_E_CORRUPT         # odd offset

    def swap_two(t):
        a = t[64 + 4 * 3: 64 + 4 * 4].clone()
        t[64 + 4 * 3: 64 + 4 * 4] = t[64 + 4 * 4: 64 + 4 * 5]
        t[64 + 4 * 4: 64 + 4 * 5] = a
    assert run(swap_two) == pb.PILC_E_CORRUPT                    # not monotone
    # payload damage: either detected or it yields a different image; never a fault
    rng = np.random.default_rng(0)
    detected = 0
    for _ in range(24):
        pos = int(rng.integers(table_end, nbytes))
        rc = run(flip(pos, 1 << int(rng.integers(0, 8))))
        assert rc in (pb.PILC_OK, pb.PILC_E_CORRUPT)
        if rc == pb.PILC_OK:
            assert not np.array_equal(d.decoded_numpy(), wl.img)
        else:
            detected += 1
    assert detected >= 18
    # the intact container still decodes afterwards
    assert d.decode(coded=good) == pb.PILC_OK and np.array_equal(d.decoded_numpy(), wl.img)


def test_decode_on_a_side_stream_and_timing_entries():
    wl = synth.make_workload(2, 16)
    d = DeviceWorkload(wl)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    pb.pilc_set_timing(True)
    try:
        rc, nbytes = pb.pilc_encode(d.geom, d.img, d.mu, d.log_scale, d.chan_coef, d.workspace,
                                    d.coded, stream=s)
        t_enc = pb.pilc_last_timing()
        pb.pilc_decode(d.geom, d.coded, nbytes, d.mu, d.log_scale, d.chan_coef, d.workspace, d.out,
                       stream=s)
        t_dec = pb.pilc_last_timing()
    finally:
        pb.pilc_set_timing(False)
    assert np.array_equal(d.decoded_numpy(), wl.img)
    assert t_enc[0][0] == "total" and len(t_enc) >= 3 and all(ms >= 0 for _, ms in t_enc)
    assert t_dec[0][0] == "total" and any(name.startswith("k_decode_") for name, _ in t_dec)
    assert abs(sum(ms for _, ms in t_enc[1:]) - t_enc[0][1]) < 0.05 * max(t_enc[0][1], 0.1) + 0.05
    pb.pilc_encode(d.geom, d.img, d.mu, d.log_scale, d.chan_coef, d.workspace, d.coded)
    assert pb.pilc_last_timing() == []
