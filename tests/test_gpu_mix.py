"""GPU parity of the mixture-of-logistics coder: containers and decoded images bit-identical to
oracle/mix_oracle.c on the same seeded inputs, through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import mix_oracle as mx
from oracle import pilc_oracle as orc
from paper_2206_05279_amd import binding as pb
from paper_2206_05279_amd import synth, synth_mix

from gpu_util import DeviceMix, first_difference

pytestmark = pytest.mark.gpu

CASES = [
    ("cfg0-k2", lambda: synth_mix.make_mix_workload(0, 8, 2)),
    ("cfg0-k10", lambda: synth_mix.make_mix_workload(0, 6, 10)),
    ("cfg2-k10-rows", lambda: synth_mix.make_mix_workload(2, 5, 10)),
    ("cfg2-k16-M16", lambda: synth_mix.make_mix_workload(2, 3, 16, prec_bits=16)),
    ("cfg3-k3-tiles", lambda: synth_mix.make_mix_workload(3, 1, 3, h=40, w=72)),
    ("cfg1-k5-long-lanes", lambda: synth_mix.make_mix_workload(1, 16 * 3 + 5, 5)),
    ("cfg4-k4-M12", lambda: synth_mix.make_mix_workload(4, 6, 4, h=32, w=32, prec_bits=12, lanes_per_image=16)),
    ("k1", lambda: synth_mix.make_mix_workload(0, 5, 1)),
    ("wild-k7-ragged-tiles", lambda: synth_mix.from_base(
        synth.make_random_case(3, 5, 37, 41, 13, 1, 8, 16, wild=True), 7, 3)),
    ("wild-k9-flat-M10", lambda: synth_mix.from_base(
        synth.make_random_case(2, 37, 12, 10, 10, 0, 360, wild=True), 9, 2)),
    ("many-lanes-k2", lambda: synth_mix.from_base(synth.make_random_case(9, 70, 16, 16, 14, 0, 8), 2, 9)),
    # K = 10 runs in kernels of its own (components in registers): the same corners again
    ("wild-k10-ragged-tiles", lambda: synth_mix.from_base(
        synth.make_random_case(13, 5, 37, 41, 13, 1, 8, 16, wild=True), 10, 13)),
    ("wild-k10-flat-M10", lambda: synth_mix.from_base(
        synth.make_random_case(12, 37, 12, 10, 10, 0, 360, wild=True), 10, 12)),
    ("cfg1-k10-long-lanes", lambda: synth_mix.make_mix_workload(1, 16 * 2 + 5, 10)),
    ("cfg4-k10-M16", lambda: synth_mix.make_mix_workload(4, 6, 10, h=32, w=32, prec_bits=16, lanes_per_image=16)),
    ("many-lanes-k10", lambda: synth_mix.from_base(synth.make_random_case(19, 70, 16, 16, 14, 0, 8), 10, 19)),
]


@pytest.mark.parametrize("name,make", CASES, ids=[c[0] for c in CASES])
def test_container_and_image_identical_to_oracle(name, make):
    wl = make()
    g = orc.make_geom(*wl.geom)
    rc, want = mx.encode(g, wl.num_comp, wl.img, wl.mu, wl.log_scale, wl.weight, wl.chan_coef)
    assert rc == mx.OK
    d = DeviceMix(wl)
    rc, nbytes = d.encode()
    got = d.coded_numpy()
    assert nbytes == want.size, "container size %d, oracle %d" % (nbytes, want.size)
    assert np.array_equal(got, want), first_difference(got, want)
    # decode the oracle's container on the GPU
    coded = torch.from_numpy(want).cuda()
    assert d.decode(coded=coded, nbytes=want.size) == pb.PILC_OK
    assert np.array_equal(d.decoded_numpy(), wl.img)


def test_ten_components_in_arrays_off_the_dword_grid_take_the_general_kernels():
    wl = synth_mix.make_mix_workload(2, 4, 10)
    g = orc.make_geom(*wl.geom)
    rc, want = mx.encode(g, wl.num_comp, wl.img, wl.mu, wl.log_scale, wl.weight, wl.chan_coef)
    assert rc == mx.OK
    d = DeviceMix(wl)

    def shifted(t):  # the same values at an address that is 2 but not 4 bytes aligned
        buf = torch.empty(t.numel() + 1, dtype=t.dtype, device=t.device)
        buf[1:] = t.reshape(-1)
        assert buf[1:].data_ptr() % 4 == 2
        return buf[1:].reshape(t.shape)

    d.mu, d.log_scale, d.weight = shifted(d.mu), shifted(d.log_scale), shifted(d.weight)
    rc, nbytes = d.encode()
    got = d.coded_numpy()
    assert nbytes == want.size and np.array_equal(got, want), first_difference(got, want)
    assert d.decode() == pb.PILC_OK
    assert np.array_equal(d.decoded_numpy(), wl.img)


def test_one_component_matches_the_single_law_path():
    base = synth.make_workload(2, 6)
    wl = synth_mix.from_base(base, 1, 1)
    assert np.array_equal(wl.mu[..., 0], base.mu) and np.all(wl.weight == 32768)
    d = DeviceMix(wl)
    d.encode()
    mix = d.coded_numpy()
    rc, single = orc.encode(orc.make_geom(*base.geom), base.img, base.mu, base.log_scale, base.chan_coef)
    assert rc == orc.OK and mix.size == single.size
    assert np.array_equal(mix[64:], single[64:]) and np.array_equal(mix[8:44], single[8:44])


@pytest.mark.parametrize("k", [3, 10])
def test_bad_weights_and_component_counts_are_rejected(k):
    wl = synth_mix.make_mix_workload(0, 4, k)
    d = DeviceMix(wl)
    rc, _ = d.encode()
    good = d.nbytes
    bad = wl.weight.copy()
    bad[2, 5, 7, 1] += 1
    bad = torch.from_numpy(bad).cuda()
    assert d.encode(check=False, weight=bad)[0] == pb.PILC_E_ARG
    d.encode()
    assert d.nbytes == good
    assert d.decode(check=False, weight=bad) == pb.PILC_E_ARG
    assert d.encode(check=False, k=0)[0] == pb.PILC_E_ARG
    assert d.encode(check=False, k=17)[0] == pb.PILC_E_ARG
    assert d.decode(check=False, k=17) == pb.PILC_E_ARG


def test_damaged_containers_fail_like_the_oracle():
    wl = synth_mix.make_mix_workload(0, 4, 2)
    g = orc.make_geom(*wl.geom)
    d = DeviceMix(wl)
    d.encode()
    coded = d.coded_numpy()
    args = (wl.mu, wl.log_scale, wl.weight, wl.chan_coef)

    def both(buf):
        rc_o, _ = mx.decode(g, 2, buf, *args)
        t = torch.from_numpy(np.ascontiguousarray(buf)).cuda()
        t = torch.cat([t, torch.zeros(16, dtype=torch.uint8, device="cuda")])
        rc_g = d.decode(coded=t, nbytes=buf.size, check=False)
        return rc_o, rc_g

    b = coded.copy(); b[0] = ord("Q")
    assert both(b) == (mx.E_FORMAT, pb.PILC_E_FORMAT)
    b = coded.copy(); b[44] = 5      # another component count
    assert both(b) == (mx.E_FORMAT, pb.PILC_E_FORMAT)
    b = coded.copy(); b[3] = ord("C")  # the single-law magic
    assert both(b) == (mx.E_FORMAT, pb.PILC_E_FORMAT)
    assert both(coded[:-2]) == (mx.E_FORMAT, pb.PILC_E_FORMAT)
    b = coded.copy(); b[64 + 4] ^= 2  # an offset
    assert both(b) == (mx.E_CORRUPT, pb.PILC_E_CORRUPT)
    b = coded.copy(); b[-3] ^= 0x10   # a stream word: detected, or a different image
    rc_o, rc_g = both(b)
    assert (rc_o == mx.OK) == (rc_g == pb.PILC_OK)
    if rc_o == mx.OK:
        assert np.array_equal(d.decoded_numpy(), mx.decode(g, 2, b, *args)[1])
    # the single-law decoder does not take a mixture container
    from gpu_util import DeviceWorkload
    base = synth.make_workload(0, 4)
    dw = DeviceWorkload(base)
    t = torch.from_numpy(coded).cuda()
    assert dw.decode(coded=t, nbytes=coded.size, check=False) == pb.PILC_E_FORMAT


def test_capacity():
    wl = synth_mix.make_mix_workload(0, 4, 2)
    d = DeviceMix(wl)
    rc, n = d.encode()
    assert d.encode(check=False, capacity=n - 2)[0] == pb.PILC_E_CAPACITY
    assert d.encode(check=False, capacity=n)[0] == pb.PILC_OK
