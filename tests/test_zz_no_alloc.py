"""pilc_encode_static (the entry point that allocates nothing: its scratch memory is an array
inside the library) against pilc_encode on the same inputs, through the C ABI: two calls in a row,
the second on a smaller input, so that what the first call left in the shared array is there when
the second runs.  Both kernel families (few long lanes, one thread per lane) are covered."""
import numpy as np
import pytest
import torch

from paper_2206_05279_amd import binding as pb
from paper_2206_05279_amd import synth

pytestmark = pytest.mark.gpu

from gpu_util import DeviceWorkload, first_difference  # noqa: E402


def _both(wl):
    d = DeviceWorkload(wl)
    _, nbytes = d.encode()
    want = d.coded_numpy().copy()
    coded = torch.zeros_like(d.coded)
    print("pilc_encode_static", wl.geom, flush=True)
    rc, nb = pb.pilc_encode_static(d.geom, d.img, d.mu, d.log_scale, d.chan_coef, coded)
    assert rc == pb.PILC_OK and nb == nbytes
    got = coded[:nb].cpu().numpy()
    assert np.array_equal(got, want), first_difference(got, want)
    # and the container decodes back to the images
    assert d.decode(coded, nb) == pb.PILC_OK
    assert torch.equal(d.out, d.img)


@pytest.mark.parametrize("first,second", [
    # thread per lane (40,960 lanes), then few long lanes (48 lanes of 2 images)
    (lambda: synth.make_workload(2, 640), lambda: synth.make_workload(1, 96, prec_bits=14)),
    # one 1920x1080 frame in 16x16 tiles, then the tiny workload
    (lambda: synth.make_workload(3, 1), lambda: synth.make_workload(0)),
])
def test_static_scratch_encode_matches_pilc_encode_twice(first, second):
    big, small = first(), second()
    assert small.subpixels < big.subpixels
    for wl in (big, small):
        ws, _ = pb.pilc_workspace_size(pb.make_geom(*wl.geom))
        assert ws <= pb.PILC_STATIC_SCRATCH_BYTES
    _both(big)
    _both(small)


def test_static_scratch_encode_refuses_what_does_not_fit():
    wl = synth.make_workload(2, 4096)          # needs about 100 MB of workspace
    d = DeviceWorkload(wl)
    assert pb.pilc_workspace_size(d.geom)[0] > pb.PILC_STATIC_SCRATCH_BYTES
    rc, _ = pb.pilc_encode_static(d.geom, d.img, d.mu, d.log_scale, d.chan_coef, d.coded, check=False)
    assert rc == pb.PILC_E_WORKSPACE
