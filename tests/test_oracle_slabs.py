"""The slab-parallel driver of the oracle that the full-size GPU tests use must give exactly what
one pass of the oracle over the whole batch gives (lane independence: a batch's payload is its
lanes' bytes in order, the offset table their running sum; header per the container's definition).
Checked here on cases small enough for one pass, with lanes that span images, ragged last lanes,
tiles and the mixture and piece containers."""
import numpy as np
import pytest

import oracle_slabs
from oracle import ansai_oracle as ao
from oracle import mix_oracle as mx
from oracle import pilc_oracle as orc
from paper_2206_05279_amd import synth, synth_mix
from paper_2206_05279_amd import synth_pieces as sp


@pytest.mark.parametrize("cfg,n,kw", [
    (0, 64, {}),
    (1, 16 * 37 + 5, {}),                 # 16-image lanes, a ragged last lane
    (2, 45, {}),
    (3, 2, {"h": 72, "w": 112}),          # tiles with a clipped bottom row
    (4, 6, {"h": 64, "w": 64, "prec_bits": 16, "lanes_per_image": 1}),
    (4, 6, {"h": 64, "w": 64, "prec_bits": 12, "lanes_per_image": 1024}),
])
@pytest.mark.parametrize("threads", [1, 3])
def test_slabs_equal_one_pass(cfg, n, kw, threads):
    wl = synth.make_workload(cfg, n, **kw)
    rc, ref = orc.encode(orc.make_geom(*wl.geom), wl.img, wl.mu, wl.log_scale, wl.chan_coef)
    assert rc == orc.OK
    assert np.array_equal(oracle_slabs.whole_container(wl, threads), ref)


def test_mixture_slabs_equal_one_pass():
    wl = synth_mix.make_mix_workload(2, 9, 5)
    rc, ref = mx.encode(orc.make_geom(*wl.geom), 5, wl.img, wl.mu, wl.log_scale, wl.weight, wl.chan_coef)
    assert rc == mx.OK
    assert np.array_equal(oracle_slabs.whole_mix_container(wl, 2), ref)


def test_piece_slabs_equal_one_pass():
    wl = sp.make_piece_workload(0, 300, threads=2)
    rc, ref = ao.encode(wl.prec_bits, wl.mass, wl.sym, wl.dist)
    assert rc == ao.OK
    assert np.array_equal(oracle_slabs.whole_piece_container(wl, 3), ref)
