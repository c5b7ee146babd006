"""Pins for the mixture-of-logistics oracle (oracle/mix_oracle.c).

Sec. 2 of arXiv 2206.05279 names the workload (rANS driven by a mixture of 10 logistic laws per
symbol) without a formula, so nothing printed in the paper can be compared byte for byte.  The
pins tie the oracle to things fixed outside it: the single-law oracle (itself pinned) for K = 1
and for equal components, the float64 closed form of a weighted sum of logistic differences,
the invariants of Sec. 3.2 (integer masses >= 1 summing to 2^M), exact round trips, the
cross-entropy bound and an exact big-integer arithmetic coder on tiny inputs.
"""
import math
import struct

import numpy as np
import pytest

from oracle import ac_bruteforce as ac
from oracle import mix_oracle as mx
from oracle import pilc_oracle as orc
from paper_2206_05279_amd import synth, synth_mix


def _geom(wl):
    return orc.make_geom(*wl.geom)


def _small(k, n=3, h=8, w=8, m=14, mode=0, la=16, lb=0, seed=5, wild=False):
    base = synth.make_random_case(seed, n, h, w, m, mode, la, lb, wild=wild)
    return synth_mix.from_base(base, k, seed)


# ------------------------------------------------------------ reductions to the single law
@pytest.mark.parametrize("m", [10, 14, 16])
def test_one_component_is_the_single_law(m):
    base = synth.make_random_case(11, 4, 8, 8, m, 0, 32)
    g = _geom(base)
    wt = np.full(base.img.shape[:3] + (1,), 32768, dtype=np.uint16)
    rc, cum, freq = mx.symbol_tables(g, 1, base.img, base.mu[..., None], base.log_scale[..., None], wt,
                                     base.chan_coef)
    cum0, freq0 = orc.symbol_tables(g, base.img, base.mu, base.log_scale, base.chan_coef)
    assert rc == mx.OK
    assert np.array_equal(cum.reshape(-1), cum0) and np.array_equal(freq.reshape(-1), freq0)
    rc, coded = mx.encode(g, 1, base.img, base.mu[..., None], base.log_scale[..., None], wt, base.chan_coef)
    rc0, coded0 = orc.encode(g, base.img, base.mu, base.log_scale, base.chan_coef)
    assert rc == mx.OK and rc0 == orc.OK
    assert coded[:4].tobytes() == b"PMIX" and coded0[:4].tobytes() == b"PILC"
    assert struct.unpack_from("<I", coded.tobytes(), 44)[0] == 1
    same = np.ones(coded.size, dtype=bool)
    same[:4] = False
    same[44:48] = False
    assert coded.size == coded0.size and np.array_equal(coded[same], coded0[same])


def test_equal_components_are_the_single_law_whatever_the_weights():
    base = synth.make_random_case(12, 3, 8, 8, 15, 1, 4, 4)
    g = _geom(base)
    k = 5
    wl = synth_mix.from_base(base, k, 12)  # only its weights are used
    mu = np.repeat(base.mu[..., None], k, axis=-1)
    ls = np.repeat(base.log_scale[..., None], k, axis=-1)
    rc, cum, freq = mx.symbol_tables(g, k, base.img, mu, ls, wl.weight, base.chan_coef)
    cum0, freq0 = orc.symbol_tables(g, base.img, base.mu, base.log_scale, base.chan_coef)
    assert rc == mx.OK and np.array_equal(cum.reshape(-1), cum0) and np.array_equal(freq.reshape(-1), freq0)


def test_zero_weight_components_do_not_matter():
    wl = _small(4, seed=21)
    g = _geom(wl)
    wt = wl.weight.copy()
    wt[..., 0] += wt[..., 3]
    wt[..., 3] = 0
    rc, cum, freq = mx.symbol_tables(g, 4, wl.img, wl.mu, wl.log_scale, wt, wl.chan_coef)
    mu2, ls2 = wl.mu.copy(), wl.log_scale.copy()
    mu2[..., 3] = 12345
    ls2[..., 3] = -7000
    rc2, cum2, freq2 = mx.symbol_tables(g, 4, wl.img, mu2, ls2, wt, wl.chan_coef)
    rc3, cum3, freq3 = mx.symbol_tables(g, 3, wl.img, wl.mu[..., :3], wl.log_scale[..., :3], wt[..., :3],
                                        wl.chan_coef)
    assert rc == rc2 == rc3 == mx.OK
    assert np.array_equal(cum, cum2) and np.array_equal(cum, cum3) and np.array_equal(freq, freq3)


# ------------------------------------------------------------ closed form and invariants
def _sigmoid(z):
    return 0.5 * (1.0 + np.tanh(0.5 * z))


def test_masses_follow_the_weighted_sum_of_logistic_differences():
    """P(v) * 2^M ~ 1 + (2^M - 256) * sum_j pi_j [s((v + 1/2 - m_j) / s_j) - s((v - 1/2 - m_j) / s_j)]
    with the outer edges at -inf / +inf, written in float64 from the definition of a discretised
    logistic mixture; means of G and B shifted by a * (x - m) of the channels before (Sec. 3.1
    eqs. (3)-(4)).  Table error of the 24-bit edge CDF is a few 2^-24 per component, the floors
    cost up to 2 units of mass."""
    k, m_bits = 3, 16
    wl = _small(k, n=2, h=4, w=4, m=m_bits, seed=33)
    g = _geom(wl)
    rc, cum, freq = mx.symbol_tables(g, k, wl.img, wl.mu, wl.log_scale, wl.weight, wl.chan_coef)
    assert rc == mx.OK
    x = wl.img.astype(np.float64)
    mu = wl.mu.astype(np.float64) / 256.0                      # [n,h,w,3,K]
    s = np.exp(np.clip(wl.log_scale.astype(np.float64) / 4096.0, -4.0, 6.0 - 1.0 / 4096))
    a = wl.chan_coef.astype(np.float64) / 16384.0               # [n,3]: a_GR, a_BR, a_BG
    a = a[:, None, None, :, None]
    e_r = x[..., 0, None] - mu[..., 0, :]
    e_g = x[..., 1, None] - mu[..., 1, :]
    me = mu.copy()
    me[..., 1, :] += a[..., 0, :] * e_r
    me[..., 2, :] += a[..., 1, :] * e_r + a[..., 2, :] * e_g
    pi = wl.weight.astype(np.float64)[..., None, :] / 32768.0  # [n,h,w,1,K]
    v = x[..., None]

    def masses(means):
        hi = np.where(v >= 255, 1.0, _sigmoid((v + 0.5 - means) / s))
        lo = np.where(v <= 0, 0.0, _sigmoid((v - 0.5 - means) / s))
        return 1.0 + (2.0 ** m_bits - 256.0) * np.sum(pi * (hi - lo), axis=-1)

    want = masses(me)
    # the shifted means are rounded to Q8.8 (one rounding per term): allow what moving every mean
    # by 1/256 does to the mass, on top of the floors
    d = 1.0 / 256.0
    slack = np.maximum(np.abs(masses(me + d) - want), np.abs(masses(me - d) - want))
    slack[..., 0] = 0.0  # red has no shift
    err = np.abs(freq.astype(np.float64) - want)
    assert np.all(err < 2.5 + slack), float(np.max(err - slack))
    assert np.median(err) < 1.0


@pytest.mark.parametrize("m", [10, 13, 16])
def test_table_invariants(m):
    rng = np.random.default_rng(m)
    for _ in range(20):
        k = int(rng.integers(1, 17))
        me = rng.integers(-70000, 140000, size=k)
        ls = rng.integers(-20000, 30000, size=k).astype(np.int16)
        wt = synth_mix.quantise_weights(rng.dirichlet(np.ones(k))[None, :])[0]
        c = [mx.cum(me, ls, wt, m, v) for v in range(257)]
        assert c[0] == 0 and c[256] == 1 << m
        assert all(b - a >= 1 for a, b in zip(c, c[1:]))


def test_weights_must_sum_to_one():
    wl = _small(3, seed=8)
    g = _geom(wl)
    bad = wl.weight.copy()
    bad[1, 2, 3, 0] += 1
    assert mx.symbol_tables(g, 3, wl.img, wl.mu, wl.log_scale, bad, wl.chan_coef)[0] == mx.E_ARG
    assert mx.encode(g, 3, wl.img, wl.mu, wl.log_scale, bad, wl.chan_coef)[0] == mx.E_ARG
    rc, coded = mx.encode(g, 3, wl.img, wl.mu, wl.log_scale, wl.weight, wl.chan_coef)
    assert rc == mx.OK
    assert mx.decode(g, 3, coded, wl.mu, wl.log_scale, bad, wl.chan_coef)[0] == mx.E_ARG
    assert mx.encode(g, 0, wl.img, wl.mu, wl.log_scale, wl.weight, wl.chan_coef)[0] == mx.E_ARG
    assert mx.encode(g, 17, wl.img, wl.mu, wl.log_scale, wl.weight, wl.chan_coef)[0] == mx.E_ARG


# ------------------------------------------------------------ coder
@pytest.mark.parametrize("k,mode,la,lb,m,wild", [(2, 0, 16, 0, 14, False), (10, 0, 64, 0, 15, False),
                                                 (3, 1, 4, 4, 12, False), (4, 0, 32, 0, 16, True),
                                                 (16, 1, 3, 5, 10, True)])
def test_round_trip_and_length_against_cross_entropy(k, mode, la, lb, m, wild):
    wl = _small(k, n=3, h=8, w=8, m=m, mode=mode, la=la, lb=lb, seed=40 + k, wild=wild)
    g = _geom(wl)
    rc, coded = mx.encode(g, k, wl.img, wl.mu, wl.log_scale, wl.weight, wl.chan_coef)
    assert rc == mx.OK
    rc, back = mx.decode(g, k, coded, wl.mu, wl.log_scale, wl.weight, wl.chan_coef)
    assert rc == mx.OK and np.array_equal(back, wl.img)
    rc, cum, freq = mx.symbol_tables(g, k, wl.img, wl.mu, wl.log_scale, wl.weight, wl.chan_coef)
    lanes = orc.lane_count(g)
    ce_bits = float(np.sum(m - np.log2(freq.astype(np.float64))))
    payload = coded.size - 64 - 4 * (lanes + 1)
    # App. A eq. (13) and the text around it: the state ends within 32 bits of the information
    # pushed into it, and a renormalised state of at least 16 bits loses at most
    # log2(1 + 2^(M-16)) bits per step; the stream cannot beat the cross entropy by more than
    # the 16 bits the start state already holds
    nsym = wl.img.size
    assert 8 * payload >= ce_bits - 16 * lanes - 1e-6
    assert 8 * payload <= ce_bits + 32 * lanes + nsym * math.log2(1 + 2.0 ** (m - 16)) + 1e-6


def test_length_against_exact_arithmetic_coding():
    k, m = 3, 12
    wl = _small(k, n=1, h=2, w=4, m=m, mode=0, la=8, seed=71)
    g = _geom(wl)
    rc, coded = mx.encode(g, k, wl.img, wl.mu, wl.log_scale, wl.weight, wl.chan_coef)
    assert rc == mx.OK
    sym = wl.img.reshape(-1)
    mu, ls = wl.mu.reshape(-1, 3, k), wl.log_scale.reshape(-1, 3, k)
    wt, coef = wl.weight.reshape(-1, k), wl.chan_coef[0]

    def cdf_fn(t, prefix):
        p, c = divmod(t, 3)
        x = [int(prefix[3 * p + i]) if i < c else 0 for i in range(3)]
        me = [orc.mean_shift(x, mu[p, :, j], coef)[c] for j in range(k)]
        return [mx.cum(me, ls[p, c], wt[p], m, v) for v in range(257)]

    bits, value = ac.encode([int(v) for v in sym], cdf_fn, m)
    assert ac.decode(bits, value, sym.size, cdf_fn, m) == [int(v) for v in sym]
    payload_bits = 8 * (coded.size - 64 - 4 * 2)
    assert payload_bits >= bits - 2
    assert payload_bits <= bits + 32 + 8  # one flushed 32-bit state, word granularity


def test_damaged_container_is_rejected():
    wl = _small(2, seed=9)
    g = _geom(wl)
    rc, coded = mx.encode(g, 2, wl.img, wl.mu, wl.log_scale, wl.weight, wl.chan_coef)
    args = (wl.mu, wl.log_scale, wl.weight, wl.chan_coef)
    bad = coded.copy(); bad[0] = ord("Q")
    assert mx.decode(g, 2, bad, *args)[0] == mx.E_FORMAT
    bad = coded.copy(); bad[44] = 3
    assert mx.decode(g, 2, bad, *args)[0] == mx.E_FORMAT
    assert mx.decode(g, 2, coded[:-2], *args)[0] == mx.E_FORMAT
    bad = coded.copy(); bad[-1] ^= 0x40
    rc, out = mx.decode(g, 2, bad, *args)
    assert rc == mx.E_CORRUPT or not np.array_equal(out, wl.img)
    assert mx.encode(g, 2, wl.img, wl.mu, wl.log_scale, wl.weight, wl.chan_coef, capacity=80)[0] == mx.E_CAPACITY
