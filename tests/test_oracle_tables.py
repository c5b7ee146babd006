"""Pins for the oracle's per-symbol arithmetic: constant tables, inverse scale, edge CDF,
cumulative counts, mean shift.  None of the expectations below is produced by the oracle."""
import hashlib
import math
import os

import numpy as np
import pytest

from oracle import pilc_oracle as orc


def _read_rows(path):
    with open(path) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_table_constants_match_golden(golden_dir):
    t, eh, el = orc.tables()
    tabs = {"T": t, "EH": eh, "EL": el}
    for row in _read_rows(os.path.join(golden_dir, "table_constants.txt")):
        if row[0] == "value":
            assert int(tabs[row[1]][int(row[2])]) == int(row[3]), row
        else:
            digest = hashlib.sha256(tabs[row[1]].astype("<u4").tobytes()).hexdigest()
            assert digest == row[2], row


def test_tables_follow_closed_forms():
    t, eh, el = orc.tables()
    i = np.arange(2049, dtype=np.float64)
    assert np.max(np.abs(t - 2.0**24 / (1.0 + np.exp(-(i - 1024) / 64)))) <= 0.5 + 1e-6
    i = np.arange(640, dtype=np.float64)
    assert np.max(np.abs(eh - 2.0**26 * np.exp(4 - i / 64))) <= 0.5 + 1e-6
    j = np.arange(64, dtype=np.float64)
    assert np.max(np.abs(el - 2.0**31 * np.exp(-j / 4096))) <= 0.5 + 1e-6
    assert np.all(np.diff(t.astype(np.int64)) >= 0)


def test_inv_scale_tracks_exp_and_clamps():
    worst = 0.0
    for ls_q in range(-16384, 24576, 7):
        got = orc.inv_scale(ls_q) / 2.0**25
        want = math.exp(-ls_q / 4096.0)
        worst = max(worst, abs(got / want - 1.0))
    assert worst <= 2.0**-15
    assert orc.inv_scale(-32768) == orc.inv_scale(-16384)
    assert orc.inv_scale(32767) == orc.inv_scale(24575)
    # strictly positive and non-increasing over every 16-bit code
    prev = None
    for ls_q in range(-32768, 32768):
        v = orc.inv_scale(ls_q)
        assert v > 0
        assert prev is None or v <= prev
        prev = v


def test_edge_cdf_tracks_float64_logistic():
    rng = np.random.default_rng(1)
    worst = 0.0
    for _ in range(3000):
        mu = int(rng.integers(-70000, 140000))
        ls_q = int(rng.integers(-16384, 24576))
        inv_s = orc.inv_scale(ls_q)
        s = math.exp(ls_q / 4096.0)
        for k in rng.integers(1, 256, size=6):
            z = (float(k) - 0.5 - mu / 256.0) / s
            z = max(-16.0, min(16.0, z))
            want = 1.0 / (1.0 + math.exp(-z))
            got = orc.edge_cdf(mu, inv_s, int(k)) / 2.0**24
            worst = max(worst, abs(got - want))
    # tolerance: 2^-16 from the sigmoid table, plus the argument error |z| * 2^-15 of inv_s
    # times the maximum slope 1/4 of the sigmoid -> well under 2^-12 overall
    assert worst <= 2.0**-12


def test_edge_cdf_tight_where_argument_is_exact():
    # log_scale = 0 -> inv_s = 2^25 exactly, so only the sigmoid table's own error remains
    assert orc.inv_scale(0) == 1 << 25
    worst = 0.0
    for mu in range(0, 65536, 997):
        for k in range(1, 256, 3):
            z = float(k) - 0.5 - mu / 256.0
            z = max(-16.0, min(16.0 - 2.0**-16, z))
            want = 1.0 / (1.0 + math.exp(-z))
            worst = max(worst, abs(orc.edge_cdf(mu, 1 << 25, k) / 2.0**24 - want))
    assert worst <= 2.0**-16


def test_golden_cumulative_counts(golden_dir):
    ks = (1, 64, 100, 101, 128, 200, 255)
    for row in _read_rows(os.path.join(golden_dir, "cdf_examples.txt")):
        mu_q, ls_q, m, inv_s = (int(v) for v in row[:4])
        assert orc.inv_scale(ls_q) == inv_s
        for k, want in zip(ks, row[4:]):
            assert orc.cum(mu_q, ls_q, m, k) == int(want), (row, k)


def test_golden_mean_shift(golden_dir):
    for row in _read_rows(os.path.join(golden_dir, "mean_shift_example.txt")):
        v = [int(a) for a in row if a != "->"]
        assert orc.mean_shift(v[0:3], v[3:6], v[6:9]) == v[9:12]


def test_mean_shift_special_cases():
    # zero innovation or zero coefficients: means unchanged
    assert orc.mean_shift([10, 20, 30], [2560, 5120, 999], [16384, -16384, 777]) == [2560, 5120, 999]
    assert orc.mean_shift([200, 3, 77], [100, 60000, 31000], [0, 0, 0]) == [100, 60000, 31000]
    # coefficient 1.0 in Q2.14 adds the innovation itself
    assert orc.mean_shift([100, 50, 0], [25000, 13000, 4000], [16384, 0, 16384]) == \
        [25000, 13000 + (25600 - 25000), 4000 + (12800 - 13000)]
    # rounding is to nearest with ties upward, also for negative products: -1.5 -> -1, 1.5 -> 2
    assert orc.mean_shift([1, 0, 0], [253, 0, 0], [8192, -8192, 0]) == [253, 2, -1]
    # extreme magnitudes stay exact
    mu_g = orc.mean_shift([255, 0, 0], [0, 0, 0], [-32768, 32767, 32767])
    assert mu_g[1] == -2 * 65280
    assert mu_g[2] == (32767 * 65280 + 8192) // 16384


@pytest.mark.parametrize("m", [10, 11, 12, 13, 14, 15, 16])
def test_cumulative_counts_invariants(m):
    """Sec. 3.2: sum of masses is 2^M, C_x = sum_{i<x} P_i; here also every mass >= 1."""
    rng = np.random.default_rng(m)
    cases = [(0, -32768), (65535, 32767), (-300000, -16384), (400000, 24575), (32768, 0)]
    cases += [(int(rng.integers(-200000, 300000)), int(rng.integers(-32768, 32768)))
              for _ in range(150)]
    for mu, ls_q in cases:
        c = [orc.cum(mu, ls_q, m, k) for k in range(257)]
        assert c[0] == 0 and c[256] == 1 << m
        d = np.diff(np.array(c, dtype=np.int64))
        assert d.min() >= 1 and d.sum() == 1 << m and d.max() <= (1 << m) - 255


def test_cumulative_counts_follow_logistic_mass():
    """freq(v)/2^M ~= the logistic mass of [v-1/2, v+1/2) (tails folded into 0 and 255), up to
    the one reserved count per symbol."""
    m = 16
    rng = np.random.default_rng(7)
    for _ in range(200):
        mu = int(rng.integers(0, 65536))
        ls_q = int(rng.integers(-8192, 16384))
        s = math.exp(ls_q / 4096.0)
        cdf = lambda e: 1.0 / (1.0 + math.exp(-max(-30.0, min(30.0, (e - mu / 256.0) / s))))
        for v in rng.integers(0, 256, size=8):
            v = int(v)
            lo = 0.0 if v == 0 else cdf(v - 0.5)
            hi = 1.0 if v == 255 else cdf(v + 0.5)
            f = orc.cum(mu, ls_q, m, v + 1) - orc.cum(mu, ls_q, m, v)
            want = 1 + (hi - lo) * ((1 << m) - 256)
            assert abs(f - want) <= 2 + 2.0**-11 * (1 << m), (mu, ls_q, v, f, want)
