"""Pins of the oracle's trace ingest, log-normal fit (Sec. 5.3: fitted "by
following the mean and standard deviation of the logarithm") and device
profiles (Sec. 5.1), none of them through the oracle's own formulas."""
import math
import os

import numpy as np
import pytest
import scipy.stats

from oracle import disco_ingest as I

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "device_profiles.txt")


def test_ingest_round_trip_with_dyadic_times():
    """Relative trace -> wall clock -> ingest gives the relative trace back exactly (all times multiples of 2^-10)."""
    rng = np.random.default_rng(1)
    n = 300
    out_len = rng.integers(1, 40, n)
    off = np.zeros(n + 1, np.int64)
    np.cumsum(out_len, out=off[1:])
    ttft = rng.integers(1, 4000, n) / 1024.0
    send = np.cumsum(rng.integers(0, 3000, n)) / 1024.0 + 1.7e5          # wall clock, large offset
    gaps = rng.integers(0, 300, int(off[-1])) / 1024.0
    arr = np.empty(int(off[-1]))
    tok = np.empty(int(off[-1]))
    for i in range(n):
        a, b = off[i], off[i + 1]
        arr[a] = 0
        arr[a + 1:b] = np.cumsum(gaps[a + 1:b])
        tok[a:b] = send[i] + ttft[i] + arr[a:b]
    got = I.ingest(send, tok, off)
    assert (got["srv_ttft"] == ttft.astype(np.float32)).all()
    assert (got["tok_arr"] == arr.astype(np.float32)).all()
    assert (got["output_len"] == out_len).all()
    assert (got["tok_arr"][off[:-1]] == 0).all()


def test_ingest_rounds_once():
    # a difference that is not representable in fp32: the fp64 difference rounded once
    send = np.array([1000.0])
    tok = np.array([1000.0 + 1 / 3, 1000.0 + 1 / 3 + 0.1])
    got = I.ingest(send, tok, np.array([0, 2]))
    assert got["srv_ttft"][0] == np.float32((1000.0 + 1 / 3) - 1000.0)
    assert got["tok_arr"][1] == np.float32((1000.0 + 1 / 3 + 0.1) - (1000.0 + 1 / 3))


def test_fit_matches_scipy_maximum_likelihood():
    rng = np.random.default_rng(4)
    x = rng.lognormal(5.5, 1.0, 50_000)
    f = I.fit_lognormal(x)
    s, loc, scale = scipy.stats.lognorm.fit(x, floc=0)
    assert abs(f["mu"] - math.log(scale)) < 1e-9 and abs(f["sigma"] - s) < 1e-9
    assert abs(f["mu"] - 5.5) < 0.02 and abs(f["sigma"] - 1.0) < 0.02
    assert f["n_used"] == 50_000 and f["n_skipped"] == 0


def test_fit_of_a_sample_with_known_log_moments():
    # ln x takes the values mu - 2 s, mu, mu + 2 s with weights 1, 6, 1: mean mu, variance s^2
    mu, s = -1.25, 0.5
    x = np.exp(np.array([mu - 2 * s] + [mu] * 6 + [mu + 2 * s]))
    f = I.fit_lognormal(x)
    assert abs(f["mu"] - mu) < 1e-14 and abs(f["sigma"] - s) < 1e-14
    g = I.fit_lognormal(np.concatenate([x, [0.0, -3.0]]))                 # no logarithm: left out
    assert g["n_skipped"] == 2 and g["n_used"] == 8 and abs(g["mu"] - mu) < 1e-14
    assert math.isnan(I.fit_lognormal(np.zeros(3))["mu"])
    ints = I.fit_lognormal(np.array([1, 2, 4, 8], np.int32))              # prompt lengths are integers
    assert abs(ints["mu"] - 1.5 * math.log(2)) < 1e-15 and abs(ints["sigma"] - math.log(2) * math.sqrt(1.25)) < 1e-15


def test_device_profiles_are_the_printed_speeds():
    rows = [ln.split("|") for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == len(I.DEVICE_PROFILES) == 3
    for idx, (dev, model, pre, dec) in enumerate(rows):
        p = I.device_profile(idx)
        assert p["device"] == dev.strip() and p["model"] == model.strip()
        assert p["dev_pre_spt_s"] == np.float32(1.0 / float(pre)) and p["dev_dec_spt_s"] == np.float32(1.0 / float(dec))
        # a 100-token prompt: device TTFT = 100 / prefill speed
        assert abs(float(p["dev_pre_spt_s"]) * 100 - 100 / float(pre)) < 1e-5
