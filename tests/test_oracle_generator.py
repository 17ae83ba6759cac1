"""Pins for the oracle's random generator, elementary functions and samplers.

Philox is pinned to the publication's known-answer vectors; the fp32
elementary functions to libm in fp64; the samplers to closed forms of the
distributions they claim to draw from."""
import math
import os

import numpy as np
import pytest

import disco_inputs as DI

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def test_philox_known_answers(oracle):
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        v = [int(x, 16) for x in row]
        got = oracle.philox_raw(v[0:4], v[4:6])
        assert [int(x) for x in got] == v[6:10]


def test_philox_counter_layout(oracle):
    # element (seed, index, field) = raw call with ctr = (idx_lo, idx_hi, field, 0), key = seed halves
    seed, index, field = 0x0123456789ABCDEF, 0x1_0000_0007, 5
    a = oracle.philox(seed, index, field)
    b = oracle.philox_raw((index & 0xFFFFFFFF, index >> 32, field, 0), (seed & 0xFFFFFFFF, seed >> 32))
    assert (a == b).all()
    # distinct fields / indices give distinct words
    assert not (oracle.philox(seed, index, 4) == a).all()
    assert not (oracle.philox(seed, index + 1, field) == a).all()


def test_philox_bits_look_uniform(oracle):
    words = np.array([oracle.philox(7, i, 0) for i in range(4096)], dtype=np.uint32).ravel()
    bits = np.unpackbits(words.view(np.uint8))
    n = bits.size
    assert abs(bits.mean() - 0.5) < 4 * 0.5 / math.sqrt(n)
    # byte histogram chi-square (255 dof): mean 255, sd ~22.6
    h = np.bincount(words.view(np.uint8), minlength=256)
    chi2 = ((h - h.mean()) ** 2 / h.mean()).sum()
    assert chi2 < 255 + 6 * 22.6


def test_u23_is_exact_and_open(oracle):
    L = oracle.lib()
    assert L.orc_u23(0) == 2.0 ** -24
    assert L.orc_u23(0xFFFFFFFF) == 1.0 - 2.0 ** -24
    for x in (1 << 9, 12345 << 9, 0x80000000):
        assert L.orc_u23(x) == ((x >> 9) + 0.5) * 2.0 ** -23


def _rel(a, b):
    return abs(a - b) / abs(b)


def test_ln_against_libm(oracle):
    L = oracle.lib()
    rng = np.random.default_rng(1)
    xs = np.concatenate([
        np.exp(rng.uniform(-17, 17, 4000)), 1.0 + rng.uniform(-1e-3, 1e-3, 500),
        [2.0 ** -24, 1 - 2.0 ** -24, 0.5, 1.0, 2.0, math.sqrt(2), math.sqrt(0.5)]]).astype(np.float32)
    for x in xs:
        got = L.orc_ln(float(x))
        ref = math.log(float(x))
        assert abs(got - ref) <= 3e-7 * abs(ref) + 1e-9, (x, got, ref)
    assert L.orc_ln(1.0) == 0.0


def test_exp_against_libm(oracle):
    L = oracle.lib()
    rng = np.random.default_rng(2)
    xs = np.concatenate([rng.uniform(-80, 80, 4000), rng.uniform(-1, 1, 1000), [0.0, -86.0, 88.0]]).astype(np.float32)
    for x in xs:
        assert _rel(L.orc_exp(float(x)), math.exp(float(x))) < 4e-7, x
    assert L.orc_exp(0.0) == 1.0
    # clamps
    assert L.orc_exp(-1000.0) == L.orc_exp(-86.0)
    assert L.orc_exp(1000.0) == L.orc_exp(88.0)
    assert math.isfinite(L.orc_exp(1000.0))


def test_cos2pi_against_libm(oracle):
    L = oracle.lib()
    rng = np.random.default_rng(3)
    us = np.concatenate([rng.random(5000), [2.0 ** -24, 1 - 2.0 ** -24, 0.125, 0.25, 0.375, 0.5, 0.625, 0.75, 0.875]]).astype(np.float32)
    for u in us:
        assert abs(L.orc_cos2pi(float(u)) - math.cos(2 * math.pi * float(u))) < 3e-7, u
    assert L.orc_cos2pi(0.5) == -1.0
    assert L.orc_cos2pi(0.25) == 0.0


def test_normal_moments(oracle):
    L = oracle.lib()
    rng = np.random.default_rng(4)
    w = rng.integers(0, 2 ** 32, (200_000, 2), dtype=np.uint64)
    z = np.array([L.orc_normal(int(a), int(b)) for a, b in w[:60_000]])
    n = z.size
    assert abs(z.mean()) < 5 / math.sqrt(n)
    assert abs(z.var() - 1) < 5 * math.sqrt(2 / n)
    assert abs((z ** 3).mean()) < 5 * math.sqrt(15 / n)
    assert abs((z ** 4).mean() - 3) < 5 * math.sqrt(96 / n)
    assert abs((z < 1.0).mean() - 0.841345) < 5 * math.sqrt(0.1335 / n)


@pytest.fixture(scope="module")
def big_trace(oracle):
    cfg = DI.config(2, n_req=200_000)
    return cfg, oracle.gen_requests(cfg["gen"])


def test_request_fields_follow_their_laws(oracle, big_trace):
    cfg, tr = big_trace
    g = cfg["gen"]
    n = tr["n_req"]
    se = 1 / math.sqrt(n)
    # per-request server gap: unclipped log-normal -> mean/sd of the logarithm
    lg = np.log(tr["srv_tbt"].astype(np.float64))
    assert abs(lg.mean() - g["tbt_mu"]) < 5 * g["tbt_sigma"] * se
    assert abs(lg.std() - g["tbt_sigma"]) < 5 * g["tbt_sigma"] * se
    assert abs(tr["srv_tbt"].astype(np.float64).mean() - math.exp(g["tbt_mu"] + g["tbt_sigma"] ** 2 / 2)) < 5 * 0.01 * se * 3
    # prompt length: floor of a log-normal clipped to [8, 4096]: median and clip bounds
    pl = tr["prompt_len"]
    assert pl.min() == g["prompt_lo"] and pl.max() == g["prompt_hi"]
    med = math.exp(g["prompt_mu"])          # 244.69 -> floor 244
    frac_below = (pl <= math.floor(med) - 1).mean()   # P(X < 244) just under 1/2
    assert abs(frac_below - 0.5) < 0.01
    # share at the lower clip = Phi((ln 9 - mu)/sigma)  (floor(x) <= 8  <=>  x < 9)
    phi = 0.5 * (1 + math.erf((math.log(9) - g["prompt_mu"]) / g["prompt_sigma"] / math.sqrt(2)))
    assert abs((pl == 8).mean() - phi) < 5 * math.sqrt(phi * se * se)
    # output length: clip [1, 2048]
    ol = tr["output_len"]
    assert ol.min() >= 1 and ol.max() == 2048
    assert abs(np.median(ol) - math.floor(math.exp(g["out_mu"]))) <= 3
    # CSR offsets are the exclusive prefix sum of output lengths
    assert tr["tok_off"][0] == 0
    assert (np.diff(tr["tok_off"]) == ol).all()


def test_server_ttft_is_a_mixture(oracle, big_trace):
    cfg, tr = big_trace
    g = cfg["gen"]
    s = tr["srv_ttft"].astype(np.float64)
    n = s.size
    p, xm, al = g["ttft_pareto_p"], g["ttft_pareto_xm"], g["ttft_pareto_alpha"]

    def ln_sf(x):
        return 0.5 * math.erfc((math.log(x) - g["ttft_mu"]) / g["ttft_sigma"] / math.sqrt(2))

    for x in (0.2, 0.3, 0.6, 1.0, 3.0, 10.0):
        pareto_sf = 1.0 if x < xm else (xm / x) ** al
        want = (1 - p) * ln_sf(x) + p * pareto_sf
        got = (s > x).mean()
        assert abs(got - want) < 5 * math.sqrt(max(want * (1 - want), 1e-6) / n) + 1e-4, (x, got, want)
    assert s.min() > 0


def test_device_speed_modes(oracle):
    c2 = DI.config(2, n_req=50_000)
    tr = oracle.gen_requests(c2["gen"])
    rate = 1.0 / tr["dev_dec_spt"].astype(np.float64)
    assert rate.min() >= 15 - 1e-4 and rate.max() <= 40 + 1e-4
    assert abs(rate.mean() - 27.5) < 5 * (25 / math.sqrt(12)) / math.sqrt(rate.size)
    np.testing.assert_allclose(tr["dev_pre_spt"], tr["dev_dec_spt"] / np.float32(40), rtol=1e-7)
    c4 = DI.config(4, n_req=50_000)
    tr = oracle.gen_requests(c4["gen"])
    vals = np.unique(tr["dev_dec_spt"])
    assert set(vals.tolist()) == {float(np.float32(1) / np.float32(8)), float(np.float32(1) / np.float32(40))}
    assert abs((tr["dev_dec_spt"] == vals.max()).mean() - 0.5) < 5 * 0.5 / math.sqrt(50_000)
    assert tr["prompt_len"].max() <= 32768
    c0 = DI.config(0, n_req=100)
    tr = oracle.gen_requests(c0["gen"])
    assert (tr["dev_dec_spt"] == np.float32(1 / 20)).all() and (tr["dev_pre_spt"] == np.float32(1 / 800)).all()


def test_token_arrivals(oracle):
    cfg = DI.config(2, n_req=3000)
    g = cfg["gen"]
    tr = oracle.gen_trace(g, tokens=True)
    off, arr = tr["tok_off"], tr["tok_arr"]
    assert arr.size == off[-1]
    assert (arr[off[:-1]] == 0).all()
    gaps = []
    for i in range(tr["n_req"]):
        seg = arr[off[i]:off[i + 1]].astype(np.float64)
        assert (np.diff(seg) > 0).all()
        gaps.append(np.diff(seg))
    gaps = np.concatenate(gaps)
    n = gaps.size
    # stalls are the only gaps >= 0.5 s (log-normal(-3.5, 0.6) above 0.5 s has probability ~1e-6)
    stall = gaps > 0.45
    assert abs(stall.mean() - g["gap_stall_p"]) < 5 * math.sqrt(0.01 * 0.99 / n)
    assert gaps[stall].max() < 2.0 + 1e-2 and abs(gaps[stall].mean() - 1.25) < 5 * (1.5 / math.sqrt(12)) / math.sqrt(stall.sum()) + 1e-3
    lg = np.log(gaps[~stall])
    # differences of a running fp32 sum carry rounding noise of the offsets; loose bounds
    assert abs(lg.mean() - g["gap_mu"]) < 0.01
    assert abs(lg.std() - g["gap_sigma"]) < 0.01
    # slices regenerate identically (counter-based)
    part = oracle.gen_tokens(g, off, 100, 110)
    assert (part == arr[off[100]:off[110]]).all()
    # the running sum is the sequential fp32 sum of the per-token draws
    L = oracle.lib()
    L.orc_gen_gap.argtypes = [__import__("ctypes").c_void_p, __import__("ctypes").c_int64]
    gc = oracle._cfg(g)
    import ctypes
    i = 7
    acc = np.float32(0)
    for j in range(int(off[i]) + 1, int(off[i + 1])):
        acc = np.float32(acc + np.float32(L.orc_gen_gap(ctypes.addressof(gc), j)))
        assert acc == arr[j]
