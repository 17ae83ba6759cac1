"""Pins for the oracle's paced delivery (max-plus recurrence) and lag-triggered
migration: brute force in exact rational arithmetic, special cases with known
answers, invariants of the buffer semantics, constructed stall cases."""
import math
from fractions import Fraction

import numpy as np
import pytest

import disco_inputs as DI

TAU = np.float32(0.25)     # dyadic: every product t*tau below is exact in fp32


def brute_delivery(r, tau):
    """delta_t = max_{u <= t} (r_u + (t - u) tau), O(n^2), exact rationals."""
    r = [Fraction(float(x)) for x in r]
    tau = Fraction(float(tau))
    return [max(r[u] + (t - u) * tau for u in range(t + 1)) for t in range(len(r))]


def sequential_delivery(r, tau):
    """delta_0 = r_0, delta_t = max(r_t, delta_{t-1} + tau) in exact rationals."""
    out = []
    for t, x in enumerate(r):
        x = Fraction(float(x))
        out.append(x if t == 0 else max(x, out[-1] + Fraction(float(tau))))
    return out


def run(oracle, r, tau=TAU, lag=False, src_dev=False, l=100, k=1 / 800, g=0.05, kappa=3.0, gap=0.0):
    n = len(r) if r is not None else 0
    return oracle.timeline(n, r, gap, src_dev, lag, float(tau), kappa, l, k, 0.0, g)


def test_scan_matches_brute_force_on_dyadic_inputs(oracle):
    rng = np.random.default_rng(0)
    for trial in range(40):
        n = int(rng.integers(1, 40))
        gaps = rng.integers(0, 64, n).astype(np.float32) / np.float32(64)       # multiples of 1/64
        r = np.concatenate([[0], np.cumsum(gaps[1:], dtype=np.float32)]).astype(np.float32)
        m, tl, delivered, tbt = run(oracle, r)
        want = brute_delivery(r, TAU)
        assert [Fraction(float(x)) for x in delivered] == want
        assert want == sequential_delivery(r, TAU)
        assert m == -1 and Fraction(float(tl)) == want[-1]
        assert [Fraction(float(x)) for x in tbt] == [want[t] - want[t - 1] for t in range(1, n)]


def test_scan_close_to_brute_force_on_general_inputs(oracle):
    rng = np.random.default_rng(1)
    tau = np.float32(0.2)
    for trial in range(20):
        n = int(rng.integers(2, 200))
        r = np.concatenate([[0], np.cumsum(rng.lognormal(-3.5, 0.8, n - 1))]).astype(np.float32)
        r[rng.integers(1, n):] += np.float32(1.3)          # one stall
        _, _, delivered, _ = run(oracle, r, tau=tau)
        want = brute_delivery(r, tau)
        for t in range(n):
            ulp = float(np.spacing(np.float32(float(want[t]))))
            assert abs(Fraction(float(delivered[t])) - want[t]) <= 2 * ulp


def test_fast_source_is_paced_and_slow_source_passes_through(oracle):
    n = 50
    fast = (np.arange(n) * np.float32(1 / 16)).astype(np.float32)     # gaps 1/16 < tau
    _, tl, delivered, tbt = run(oracle, fast)
    assert (delivered == np.arange(n) * TAU).all() and (tbt == TAU).all() and tl == (n - 1) * TAU
    slow = (np.arange(n) * np.float32(0.5)).astype(np.float32)        # gaps 1/2 > tau
    _, _, delivered, tbt = run(oracle, slow)
    assert (delivered == slow).all() and (tbt == 0.5).all()
    # constant-gap forms (no per-token trace) are the same sequences
    _, _, d2, _ = oracle.timeline(n, None, 1 / 16, False, False, float(TAU), 3.0, 1, 0.0, 0.0, 0.0)
    assert (d2 == np.arange(n) * TAU).all()
    _, _, d3, _ = oracle.timeline(n, None, 0.0, True, False, float(TAU), 3.0, 1, 0.0, 0.0, 0.5)
    assert (d3 == slow).all()
    # single token: no gaps at all
    m, tl, d1, tbt1 = run(oracle, np.zeros(1, np.float32))
    assert m == -1 and tl == 0 and d1.tolist() == [0.0] and tbt1.size == 0


def test_delivery_invariants_on_synthetic_tokens(oracle):
    cfg = DI.config(2, n_req=300)
    tr = oracle.gen_trace(cfg["gen"], tokens=True)
    tau = np.float32(cfg["tau"])
    for i in range(tr["n_req"]):
        r = tr["tok_arr"][tr["tok_off"][i]:tr["tok_off"][i + 1]]
        _, _, delivered, tbt = run(oracle, r, tau=tau)
        assert (delivered >= r).all()
        assert (np.diff(delivered) >= 0).all()
        slack = 2 * np.spacing(delivered[1:])
        assert (tbt >= tau - slack).all()


def test_no_stall_means_no_migration(oracle):
    rng = np.random.default_rng(2)
    for _ in range(20):
        n = int(rng.integers(2, 300))
        gaps = rng.uniform(0, float(TAU), n - 1).astype(np.float32)      # every gap <= tau
        r = np.concatenate([[0], np.cumsum(gaps, dtype=np.float32)]).astype(np.float32)
        m, _, _, _ = run(oracle, r, lag=True)
        assert m == -1
    # a device source never lags (constant gaps), even when slower than the pacing
    m, _, _, _ = oracle.timeline(100, None, 0.0, True, True, float(TAU), 3.0, 10, 1 / 800, 0.0, 2.0)
    assert m == -1


@pytest.mark.parametrize("t0", [1, 2, 17, 63, 64, 65, 130])
def test_single_stall_with_an_empty_buffer(oracle, t0):
    # source exactly at the pacing rate (buffer always empty), one stall of S seconds in front of token t0
    n = 200
    l, k, g = 160, np.float32(1 / 64), np.float32(0.5)       # dyadic: t_mig exact
    for S, fires in [(0.5, False), (0.75, False), (1.0, True), (4.0, True)]:
        # lag = (S + tau) - tau - ... : token t0 arrives at (t0-1) tau + tau + S; its slot is t0 tau; lag = S; 3 tau = 0.75
        r = (np.arange(n) * TAU).astype(np.float32)
        r[t0:] += np.float32(S)
        m, tl, delivered, tbt = run(oracle, r, lag=True, l=l, k=float(k), g=float(g))
        if not (S > 3 * float(TAU)):
            assert m == -1
            continue
        assert fires and m == t0
        # before the hand-off nothing changes
        assert (delivered[:t0] == np.arange(t0) * TAU).all()
        # hand-off: decision at slot + 3 tau, re-prefill of l + m tokens, then the device's constant gap
        t_dec = t0 * float(TAU) + 3 * float(TAU)
        t_mig = (l + t0) * float(k)
        first = t_dec + t_mig + float(g)
        assert delivered[t0] == np.float32(first)
        assert (tbt[t0:] == max(float(g), float(TAU))).all() and len(tbt[t0:]) == n - t0 - 1
        assert tl == np.float32(first + (n - 1 - t0) * max(float(g), float(TAU)))


def test_buffered_tokens_absorb_a_stall(oracle):
    # a fast source builds a buffer: the same stall that fires with an empty buffer is absorbed
    n, t0 = 200, 100
    r = (np.arange(n) * np.float32(1 / 16)).astype(np.float32)
    r[t0:] += np.float32(2.0)
    m, _, delivered, _ = run(oracle, r, lag=True)
    # token t0 arrives at 100/16 + 2 = 8.25 s; its paced slot is 100 * 0.25 = 25 s: not late at all
    assert m == -1 and (delivered == np.arange(n) * TAU).all()
    # the same stall right at the start is late by 2 - 0.25 + 1/16 > 3 tau
    r = (np.arange(n) * np.float32(1 / 16)).astype(np.float32)
    r[1:] += np.float32(2.0)
    m, _, _, _ = run(oracle, r, lag=True)
    assert m == 1


def test_fast_device_after_hand_off_is_paced(oracle):
    n, t0 = 50, 10
    r = (np.arange(n) * TAU).astype(np.float32)
    r[t0:] += np.float32(2.0)
    g = 1 / 16           # device faster than the pacing: deliveries continue every tau
    m, tl, delivered, tbt = run(oracle, r, lag=True, l=64, k=1 / 64, g=g)
    assert m == t0
    assert (tbt[t0:] == TAU).all()
    assert delivered[t0] == np.float32(t0 * 0.25 + 0.75 + (64 + t0) / 64 + g)


def test_migration_token_accounting(oracle):
    P = oracle.Policy
    tr = DI.handmade_trace(11, 400, tokens=True, stall_p=0.05)
    tau, kappa = 0.2, 3.0
    pol = [P(mode=1, l_th=-1, w_tail=math.inf, mig_mode=1),      # all server-sourced, lag hand-off
           P(mode=1, l_th=-1, w_tail=math.inf, mig_mode=0),      # all server-sourced, no hand-off
           P(mode=0, l_th=10 ** 9, mig_mode=1)]                  # all device-sourced
    r = oracle.migration(tr, pol, tau, kappa, tbt_col=0, want_delivered=True)
    n = tr["output_len"].astype(np.int64)
    l = tr["prompt_len"].astype(np.int64)
    m = r["mig_idx"][0].astype(np.int64)
    mig = m >= 0
    assert mig.any() and (~mig).any()
    assert ((m >= 1) | ~mig).all() and (m < n).all()
    assert (r["n_src_tok"][0] == np.where(mig, m, n)).all()
    assert r["m_s_dec"][0] == np.where(mig, m, n).sum()
    assert r["m_d_dec"][0] == np.where(mig, n - m, 0).sum()
    assert r["m_d_repre"][0] == (l + m)[mig].sum()
    assert r["n_migrated"][0] == mig.sum()
    assert r["tbt_count"][0] == (n - 1).sum() == r["tbt"].size
    # no hand-off / device source: the source produces every token
    assert (r["mig_idx"][1] == -1).all() and r["m_s_dec"][1] == n.sum() and r["m_d_dec"][1] == 0
    assert (r["mig_idx"][2] == -1).all() and r["m_d_dec"][2] == n.sum() and r["m_s_dec"][2] == 0
    # mean TBT telescopes: sum of last delivery offsets = sum of all gaps
    assert abs(r["tlast_sum"][0] - r["tbt"].astype(np.float64).sum()) <= 1e-6 * r["tlast_sum"][0]
    # per-request check of the first hand-off index against the definition, from the delivered offsets
    off = tr["tok_off"]
    kt = np.float32(kappa) * np.float32(tau)
    for i in range(tr["n_req"]):
        rr = tr["tok_arr"][off[i]:off[i + 1]]
        dd = r["delivered"][off[i]:off[i + 1]]
        lag = rr[1:] - (dd[:-1] + np.float32(tau))
        upto = int(m[i]) if mig[i] else len(rr)
        assert not (lag[:max(upto - 1, 0)] > kt).any()
        if mig[i]:
            assert lag[m[i] - 1] > kt
            assert r["t_last"][0][i] == dd[-1]
    # without hand-off the same requests show the stall as a long gap; with it the tail is the device's pace
    st = oracle.stats(tr, pol[:2], DI.COST_S, tau=tau, kappa=kappa)
    assert st[0]["n_migrated"] == mig.sum() and st[1]["n_migrated"] == 0
    assert st[0]["s_dec"] + st[0]["d_dec"] == n.sum()
    assert st[0]["tbt_q"][0] >= np.float32(tau) - 1e-4
