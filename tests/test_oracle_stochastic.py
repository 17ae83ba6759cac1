"""Pins of the oracle's stochastic baselines (Sec. 5.1: Stoch-S routes requests
at random to the device while capping the server's budget, Stoch-D the mirror
image; the budget is the constrained endpoint's share of the input tokens).

None of these go through the oracle's own routing formula: the limits b = 0
and b = 1 are single-endpoint columns (evaluated by the threshold and wait
paths, pinned elsewhere), the routing frequency and the token share are
binomial around b, budget levels of one run are nested, runs are independent,
and the variate is rebuilt here from the generator's pinned raw function with
counter and key written out."""
import math

import numpy as np
import pytest

import disco_inputs as DI


def cols(oracle, mode, levels, run=0, mig=0):
    return [oracle.Policy(mode=mode, beta=DI.f32(b), l_mid=run, mig_mode=mig) for b in levels]


@pytest.fixture(scope="module")
def trace(oracle):
    return oracle.gen_trace(DI.config(0, n_req=200_000, seed=3)["gen"])


def test_limits_are_the_single_endpoint_columns(oracle, trace):
    dev_only = oracle.Policy(mode=0, l_th=2 ** 31 - 1)              # Alg. 3 with every request below the threshold
    srv_only = oracle.Policy(mode=1, l_th=-1, w_tail=math.inf)      # never start the device
    r = oracle.dispatch(trace, cols(oracle, 2, [0.0, 1.0]) + cols(oracle, 3, [0.0, 1.0]) + [dev_only, srv_only])
    for j, ref in ((0, 4), (1, 5), (2, 5), (3, 4)):      # Stoch-S: b = share of the server; Stoch-D: of the device
        assert (r["decision"][j] == r["decision"][ref]).all()
        assert (r["ttft"][j].view(np.uint32) == r["ttft"][ref].view(np.uint32)).all()
        for f in ("s_pre", "s_dec", "d_pre", "d_dec", "n_dev_started", "n_dev_win"):
            assert r[f][j] == r[f][ref], (f, j)
    assert set(np.unique(r["decision"][4])) == {6} and set(np.unique(r["decision"][5])) == {1}


@pytest.mark.parametrize("mode", [2, 3])
def test_routing_frequency_and_token_share_meet_the_budget(oracle, trace, mode):
    N = trace["n_req"]
    l = trace["prompt_len"].astype(np.float64)
    levels = [0.05, 0.3, 0.5, 0.9]
    r = oracle.dispatch(trace, cols(oracle, mode, levels, run=7))
    constrained_bit = 1 if mode == 2 else 2
    for j, b in enumerate(levels):
        dec = r["decision"][j]
        assert set(np.unique(dec)) <= {1, 6}                        # one endpoint per request, no race
        hit = (dec & constrained_bit) != 0
        # binomial: 5 standard deviations
        assert abs(hit.mean() - b) < 5 * math.sqrt(b * (1 - b) / N), (b, hit.mean())
        share = (l * hit).sum() / l.sum()                           # the paper's budget: share of the input tokens
        sd = math.sqrt(b * (1 - b) * (l ** 2).sum()) / l.sum()
        assert abs(share - b) < 5 * sd, (b, share)
        tok = r["s_pre"][j] if mode == 2 else r["d_pre"][j]
        assert tok == int((trace["prompt_len"].astype(np.int64) * hit).sum())
        # TTFT is the chosen endpoint's
        k = trace["dev_pre_spt"] if trace.get("dev_pre_spt") is not None else np.float32(trace["dev_pre_spt_s"])
        d = (trace["prompt_len"].astype(np.float32) * k).astype(np.float32)          # T_d = k l (intercept 0 here)
        srv = (dec == 1)
        assert (r["ttft"][j][srv] == trace["srv_ttft"][srv]).all() and (r["ttft"][j][~srv] == d[~srv]).all()


def test_levels_of_one_run_are_nested_and_runs_are_independent(oracle, trace):
    N = trace["n_req"]
    levels = [0.1, 0.4, 0.8]
    a = oracle.dispatch(trace, cols(oracle, 2, levels, run=0) + cols(oracle, 2, levels, run=1))["decision"] == 1
    assert not (a[0] & ~a[1]).any() and not (a[1] & ~a[2]).any()     # same draw, growing budget
    assert (a[0] != a[3]).any()
    for j in range(3):                                               # correlation of two runs at the same level
        x, y = a[j].astype(np.float64), a[j + 3].astype(np.float64)
        rho = np.corrcoef(x, y)[0, 1]
        assert abs(rho) < 5 / math.sqrt(N), rho
    # Stoch-S and Stoch-D of the same run and level use the same variate: complementary endpoints at b and 1 - b
    b = DI.f32(0.25)
    r = oracle.dispatch(trace, [oracle.Policy(mode=2, beta=b, l_mid=5), oracle.Policy(mode=3, beta=b, l_mid=5)])
    assert ((r["decision"][0] == 1) == (r["decision"][1] == 6)).all()


def test_variate_is_word_zero_of_the_pinned_generator(oracle):
    """key = (run, tag 'STOC'), counter = (i_lo, i_hi, field 6, 0); U = (floor(x / 2^9) + 1/2) 2^-23."""
    tr = {"n_req": 5, "prompt_len": np.full(5, 100, np.int32), "output_len": np.full(5, 3, np.int32),
          "srv_ttft": np.full(5, 0.5, np.float32), "srv_tbt": np.full(5, 0.05, np.float32),
          "dev_pre_spt": None, "dev_dec_spt": None, "tok_off": None, "tok_arr": None,
          "dev_pre_spt_s": 0.001, "dev_dec_spt_s": 0.05, "dev_ttft_c": 0.0}
    for run in (0, 3, 2 ** 31 - 1):
        us = []
        for i in range(5):
            x = int(oracle.philox_raw([i, 0, 6, 0], [run, 0x53544F43])[0])
            us.append(((x >> 9) + 0.5) * 2.0 ** -23)
        # routed to the constrained endpoint iff U < b: probe both sides of every variate
        for i, u in enumerate(us):
            for b, expect in ((np.nextafter(np.float32(u), np.float32(1)), True), (np.float32(u), False)):
                dec = oracle.dispatch(tr, [oracle.Policy(mode=2, beta=float(b), l_mid=run)])["decision"][0]
                assert (dec[i] == 1) == expect, (run, i, u, b)


def test_timelines_and_hand_offs_follow_the_routed_endpoint(oracle):
    tr = DI.handmade_trace(12, 600, tokens=True, max_out=150, stall_p=0.03)
    pol = cols(oracle, 2, [0.5], run=2, mig=1) + [oracle.Policy(mode=1, l_th=-1, w_tail=math.inf, mig_mode=1),
                                                   oracle.Policy(mode=0, l_th=2 ** 31 - 1, mig_mode=1)]
    d = oracle.dispatch(tr, pol)
    m = oracle.migration(tr, pol, DI.TAU, DI.KAPPA_LAG)
    srv = d["decision"][0] == 1
    # a request routed to the server has the server-only column's timeline, one routed to the device the device-only column's
    for f in ("mig_idx", "n_src_tok", "t_last"):
        assert (m[f][0][srv] == m[f][1][srv]).all() and (m[f][0][~srv] == m[f][2][~srv]).all(), f
    assert (m["mig_idx"][0][~srv] == -1).all() and (m["mig_idx"][0][srv] >= 0).sum() > 5


def test_average_over_runs_hand_computed(oracle):
    """Two groups of three runs with values chosen so that every mean is exact."""
    def rec(mean_ttft, cost, s_pre, q):
        return {"mean_ttft": mean_ttft, "mean_tbt": 0.25, "server_cost": cost, "device_energy": 0.0, "device_cost": 0.0,
                "total_cost": cost, "s_pre": s_pre, "s_dec": 1, "d_pre": 2, "d_dec": 3, "n_req": 10, "tbt_count": 4,
                "n_migrated": 0, "n_dev_started": 5, "n_dev_win": 6, "ttft_rank": [5, 10], "tbt_rank": [2, 4],
                "ttft_q": [np.float32(q), np.float32(2 * q)], "tbt_q": [np.float32(0.5), np.float32(0.75)]}
    runs = [rec(1.0, 3.0, 7, 0.5), rec(2.0, 6.0, 8, 1.5), rec(6.0, 0.0, 9, 2.5),
            rec(0.5, 1.0, 1, 4.0), rec(0.5, 1.0, 1, 4.0), rec(0.5, 1.0, 1, 4.0)]
    a = oracle.average_runs(runs, 3)
    assert len(a) == 2
    assert a[0]["mean_ttft"] == 3.0 and a[0]["server_cost"] == 3.0 and a[0]["total_cost"] == 3.0 and a[0]["mean_tbt"] == 0.25
    assert a[0]["s_pre"] == 24 and a[0]["n_req"] == 30 and a[0]["d_dec"] == 9
    assert a[0]["ttft_q"] == [np.float32(1.5), np.float32(3.0)] and a[0]["ttft_rank"] == [5, 10]
    assert a[1]["mean_ttft"] == 0.5 and a[1]["ttft_q"] == [np.float32(4.0), np.float32(8.0)] and a[1]["s_pre"] == 3
    same = oracle.average_runs(runs[3:], 1)                    # one run per group: the record itself
    assert all(same[i]["mean_ttft"] == runs[3 + i]["mean_ttft"] and same[i]["ttft_q"] == runs[3 + i]["ttft_q"] for i in range(3))
