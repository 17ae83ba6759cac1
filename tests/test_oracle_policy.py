"""Pins for the oracle's dispatch, cost, statistics and budget search.

Each check compares the oracle with something fixed by the paper or by plain
mathematics (degenerate policies, closed forms, sort-based solves, brute
force), never with the oracle's own formulas retyped."""
import math
from fractions import Fraction
from statistics import NormalDist

import numpy as np
import pytest

import disco_inputs as DI


@pytest.fixture(scope="module")
def tr0(oracle):
    return oracle.gen_trace(DI.config(0, n_req=20_000)["gen"])


def _d(tr):
    k = tr["dev_pre_spt"] if tr["dev_pre_spt"] is not None else np.float32(tr["dev_pre_spt_s"])
    # k*l + 0 has a single rounding, so the fp32 product is the fused result when c = 0
    return (tr["prompt_len"].astype(np.float32) * k).astype(np.float32)


def test_zero_budget_runs_everything_on_the_device(oracle, tr0):
    # Alg. 3 with a threshold above every prompt: device only, TTFT = k l + c, no server tokens
    P = oracle.Policy
    big = int(tr0["prompt_len"].max()) + 1
    r = oracle.dispatch(tr0, [P(mode=0, l_th=big)])
    assert (r["decision"] == 6).all()
    assert (r["ttft"][0] == _d(tr0)).all()
    assert r["s_pre"][0] == 0 and r["s_dec"][0] == 0
    assert r["d_pre"][0] == tr0["prompt_len"].sum() and r["d_dec"][0] == tr0["output_len"].sum()
    assert r["n_dev_started"][0] == tr0["n_req"] == r["n_dev_win"][0]


def test_full_budget_races_everything(oracle, tr0):
    P = oracle.Policy
    r = oracle.dispatch(tr0, [P(mode=0, l_th=0), P(mode=1, l_th=-1, w_tail=0.0)])
    d, s = _d(tr0), tr0["srv_ttft"]
    for j in range(2):
        assert (r["ttft"][j] == np.minimum(s, d)).all()
        assert set(np.unique(r["decision"][j])) <= {3, 7}
        assert ((r["decision"][j] == 7) == (d < s)).all()
        assert r["s_pre"][j] == r["d_pre"][j] == tr0["prompt_len"].sum()
        assert r["s_dec"][j] + r["d_dec"][j] == tr0["output_len"].sum()
        assert r["d_dec"][j] == tr0["output_len"][d < s].sum()


def test_wait_beyond_every_server_ttft_is_server_only(oracle, tr0):
    P = oracle.Policy
    w = float(tr0["srv_ttft"].max()) * 2
    r = oracle.dispatch(tr0, [P(mode=1, l_th=-1, w_tail=w), P(mode=1, l_th=-1, w_tail=math.inf)])
    for j in range(2):
        assert (r["decision"][j] == 1).all()
        assert (r["ttft"][j] == tr0["srv_ttft"]).all()
        assert r["d_pre"][j] == 0 and r["d_dec"][j] == 0 and r["n_dev_started"][j] == 0
    cost = DI.COST_D
    tot = oracle.total_cost(cost, r["s_pre"][0], r["s_dec"][0], r["d_pre"][0], r["d_dec"][0])
    closed = cost["cs_pre"] * (int(tr0["prompt_len"].sum()) + int(tr0["output_len"].sum()))
    assert abs(tot - closed) <= 1e-12 * closed


def test_server_ttft_below_the_wait_is_reproduced(oracle, tr0):
    # device-constrained, any wait: requests whose server answers before the wait keep the server TTFT
    P = oracle.Policy
    w = 0.35
    r = oracle.dispatch(tr0, [P(mode=1, l_th=-1, w_tail=w)])
    s, d = tr0["srv_ttft"], _d(tr0)
    w32 = np.float32(w)
    early = s <= w32
    assert (r["ttft"][0][early] == s[early]).all() and (r["decision"][0][early] == 1).all()
    late = ~early
    x = (w32 + d).astype(np.float32)
    assert (r["ttft"][0][late] == np.minimum(s, x)[late]).all()
    assert ((r["decision"][0] == 7) == (late & (x < s))).all()
    assert ((r["decision"][0] == 3) == (late & ~(x < s))).all()
    assert r["d_pre"][0] == tr0["prompt_len"][late].sum()


def test_wait_function_shapes(oracle):
    import ctypes
    L = oracle.lib()
    P = oracle._Policy

    def w(p, l):
        L.orc_wait.argtypes = [ctypes.c_void_p, ctypes.c_int32]
        return L.orc_wait(ctypes.addressof(p), l)
    inf = math.inf
    ramp = P(1, 100, -1, 0.0, 0.001, 0.5, 0)          # Eq. 1: 0 up to l_th, then min(beta l, w_tail)
    assert w(ramp, 100) == 0.0 and w(ramp, 50) == 0.0
    assert w(ramp, 101) == float(np.float32(0.001) * np.float32(101))
    assert w(ramp, 1000) == 0.5
    step = P(1, 100, 101, 0.25, inf, 0.5, 0)           # Alg. 2: zeros, one partial wait, then w_tail
    assert [w(step, l) for l in (99, 100, 101, 102, 5000)] == [0.0, 0.0, 0.25, 0.5, 0.5]
    glob = P(1, -1, -1, 0.0, inf, 0.75, 0)
    assert [w(glob, l) for l in (0, 1, 4096)] == [0.75, 0.75, 0.75]


def test_ties_and_boundaries(oracle):
    P = oracle.Policy
    k = float(np.float32(1 / 800))
    l = np.array([800, 800, 800, 100, 101], np.int32)
    d800 = float(np.float32(800) * np.float32(k))
    s = np.array([d800, np.nextafter(np.float32(d800), np.float32(9)), np.nextafter(np.float32(d800), np.float32(0)), 0.5, 0.5], np.float32)
    tr = {"n_req": 5, "prompt_len": l, "output_len": np.ones(5, np.int32), "srv_ttft": s,
          "dev_pre_spt": None, "dev_pre_spt_s": k, "dev_ttft_c": 0.0}
    r = oracle.dispatch(tr, [P(mode=0, l_th=101), P(mode=1, l_th=100, w_tail=0.5)])
    # server-constrained: strict l < l_th; a tie in the race goes to the server
    assert r["decision"][0].tolist() == [3, 7, 3, 6, 7]
    # device-constrained: l <= l_th waits 0; l = 101 waits 0.5 and the server token at exactly 0.5 s cancels the device
    assert r["decision"][1].tolist()[3:] == [7, 1]


def test_budget_accounting_and_cost_monotone(oracle, tr0):
    P = oracle.Policy
    levels = DI.budget_levels(16)
    total = int(tr0["prompt_len"].sum())
    lmax = int(tr0["prompt_len"].max())
    pols = []
    for num, den in levels:
        target = num * total / den
        l_th, _, _ = oracle.search_lth(tr0, P(mode=0), 0, lmax + 1, 20, "server_prefill_tok", DI.COST_S, target)
        pols.append(P(mode=0, l_th=l_th))
    r = oracle.dispatch(tr0, pols, materialise=False)
    for j, (num, den) in enumerate(levels):
        assert r["s_pre"][j] * den <= num * total          # server share of input tokens <= b
        assert r["d_pre"][j] == total                      # the device always starts
    assert pols[0].l_th == lmax + 1 and pols[-1].l_th == 0
    assert (np.diff(r["s_pre"]) >= 0).all() and (np.diff(r["s_dec"]) >= 0).all()
    assert (np.diff(r["d_dec"]) <= 0).all()
    tot = [oracle.total_cost(DI.COST_S, r["s_pre"][j], r["s_dec"][j], r["d_pre"][j], r["d_dec"][j]) for j in range(16)]
    assert (np.diff(tot) >= 0).all()
    # device-constrained sweep of the wait: device tokens and total cost fall as the wait grows
    waits = [0.0, 0.1, 0.2, 0.4, 0.8, 1.6, 3.2, math.inf]
    r = oracle.dispatch(tr0, [P(mode=1, l_th=-1, w_tail=w) for w in waits], materialise=False)
    assert (np.diff(r["d_pre"]) <= 0).all() and (np.diff(r["d_dec"]) <= 0).all()
    assert (np.diff(r["s_dec"]) >= 0).all() and (np.diff(r["s_pre"]) == 0).all()
    tot = [oracle.total_cost(DI.COST_D, r["s_pre"][j], r["s_dec"][j], r["d_pre"][j], r["d_dec"][j]) for j in range(len(waits))]
    assert (np.diff(tot) <= 0).all()


def test_cost_is_the_linear_model(oracle):
    c = {"cs_pre": 1.5e-6, "cs_dec": 6e-6, "e_pre": 1e-3, "e_dec": 3e-3, "lam": 0.01}
    got = oracle.total_cost(c, 1000, 200, 30, 4)
    want = Fraction(c["cs_pre"]) * 1000 + Fraction(c["cs_dec"]) * 200 + Fraction(c["lam"]) * (Fraction(c["e_pre"]) * 30 + Fraction(c["e_dec"]) * 4)
    assert abs(got - float(want)) <= 4e-16 * float(want)
    assert oracle.server_cost(c, 1, 0) == c["cs_pre"] and oracle.device_energy(c, 0, 1) == c["e_dec"]


def test_threshold_search_equals_sort_and_prefix_sum(oracle, tr0):
    P = oracle.Policy
    l = tr0["prompt_len"].astype(np.int64)
    total = int(l.sum())
    lmax = int(l.max())
    srt = np.sort(l)
    suffix = np.concatenate([np.cumsum(srt[::-1])[::-1], [0]])    # suffix[i] = sum of srt[i:]
    for num, den in [(0, 1), (1, 15), (1, 3), (1, 2), (7, 15), (14, 15), (1, 1)]:
        target = num * total / den
        got, hist_p, hist_a = oracle.search_lth(tr0, P(mode=0), 0, lmax + 1, 20, "server_prefill_tok", DI.COST_S, target)
        # smallest L with sum_{l >= L} l <= b * total, by sorting (Alg. 3's sorted accumulation)
        want = None
        for L in range(0, lmax + 2):
            a = int(suffix[np.searchsorted(srt, L, side="left")])
            if a * den <= num * total:
                want = L
                break
        assert got == want
        a_at = int(l[l >= got].sum())
        assert a_at * den <= num * total
        if got > 0:
            assert int(l[l >= got - 1].sum()) * den > num * total
        assert hist_a[-1] == a_at


def test_threshold_matches_the_lognormal_closed_form(oracle):
    # Eq. 3 for an unclipped log-normal: l_th = exp(mu + sigma^2 + sigma * Phi^-1(1 - b))
    g = dict(DI.config(0, n_req=200_000)["gen"])
    g["prompt_lo"], g["prompt_hi"] = 0, 2_000_000_0
    tr = oracle.gen_requests(g)
    l = tr["prompt_len"].astype(np.int64)
    total = int(l.sum())
    for b in (0.2, 0.5, 0.8):
        got, _, _ = oracle.search_lth(tr, oracle.Policy(mode=0), 0, int(l.max()) + 1, 32, "server_prefill_tok", DI.COST_S, b * total)
        want = math.exp(g["prompt_mu"] + g["prompt_sigma"] ** 2 + g["prompt_sigma"] * NormalDist().inv_cdf(1 - b))
        assert abs(got - want) / want < 0.03, (b, got, want)


def test_wait_search_brackets_the_exact_root(oracle):
    P = oracle.Policy
    tr = oracle.gen_trace(DI.config(3, n_req=3000)["gen"])
    cost = DI.COST_D
    c_all = cost["cs_pre"] * (int(tr["prompt_len"].sum()) + int(tr["output_len"].sum()))
    target = 0.30 * c_all
    w, hp, ha = oracle.search_wait(tr, P(mode=1, l_th=-1), 0.0, 5.0, 32, "device_cost", cost, target)

    def spend(wv):
        r = oracle.dispatch(tr, [P(mode=1, l_th=-1, w_tail=float(wv))], materialise=False)
        return cost["lam"] * oracle.device_energy(cost, r["d_pre"][0], r["d_dec"][0])
    # the bracket has shrunk to 5 * 2^-32 (or to adjacent floats) around a sign change of A - target
    assert spend(w) <= target
    lo = np.float32(hp[ha > target].max())
    assert spend(lo) > target
    assert 0 <= float(w) - float(lo) <= 5 * 2.0 ** -32 * 1.0001 + float(np.spacing(np.float32(w)))
    assert hp[0] == np.float32(2.5) and len(hp) == 32
    # brute force: the spend only changes at waits equal to a server TTFT or where w + d crosses it;
    # scan all fp32 candidates next to those breakpoints and take the smallest feasible one
    s = tr["srv_ttft"]
    d = (tr["prompt_len"].astype(np.float32) * np.float32(tr["dev_pre_spt"][0])).astype(np.float32)
    cands = np.unique(np.concatenate([s, (s - d).astype(np.float32)]))
    cands = cands[(cands >= 0) & (cands <= 5)]
    near = np.unique(np.concatenate([cands, np.nextafter(cands, np.float32(9)), np.nextafter(cands, np.float32(-9)),
                                     np.nextafter(np.nextafter(cands, np.float32(9)), np.float32(9))]))
    near = near[(near >= 0) & (near <= 5)]
    # monotone => binary search over the sorted candidates for the first feasible one
    a, b = 0, len(near) - 1
    assert spend(near[b]) <= target
    while a < b:
        mid = (a + b) // 2
        if spend(near[mid]) <= target:
            b = mid
        else:
            a = mid + 1
    root = near[a]
    # bisection converges onto the first feasible float up to its final bracket width
    assert abs(float(w) - float(root)) <= 5 * 2.0 ** -32 * 1.0001 + float(np.spacing(np.float32(w)))
    # the spend at the answer equals the spend at the exact root (no breakpoint in between)
    assert spend(w) == spend(root)


def test_slope_search_finds_the_root_of_eq2_on_the_trace(oracle):
    """Eq. 2: the slope beta of the ramp w(l) = min(beta l, w_tail) at which the device prefill of the prompts above
    l_th uses up the rest of the budget.  Its left-hand side is written out here on the trace (a request starts the
    device iff its own server TTFT exceeds its wait), without the oracle's dispatch."""
    P = oracle.Policy
    tr = oracle.gen_trace(DI.config(3, n_req=3000)["gen"])
    l = tr["prompt_len"].astype(np.int64)
    s = tr["srv_ttft"]
    l_th, w_tail, hi0 = 40, np.float32(2.0), 0.02
    lf = tr["prompt_len"].astype(np.float32)

    def device_prefill(beta):
        ramp = (np.float32(beta) * lf).astype(np.float32)
        w = np.where(ramp < w_tail, ramp, w_tail).astype(np.float32)
        w = np.where(l <= l_th, np.float32(0.0), w)
        return int(l[s > w].sum())
    at_zero, at_hi = device_prefill(0.0), device_prefill(hi0)
    assert at_hi < at_zero
    target = at_hi + 0.4 * (at_zero - at_hi)
    beta, hp, ha = oracle.search_slope(tr, P(mode=1, l_th=l_th, w_tail=float(w_tail), beta=0.0), 0.0, hi0, 32,
                                       "device_prefill_tok", DI.COST_D, target)
    assert hp[0] == np.float32(0.5 * hi0) and len(hp) == 32
    for b, a in zip(hp, ha):                       # every recorded accumulator is Eq. 2's left-hand side at that slope
        assert a == device_prefill(b), b
    assert device_prefill(beta) <= target
    lo = np.float32(hp[ha > target].max())
    assert device_prefill(lo) > target
    assert 0 <= float(beta) - float(lo) <= hi0 * 2.0 ** -32 * 1.0001 + float(np.spacing(np.float32(beta)))
    # brute force: the sum only changes where beta l crosses a server TTFT; the smallest feasible fp32 slope next to
    # those breakpoints is the exact root
    big = l > l_th
    cands = (s[big] / lf[big]).astype(np.float32)
    cands = cands[(cands >= 0) & (cands <= hi0)]
    near = np.unique(np.concatenate([cands] + [np.nextafter(cands, np.float32(d)) for d in (9, -9)]
                                    + [np.nextafter(np.nextafter(cands, np.float32(d)), np.float32(d)) for d in (9, -9)]))
    near = near[(near >= 0) & (near <= hi0)]
    a, b = 0, len(near) - 1
    assert device_prefill(near[b]) <= target
    while a < b:
        mid = (a + b) // 2
        if device_prefill(near[mid]) <= target:
            b = mid
        else:
            a = mid + 1
    root = near[a]
    assert abs(float(beta) - float(root)) <= hi0 * 2.0 ** -32 * 1.0001 + float(np.spacing(np.float32(beta)))
    assert device_prefill(beta) == device_prefill(root)


def test_quantile_is_sort_plus_nearest_rank(oracle):
    rng = np.random.default_rng(5)
    for M in (1, 2, 7, 100, 101, 9999):
        v = rng.lognormal(0, 1, M).astype(np.float32)
        for num, den in [(50, 100), (99, 100), (1, 100), (100, 100), (0, 100), (999, 1000)]:
            k, x = oracle.quantile(v, num, den)
            kk = min(max(math.ceil(Fraction(num, den) * M), 1), M)
            assert k == kk and x == np.sort(v)[kk - 1]
    # heavy ties
    v = np.full(5000, np.float32(0.2))
    v[:30] = 0.5
    assert oracle.quantile(v, 99, 100) == (4950, np.float32(0.2))
    assert oracle.quantile(v, 995, 1000) == (4975, np.float32(0.5))
    k, x = oracle.quantile(np.empty(0, np.float32), 1, 2)
    assert k == 0 and math.isnan(x)


def test_stats_assembly(oracle, tr0):
    P = oracle.Policy
    pols = [P(mode=0, l_th=300), P(mode=1, l_th=-1, w_tail=0.4)]
    st = oracle.stats(tr0, pols, DI.COST_S)
    dp = oracle.dispatch(tr0, pols)
    for j in range(2):
        col = dp["ttft"][j].astype(np.float64)
        assert abs(st[j]["mean_ttft"] - col.mean()) < 1e-12 * col.mean() * 10
        assert st[j]["ttft_q"][0] == np.sort(dp["ttft"][j])[math.ceil(0.5 * tr0["n_req"]) - 1]
        assert st[j]["ttft_q"][1] == np.sort(dp["ttft"][j])[math.ceil(0.99 * tr0["n_req"]) - 1]
        assert st[j]["total_cost"] == pytest.approx(st[j]["server_cost"] + DI.COST_S["lam"] * st[j]["device_energy"], rel=1e-15)


def test_policy_type_follows_alg1(oracle):
    """Alg. 1: device-constrained iff min(device prefill, decode cost) > max(server prefill, decode cost); the two
    exchange rates of the workloads put a device token at 0.3 and at 5 server tokens (App. E)."""
    import disco_inputs as DI
    assert oracle.policy_type(DI.COST_S) == 0 and oracle.policy_type(DI.COST_D) == 1
    base = {"cs_pre": 2.0, "cs_dec": 3.0, "e_pre": 1.0, "e_dec": 1.0, "lam": 1.0}
    # all four orderings of the cheaper device token against the dearer server token, and the boundary
    assert oracle.policy_type(dict(base, e_pre=4.0, e_dec=5.0)) == 1        # both device tokens dearer than both server tokens
    assert oracle.policy_type(dict(base, e_pre=2.5, e_dec=5.0)) == 0        # device prefill cheaper than server decode
    assert oracle.policy_type(dict(base, e_pre=5.0, e_dec=2.5)) == 0        # device decode cheaper than server decode
    assert oracle.policy_type(dict(base, e_pre=3.0, e_dec=3.0)) == 0        # equality is not "greater": server-constrained
    assert oracle.policy_type(dict(base, e_pre=3.0, e_dec=3.0, lam=1.0 + 1e-9)) == 1
    assert oracle.policy_type(dict(base, e_pre=4.0, e_dec=5.0, lam=0.5)) == 0     # the exchange rate scales the device side only
