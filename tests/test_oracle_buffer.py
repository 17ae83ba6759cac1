"""Pins of the oracle's buffer-based, cost-triggered migration (Sec. 4.3: the
source stops once the buffer can hide the hand-off and the decode cost saved
exceeds the target's prefill overhead).

None of these go through the oracle's own formulas: closed forms for constant
gaps worked out by hand, a sequential token-buffer simulation in exact
rational arithmetic (inputs are dyadic, so the oracle's fp32 arithmetic is
exact and must agree to the bit), and the breakpoints of the cost condition."""
from fractions import Fraction as F

import numpy as np
import pytest

TAU = 0.25


def brute_force(n, r_src, tgt_arrival, t_mig, dc, cp, l, tau):
    """Sequential buffer simulation in exact arithmetic.  delivered_t = max(arrival_t, delivered_{t-1} + tau);
    hand-off after the first token whose remaining playback time covers the migration time and whose
    remaining decode saving exceeds the prefill overhead.  Returns (m, delivered, delayed)."""
    tau = F(tau)
    m = None
    delivered = []
    delayed = 0
    base = None
    for t in range(n):
        r = F(r_src(t)) if m is None else base + F(tgt_arrival(t, m))
        d = r if t == 0 else max(r, delivered[-1] + tau)
        if m is not None and d - delivered[-1] > tau:
            delayed += 1
        delivered.append(d)
        if m is None and t + 1 < n:
            if d - r >= F(t_mig(t)) and F(dc) * (n - 1 - t) > F(cp) * (l + t + 1):
                m = t
                base = r + F(t_mig(t))
    return (-1 if m is None else m), delivered, delayed


@pytest.mark.parametrize("g_src,g_tgt,k,l,n", [
    (0.125, 0.0625, 2.0 ** -9, 64, 40),      # fast target: nobody waits
    (0.125, 0.375, 2.0 ** -9, 64, 60),       # target slower than the reader: late once the buffer has drained
    (0.0625, 0.3125, 2.0 ** -7, 200, 300),
    (0.1875, 0.25, 2.0 ** -8, 33, 25),       # target exactly at the pacing interval
])
def test_server_source_constant_gaps_match_exact_simulation(oracle, g_src, g_tgt, k, l, n):
    dc, cp = 3.0, 0.5
    m, dn, tl, deliv, tbt = oracle.timeline_buffer(n, None, g_src, False, dc, cp, 0.0, TAU, l, k, 0.0, g_tgt)
    bm, bd, bdel = brute_force(n, lambda t: F(g_src) * t, lambda t, mm: F(g_tgt) * (t - mm),
                               lambda t: F(k) * (l + t + 1), dc, cp, l, TAU)
    assert m == bm and m >= 0
    assert dn == bdel
    assert [F(float(x)) for x in deliv] == bd
    assert F(float(tl)) == bd[-1]


def test_hand_off_index_closed_form(oracle):
    # slack_t = t (tau - g) = t / 8 ; t_mig(t) = (65 + t) / 512 ; first t with 64 t >= 65 + t is t = 2
    m, dn, tl, deliv, tbt = oracle.timeline_buffer(50, None, 0.125, False, 1.0, 1e-3, 0.0, TAU, 64, 2.0 ** -9, 0.0, 0.0625)
    assert m == 2 and dn == 0
    assert (deliv == np.arange(50, dtype=np.float32) * np.float32(TAU)).all()       # the user never notices
    assert (tbt == np.float32(TAU)).all()


def test_delayed_tokens_closed_form(oracle):
    # hand-off at m with slack S = m / 8; token m + j is late iff j (g - tau) > S - t_mig(m)
    g_tgt, k, l, n = 0.375, 2.0 ** -9, 64, 80
    m, dn, tl, deliv, tbt = oracle.timeline_buffer(n, None, 0.125, False, 1.0, 1e-3, 0.0, TAU, l, k, 0.0, g_tgt)
    assert m == 2
    room = F(m, 8) - F(l + m + 1, 512)
    on_time = int(room / (F(g_tgt) - F(TAU)))          # j = 1 .. on_time are not late (j (g - tau) <= room)
    assert dn == (n - 1 - m) - on_time
    # paced until the buffer has drained, one transition gap, then the target's own gaps
    first_late = F(m, 8) + F(l + m + 1, 512) + (on_time + 1) * F(g_tgt) - (m + on_time) * F(TAU)   # r'_j - delta_{j-1}
    assert (tbt[:m + on_time] == np.float32(TAU)).all()
    assert F(float(tbt[m + on_time])) == first_late and F(TAU) < first_late <= F(g_tgt)
    assert (tbt[m + on_time + 1:] == np.float32(g_tgt)).all()


def test_device_source_hands_off_to_the_server(oracle):
    # device source (gap 1/16), server target with TTFT 1.5 s: slack_t = t (1/4 - 1/16) >= 3/2 first at t = 8
    n, l = 64, 100
    m, dn, tl, deliv, tbt = oracle.timeline_buffer(n, None, 0.125, True, 2.0, 1.0 / 64, 1.5, TAU, l, 2.0 ** -9, 0.0, 0.0625)
    assert m == 8
    bm, bd, bdel = brute_force(n, lambda t: F(1, 16) * t, lambda t, mm: F(1, 8) * (t - mm), lambda t: F(3, 2),
                               2.0, 1.0 / 64, l, TAU)
    assert bm == 8 and dn == bdel and [F(float(x)) for x in deliv] == bd


def test_device_source_with_a_server_token_trace(oracle):
    # the target's arrivals follow the server trace's own gaps after the hand-off
    rng = np.random.default_rng(3)
    n, l = 90, 40
    gaps = rng.integers(1, 12, n).astype(np.float32) / np.float32(64)
    r_srv = np.concatenate([[0], np.cumsum(gaps[1:], dtype=np.float32)]).astype(np.float32)
    m, dn, tl, deliv, tbt = oracle.timeline_buffer(n, r_srv, 0.0, True, 2.0, 1.0 / 64, 0.75, TAU, l, 2.0 ** -9, 0.0, 0.0625)
    bm, bd, bdel = brute_force(n, lambda t: F(1, 16) * t,
                               lambda t, mm: F(float(r_srv[t])) - F(float(r_srv[mm])), lambda t: F(3, 4),
                               2.0, 1.0 / 64, l, TAU)
    assert m == bm == 4 and dn == bdel and [F(float(x)) for x in deliv] == bd


@pytest.mark.parametrize("dc,cp,expect", [
    (0.0, 1.0, -1),          # nothing to save
    (-1.0, 0.0, -1),         # the target is dearer
    (1.0, 1.0, -1),          # saving (n-1-t) never exceeds the overhead (l+t+1) when l + 2 >= n - 1
    (1.0, 0.25, 2),          # cheap prefill: hand-off as soon as the buffer allows
])
def test_cost_condition(oracle, dc, cp, expect):
    n, l = 60, 64
    m, dn, tl, deliv, tbt = oracle.timeline_buffer(n, None, 0.125, False, dc, cp, 0.0, TAU, l, 2.0 ** -9, 0.0, 0.0625)
    assert m == expect
    if expect < 0:
        # identical to the timeline without any migration
        m0, tl0, deliv0, tbt0 = oracle.timeline(n, None, 0.125, False, False, TAU, 3.0, l, 2.0 ** -9, 0.0, 0.0625)
        assert m0 == -1 and (deliv == deliv0).all() and tl == tl0


def test_cost_condition_breakpoint(oracle):
    # the buffer allows the hand-off from t = 10 on (t_mig = 5/4 = 10 (tau - g)), the cost condition only while
    # dc (n-1-t) > cp (l+t+1)  <=>  t < (dc (n-1) - cp (l+1)) / (dc + cp): breakpoint moved across t = 10
    n, l, k = 200, 0, 0.0
    for cp, expect in ((1.0, 10), (17.0, 10), (18.0, -1), (50.0, -1)):
        # dc = 1: t < (199 - cp) / (1 + cp)  -> cp = 17: t < 10.11 ok at 10;  cp = 18: t < 9.53 not at 10
        m, *_ = oracle.timeline_buffer(n, None, 0.125, False, 1.0, cp, 0.0, TAU, l, k, 1.25, 0.0625)
        assert m == expect, (cp, m)


def test_accounting_and_first_target_token(oracle):
    """Per column: the source is charged m + 1 decode tokens, the target the rest and a re-prefill of the
    prompt plus the m + 1 tokens produced; mig_idx is the first token produced by the target."""
    import disco_inputs as DI
    tr = DI.handmade_trace(5, 400, tokens=True, max_out=120, stall_p=0.01)
    tr["prompt_len"] = (tr["prompt_len"] % 48 + 1).astype(np.int32)     # short prompts: re-prefilling them is cheap
    tr["dev_pre_spt"] = (tr["dev_pre_spt"] * np.float32(64)).astype(np.float32)   # slow prefill: the server wins many races
    cost = DI.COST_S       # device token = 0.3 server tokens: server-constrained columns save by handing off
    pol = [oracle.Policy(mode=0, l_th=0, mig_mode=2), oracle.Policy(mode=0, l_th=0, mig_mode=0),
           oracle.Policy(mode=1, l_th=-1, w_tail=0.0, mig_mode=2)]
    r = oracle.migration(tr, pol, 0.2, 3.0, cost=cost)
    d = oracle.dispatch(tr, pol)
    n = tr["output_len"].astype(np.int64)
    l = tr["prompt_len"].astype(np.int64)
    for j in range(3):
        src_dev = (d["decision"][j] & 4) != 0
        mig = r["mig_idx"][j] >= 0
        ns = r["n_src_tok"][j].astype(np.int64)
        assert (ns[mig] == r["mig_idx"][j][mig]).all() and (ns[~mig] == n[~mig]).all()
        assert r["m_s_dec"][j] == ns[~src_dev].sum() + (n - ns)[src_dev].sum()
        assert r["m_d_dec"][j] == ns[src_dev].sum() + (n - ns)[~src_dev].sum()
        assert r["m_d_repre"][j] == (l + ns)[mig & ~src_dev].sum()
        assert r["m_s_repre"][j] == (l + ns)[mig & src_dev].sum()
        assert r["delay_sum"][j] == r["delay_num"][j][mig].sum() and (r["delay_num"][j][~mig] == 0).all()
    assert (r["mig_idx"][1] == -1).all()
    # server-constrained column: only server-sourced requests hand off; with lam_S the device is cheaper
    src_dev0 = (d["decision"][0] & 4) != 0
    assert not (r["mig_idx"][0][src_dev0] >= 0).any() and (r["mig_idx"][0][~src_dev0] >= 0).sum() > 50
    # device-constrained column under a server-constrained price (device cheaper than server): never worth it
    assert (r["mig_idx"][2] == -1).all()
    # ... but it is under the device-constrained price
    r2 = oracle.migration(tr, [pol[2]], 0.2, 3.0, cost=DI.COST_D)
    src_dev2 = (d["decision"][2] & 4) != 0
    assert (r2["mig_idx"][0][src_dev2] >= 0).sum() > 20 and not (r2["mig_idx"][0][~src_dev2] >= 0).any()


def test_delay_num_order_statistics(oracle):
    """Mean and tail of the delayed tokens over the migrated requests (TBT table of Sec. 5.2), against numpy on the
    per-request counts, which the tests above pin."""
    import disco_inputs as DI
    tr = DI.handmade_trace(5, 400, tokens=True, max_out=120, stall_p=0.01)
    tr["prompt_len"] = (tr["prompt_len"] % 48 + 1).astype(np.int32)
    tr["dev_pre_spt"] = (tr["dev_pre_spt"] * np.float32(64)).astype(np.float32)
    tr["dev_dec_spt"] = (tr["dev_dec_spt"] * np.float32(6)).astype(np.float32)      # slow device: late tokens after a hand-off
    pol = [oracle.Policy(mode=0, l_th=0, mig_mode=2), oracle.Policy(mode=0, l_th=0, mig_mode=0)]
    st = oracle.stats(tr, pol, DI.COST_S, quantiles=((50, 100), (99, 100), (0, 1), (1, 1)), tau=0.2, kappa=3.0)
    r = oracle.migration(tr, pol, 0.2, 3.0, cost=DI.COST_S)
    d = np.sort(r["delay_num"][0][r["mig_idx"][0] >= 0])
    m = len(d)
    assert m > 50 and d[-1] > 0
    want = [d[max(-(-50 * m // 100), 1) - 1], d[max(-(-99 * m // 100), 1) - 1], d[0], d[-1]]
    assert [float(x) for x in st[0]["delay_q"]] == [float(x) for x in want]
    assert st[0]["delay_sum"] == int(d.sum())
    assert all(np.isnan(x) for x in st[1]["delay_q"])                 # no migration, no order statistic


# ---- delayed tokens at a pacing interval that is not a dyadic number (0.2 s: five tokens a second, Sec. 2.1) ----
# There two paced deliveries fma(t, tau, M) and fma(t-1, tau, M) differ by tau only up to an ulp, so "late" must
# be decided on the arrival (token arrives after its pacing slot), not on the rounded difference of deliveries.

TAU5 = float(np.float32(0.2))


def exact_late_count(n, r_src, tgt_arrival, t_mig, tau, m):
    """Exact replay with the hand-off index given: number of tokens after m that arrive after their slot, and the
    smallest distance |arrival - slot| met (to tell apart counts that hinge on a rounding)."""
    tau = F(tau)
    prev, late, margin = None, 0, None
    base = None
    for t in range(n):
        r = F(r_src(t)) if t <= m else base + F(tgt_arrival(t, m))
        d = r if t == 0 else max(r, prev + tau)
        if t > m:
            late += r > prev + tau
            gap = abs(r - (prev + tau))
            margin = gap if margin is None else min(margin, gap)
        if t == m:
            base = r + F(t_mig(t))
        prev = d
    return late, margin


@pytest.mark.parametrize("g_src,g_tgt,n", [(0.03, 0.025, 600), (0.05, 0.125, 900), (0.11, 0.19, 300)])
def test_no_token_is_late_behind_a_fast_target_at_tau_one_fifth(oracle, g_src, g_tgt, n):
    # the target is faster than the reader: the buffer never runs dry after the hand-off, although about half of
    # the paced gaps come out one ulp above tau
    m, dn, tl, deliv, tbt = oracle.timeline_buffer(n, None, g_src, False, 1.0, 1e-3, 0.0, TAU5, 64, 1.0 / 800, 0.0, g_tgt)
    assert m >= 0 and dn == 0
    assert (tbt > np.float32(TAU5)).sum() > 10               # the rounding scatter the count must not see
    assert np.abs(tbt.astype(np.float64) - TAU5).max() < 1e-4


@pytest.mark.parametrize("g_src,g_tgt,k,l,n", [(0.05, 0.3, 1.0 / 800, 64, 400), (0.03, 0.21, 1.0 / 512, 200, 800),
                                               (0.125, 0.22, 1.0 / 800, 17, 150), (0.02, 0.205, 1.0 / 800, 333, 500)])
def test_late_tokens_behind_a_slow_target_closed_form_at_tau_one_fifth(oracle, g_src, g_tgt, k, l, n):
    f = lambda x: F(float(np.float32(x)))
    tau, gs, gt, kk = f(TAU5), f(g_src), f(g_tgt), f(k)
    m, dn, tl, deliv, tbt = oracle.timeline_buffer(n, None, g_src, False, 1.0, 1e-3, 0.0, TAU5, l, float(np.float32(k)), 0.0,
                                                   g_tgt)
    # hand-off after the first token whose buffered playback t (tau - g_src) covers t_mig(t) = k (l + t + 1)
    want_m = next(t for t in range(n) if t * (tau - gs) >= kk * (l + t + 1))
    assert m == want_m
    # token m + j arrives at r_m + t_mig + j g_tgt, its slot is delta_m + j tau: late iff j (g_tgt - tau) > room
    room = m * (tau - gs) - kk * (l + m + 1)
    on_time = int(room / (gt - tau))
    assert min(room / (gt - tau) - on_time, on_time + 1 - room / (gt - tau)) > F(1, 1000)      # no rounding can move it
    assert dn == (n - 1 - m) - on_time and 0 < dn
    assert on_time >= 1 or g_tgt > 0.25


def test_late_tokens_on_a_server_token_trace_at_tau_one_fifth(oracle):
    # device source, server target whose arrivals follow a recorded trace with stalls: some tokens are late
    rng = np.random.default_rng(11)
    total = 0
    for case in range(150):
        n, l = int(rng.integers(60, 400)), int(rng.integers(8, 300))
        gaps = np.exp(rng.normal(-3.5, 0.6, n)).astype(np.float32)
        stall = rng.random(n) < 0.03
        gaps[stall] = rng.uniform(0.5, 2.0, int(stall.sum())).astype(np.float32)
        r_srv = np.concatenate([[0], np.cumsum(gaps[1:], dtype=np.float32)]).astype(np.float32)
        g_dev, s = float(np.float32(1.0 / rng.uniform(8, 40))), float(np.float32(rng.uniform(0.2, 1.5)))
        m, dn, tl, deliv, tbt = oracle.timeline_buffer(n, r_srv, 0.0, True, 2.0, 1.0 / 64, s, TAU5, l, 1.0 / 800, 0.0, g_dev)
        if m < 0:
            continue
        late, margin = exact_late_count(n, lambda t: F(float(np.float32(t) * np.float32(g_dev))),
                                        lambda t, mm: F(float(np.float32(r_srv[t] - r_srv[mm]))), lambda t: F(s), TAU5, m)
        if margin > F(1, 10000):                # far from every slot: fp32 rounding of the deliveries cannot change a verdict
            assert dn == late, case
            total += late
    assert total > 20
