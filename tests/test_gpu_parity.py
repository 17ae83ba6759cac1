"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.

Bars: decisions, token indices, token totals, selected ranks and every fp32
time that both sides obtain by the same sequence of IEEE operations are
compared bit for bit; fp64 sums and costs (whose summation order differs) to
1e-9 relative, far inside the 1e-5 the method's statement asks for."""
import math

import numpy as np
import pytest
import torch

import disco_inputs as DI

pytestmark = pytest.mark.gpu

REL = 1e-9


def both(B, O, specs):
    """Policy columns for both sides from one list of dicts."""
    return [B.Policy(**s) for s in specs], [O.Policy(**s) for s in specs]


def mixed_policies(lag=False):
    mg = 1 if lag else 0
    inf = math.inf
    return [
        dict(mode=0, l_th=0, mig_mode=mg),                       # race everything
        dict(mode=0, l_th=10 ** 9, mig_mode=mg),                 # device only
        dict(mode=0, l_th=240, mig_mode=mg),
        dict(mode=0, l_th=1500, mig_mode=0),
        dict(mode=1, l_th=-1, w_tail=inf, mig_mode=mg),          # server only
        dict(mode=1, l_th=-1, w_tail=0.0, mig_mode=mg),
        dict(mode=1, l_th=-1, w_tail=DI.f32(0.35), mig_mode=mg),
        dict(mode=1, l_th=200, l_mid=201, w_mid=DI.f32(0.1), w_tail=DI.f32(0.6), mig_mode=0),      # Alg. 2 step map
        dict(mode=1, l_th=100, beta=DI.f32(0.0005), w_tail=DI.f32(0.5), mig_mode=mg),              # Eq. 1 ramp
    ]


def assert_same_bits(a, b, what=""):
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    assert a.shape == b.shape, what
    if a.dtype.kind == "f":
        a, b = a.view(np.uint32), b.view(np.uint32)
    bad = np.flatnonzero(a.ravel() != b.ravel())
    assert bad.size == 0, f"{what}: {bad.size} mismatches, first at {bad[:5]}"


def close(a, b, rel=REL):
    return abs(a - b) <= rel * max(abs(a), abs(b), 1e-300)


# --------------------------------------------------------------- generator

@pytest.mark.parametrize("idx,n_req", [(0, 20_000), (2, 3_001), (3, 20_000), (4, 2_500)])
def test_gen_trace_is_bit_identical(B, oracle, idx, n_req):
    cfg = DI.config(idx, n_req=n_req, seed=idx + 3)
    print(f"gen parity config{idx} n_req={n_req}", flush=True)
    want = oracle.gen_trace(cfg["gen"])
    got = B.disco_gen_trace(cfg["gen"])
    torch.cuda.synchronize()
    for name in ("prompt_len", "output_len", "srv_ttft", "srv_tbt", "dev_pre_spt", "dev_dec_spt", "tok_off"):
        assert_same_bits(getattr(got, name).cpu().numpy(), want[name], name)
    if cfg["gen"]["tokens"]:
        assert got.n_tok == want["n_tok"]
        assert_same_bits(got.tok_arr.cpu().numpy(), want["tok_arr"], "tok_arr")


def test_gen_trace_empty(B):
    cfg = DI.config(2, n_req=1)
    g = dict(cfg["gen"], n_req=0)
    t = B.disco_gen_trace(g)
    assert t.n_tok == 0 and t.tok_off.cpu().tolist() == [0]


# ---------------------------------------------------------------- dispatch

def check_dispatch(B, O, tr, specs, materialise=True):
    bp, op = both(B, O, specs)
    P = len(specs)
    dt = B.upload_trace(tr)
    got = B.disco_eval_dispatch(dt, bp, materialise=materialise)
    want = O.dispatch(tr, op, materialise=materialise)
    acc = B.accum_to_host(got["acc"], P)
    for j in range(P):
        for f in ("s_pre", "s_dec", "d_pre", "d_dec", "n_dev_started", "n_dev_win"):
            assert int(acc[f][j]) == int(want[f][j]), (f, j)
        if tr["n_req"]:
            assert close(float(acc["ttft_sum"][j]), float(want["ttft_sum"][j])), j
    if materialise and tr["n_req"]:
        assert_same_bits(got["decision"].cpu().numpy(), want["decision"], "decision")
        assert_same_bits(got["ttft"].cpu().numpy(), want["ttft"], "ttft")
        t = want["ttft"].view(np.uint32)
        assert (acc["ttft_min_bits"] == t.min(axis=1)).all() and (acc["ttft_max_bits"] == t.max(axis=1)).all()
    return dt, acc


@pytest.mark.parametrize("n_req", [0, 1, 63, 64, 65, 1000, 10_007])
def test_dispatch_matches_oracle_on_handmade_traces(B, oracle, n_req):
    print(f"dispatch parity handmade n_req={n_req}", flush=True)
    tr = DI.handmade_trace(100 + n_req, n_req, tokens=False, ties=True, per_request_device=(n_req % 2 == 1))
    check_dispatch(B, oracle, tr, mixed_policies())


@pytest.mark.parametrize("P", [1, 2, 3, 5, 16, 33, 64])
def test_dispatch_column_counts(B, oracle, P):
    print(f"dispatch parity columns P={P}", flush=True)
    tr = oracle.gen_trace(DI.config(0, n_req=5_003, seed=P)["gen"])
    rng = np.random.default_rng(P)
    specs = []
    for j in range(P):
        if j % 2 == 0:
            specs.append(dict(mode=0, l_th=int(rng.integers(0, 3000))))
        else:
            specs.append(dict(mode=1, l_th=int(rng.integers(-1, 300)), w_tail=DI.f32(rng.uniform(0, 2))))
    check_dispatch(B, oracle, tr, specs)


# --------------------------------------------------------------- timelines

def check_migration(B, O, tr, specs, tau, kappa, delivered_col=0, cost=None, policies=None):
    """``policies``: a device-resident table holding the same columns as ``specs`` (else a host table is passed)."""
    bp, op = both(B, O, specs)
    P = len(specs)
    dt = B.upload_trace(tr)
    got = B.disco_eval_migration(dt, tau, kappa, policies if policies is not None else bp, materialise=True,
                                 delivered_col=delivered_col, cost=cost)
    want = O.migration(tr, op, tau, kappa, materialise=True, cost=cost)
    acc = B.accum_to_host(got["acc"], P)
    for j in range(P):
        for f in ("m_s_dec", "m_d_dec", "m_d_repre", "m_s_repre", "delay_sum", "n_migrated", "tbt_count"):
            assert int(acc[f][j]) == int(want[f][j]), (f, j)
        if tr["n_req"]:
            assert close(float(acc["tlast_sum"][j]), float(want["tlast_sum"][j])), j
    if tr["n_req"]:
        assert_same_bits(got["mig_idx"].cpu().numpy(), want["mig_idx"], "mig_idx")
        assert_same_bits(got["n_src_tok"].cpu().numpy(), want["n_src_tok"], "n_src_tok")
        assert_same_bits(got["t_last"].cpu().numpy(), want["t_last"], "t_last")
        assert_same_bits(got["delay_num"].cpu().numpy(), want["delay_num"], "delay_num")
    if delivered_col is not None:
        w1 = O.migration(tr, [op[delivered_col]], tau, kappa, materialise=False, tbt_col=0, want_delivered=True,
                         cost=cost)
        assert_same_bits(got["delivered"].cpu().numpy(), w1["delivered"], "delivered")
    return dt, acc, want


@pytest.mark.parametrize("n_req,max_out", [(0, 10), (1, 1), (1, 4096), (257, 300), (1500, 200)])
def test_migration_matches_oracle_on_token_traces(B, oracle, n_req, max_out):
    print(f"migration parity handmade n_req={n_req} max_out={max_out}", flush=True)
    tr = DI.handmade_trace(7 + n_req, n_req, tokens=True, max_out=max_out, stall_p=0.03, ties=True)
    if n_req == 1 and max_out == 4096:
        tr = DI.handmade_trace(8, 3, tokens=True, max_out=4096, stall_p=0.002)
        tr["output_len"][:] = [4096, 1, 129]
        tr = _rebuild_tokens(tr, 9)
    for col in (0, 6):
        _, acc, want = check_migration(B, oracle, tr, mixed_policies(lag=True), DI.TAU, DI.KAPPA_LAG, delivered_col=col)
    if n_req >= 257:
        assert want["n_migrated"].max() > 0


def _rebuild_tokens(tr, seed):
    rng = np.random.default_rng(seed)
    n = tr["output_len"]
    off = np.zeros(len(n) + 1, np.int64)
    np.cumsum(n, out=off[1:])
    gaps = rng.lognormal(-3.5, 0.6, int(off[-1])).astype(np.float32)
    gaps[rng.random(gaps.size) < 0.002] = np.float32(1.7)
    arr = np.empty(int(off[-1]), np.float32)
    for i in range(len(n)):
        a, b = int(off[i]), int(off[i + 1])
        arr[a] = 0
        arr[a + 1:b] = np.cumsum(gaps[a + 1:b], dtype=np.float32)
    tr = dict(tr, tok_off=off, tok_arr=arr, n_tok=int(off[-1]))
    return tr


def test_migration_constant_gap_server(B, oracle):
    # no per-token trace: the server's arrivals are t * srv_tbt (the per-request constant gap of workload 0)
    print("migration parity constant-gap", flush=True)
    tr = oracle.gen_trace(DI.config(0, n_req=2_001, seed=5)["gen"])
    tr["tok_arr"] = None
    check_migration(B, oracle, tr, mixed_policies(lag=True), DI.TAU, DI.KAPPA_LAG, delivered_col=2)


def test_migration_generated_tokens(B, oracle):
    print("migration parity config2-like", flush=True)
    cfg = DI.config(2, n_req=4_000, seed=11)
    tr = oracle.gen_trace(cfg["gen"])
    specs = [dict(mode=0, l_th=0, mig_mode=1), dict(mode=1, l_th=-1, w_tail=math.inf, mig_mode=1)]
    _, acc, want = check_migration(B, oracle, tr, specs, cfg["tau"], cfg["kappa"], delivered_col=1)
    assert want["n_migrated"][1] > 100


# -------------------------------------------------------------- statistics

def check_stats(B, O, tr, specs, cost, tau=None, kappa=3.0, quantiles=((50, 100), (99, 100)), ws_requests=None):
    bp, op = both(B, O, specs)
    P = len(specs)
    dt = B.upload_trace(tr)
    ws = B.workspace(tr["n_req"] if ws_requests is None else ws_requests, P)
    r = B.disco_eval_dispatch(dt, bp, ws=ws)
    if tau is not None:
        B.disco_eval_migration(dt, tau, kappa, bp, ws=ws, acc=r["acc"], cost=cost)
    want = O.stats(tr, op, cost, quantiles=quantiles, tau=tau, kappa=kappa)
    # with timelines: once from the summaries the evaluation's token walk left in the workspace, once walking again
    for reuse in ((True, False) if tau is not None else (False,)):
        out = B.disco_reduce_stats(dt, cost, bp, r["acc"], quantiles=quantiles, tau=tau, kappa=kappa, ws=ws, mig_cost=cost,
                                   reuse_walk=reuse)
        got = B.stats_to_host(out, P)
        compare_stats(got, want, tr, P, quantiles, tau)
    return got, want


def compare_stats(got, want, tr, P, quantiles, tau):
    for j in range(P):
        w, g = want[j], got[j]
        for f in ("s_pre", "s_dec", "d_pre", "d_dec", "n_dev_started", "n_dev_win", "n_migrated", "tbt_count", "n_req"):
            assert int(g[f]) == int(w[f]), (f, j)
        for f in ("server_cost", "device_energy", "device_cost", "total_cost"):
            assert close(float(g[f]), float(w[f]), 1e-12), (f, j)
        if tr["n_req"]:
            assert close(float(g["mean_ttft"]), w["mean_ttft"]), j
        for qi in range(len(quantiles)):
            assert int(g["ttft_rank"][qi]) == w["ttft_rank"][qi], (j, qi)
            if tr["n_req"]:
                assert np.float32(g["ttft_q"][qi]).view(np.uint32) == np.float32(w["ttft_q"][qi]).view(np.uint32), (j, qi, g["ttft_q"][qi], w["ttft_q"][qi])
            else:
                assert math.isnan(g["ttft_q"][qi])
            if tau is not None:
                assert int(g["tbt_rank"][qi]) == w["tbt_rank"][qi], (j, qi)
                if w["tbt_count"]:
                    assert np.float32(g["tbt_q"][qi]).view(np.uint32) == np.float32(w["tbt_q"][qi]).view(np.uint32), (j, qi, g["tbt_q"][qi], w["tbt_q"][qi])
                else:
                    assert math.isnan(g["tbt_q"][qi])
        if tau is not None and w["tbt_count"]:
            assert close(float(g["mean_tbt"]), w["mean_tbt"]), j
        if tau is not None:
            if w["n_migrated"]:
                assert close(float(g["mean_delay_num"]), w["delay_sum"] / w["n_migrated"], 1e-15), j
            else:
                assert math.isnan(g["mean_delay_num"]), j
            for qi in range(len(quantiles)):
                if w["n_migrated"]:
                    assert float(g["delay_q"][qi]) == float(w["delay_q"][qi]), (j, qi, g["delay_q"][qi], w["delay_q"][qi])
                else:
                    assert math.isnan(g["delay_q"][qi]), (j, qi)


@pytest.mark.parametrize("n_req", [0, 1, 100, 4_097])
def test_stats_dispatch_only(B, oracle, n_req):
    print(f"stats parity dispatch-only n_req={n_req}", flush=True)
    tr = DI.handmade_trace(31 + n_req, n_req, tokens=False, ties=True)
    check_stats(B, oracle, tr, mixed_policies(), DI.COST_S,
                quantiles=((50, 100), (99, 100), (0, 1), (1, 1)))


def test_stats_all_values_equal(B, oracle):
    print("stats parity ties", flush=True)
    tr = DI.handmade_trace(3, 500, tokens=False)
    tr["srv_ttft"][:] = np.float32(0.25)
    tr["prompt_len"][:] = 40
    tr["dev_pre_spt"] = None
    check_stats(B, oracle, tr, [dict(mode=1, l_th=-1, w_tail=math.inf), dict(mode=0, l_th=0)], DI.COST_D)


@pytest.mark.parametrize("n_req,max_out", [(1, 1), (40, 1), (300, 250), (1200, 120)])
def test_stats_with_timelines(B, oracle, n_req, max_out):
    print(f"stats parity timelines n_req={n_req} max_out={max_out}", flush=True)
    tr = DI.handmade_trace(51 + n_req, n_req, tokens=True, max_out=max_out, stall_p=0.03)
    specs = mixed_policies(lag=True)
    check_stats(B, oracle, tr, specs, DI.COST_S, tau=DI.TAU, kappa=DI.KAPPA_LAG)


def test_config0_end_to_end(B, oracle):
    """Workload 0 at full size: 10^4 requests x 16 budget levels, thresholds from the search, all statistics."""
    print("config0 end to end", flush=True)
    cfg = DI.config(0)
    tr = oracle.gen_trace(cfg["gen"])
    dt = B.disco_gen_trace(cfg["gen"])
    levels = DI.budget_levels(cfg["levels"])
    total = int(tr["prompt_len"].astype(np.int64).sum())
    lmax = int(tr["prompt_len"].max())
    templ = [B.Policy(mode=0, mig_mode=1) for _ in levels]
    specs = [dict(which_param=B.PARAM_L_TH, which_acc="server_prefill_tok", n_steps=14, lo=0, hi=lmax + 1,
                  target=num * total / den) for num, den in levels]
    res = B.disco_budget_search(dt, cfg["cost"], templ, specs)
    found = B.policies_to_host(res["pol_out"], len(levels))
    so = B.search_to_host(res["out"], len(levels))
    for j, (num, den) in enumerate(levels):
        l_th, hp, ha = oracle.search_lth(tr, oracle.Policy(mode=0), 0, lmax + 1, 14, "server_prefill_tok",
                                         cfg["cost"], num * total / den)
        assert found[j].l_th == l_th == int(so["param"][j])
        assert (so["hist_param"][j][:14] == hp).all() and (so["hist_acc"][j][:14] == ha).all()
    pol_specs = [dict(mode=0, l_th=p.l_th, mig_mode=1) for p in found]
    tr_host = dict(tr, tok_arr=None)
    got, want = check_stats(B, oracle, tr_host, pol_specs, cfg["cost"], tau=cfg["tau"], kappa=cfg["kappa"])
    assert want[0]["s_pre"] == 0 and want[-1]["s_pre"] == total


def test_config0_device_constrained_sweep(B, oracle):
    """Workload 0 with its 16 budget levels read as device-constrained columns: one global wait per level, bisected
    so that the device's share of the prompt tokens meets b_j (Sec. 4.2), then every statistic incl. timelines."""
    print("config0 device-constrained sweep", flush=True)
    cfg = DI.config(0)
    tr = oracle.gen_trace(cfg["gen"])
    dt = B.disco_gen_trace(cfg["gen"])
    levels = DI.budget_levels(cfg["levels"])
    total = int(tr["prompt_len"].astype(np.int64).sum())
    templ = [B.Policy(mode=1, l_th=-1, mig_mode=1) for _ in levels]
    specs = [dict(which_param=B.PARAM_W_TAIL, which_acc="device_prefill_tok", n_steps=24, lo=0.0, hi=128.0,
                  target=num * total / den) for num, den in levels]
    res = B.disco_budget_search(dt, DI.COST_D, templ, specs)
    so = B.search_to_host(res["out"], len(levels))
    found = B.policies_to_host(res["pol_out"], len(levels))
    waits = []
    for j, (num, den) in enumerate(levels):
        w, hp, ha = oracle.search_wait(tr, oracle.Policy(mode=1, l_th=-1), 0.0, 128.0, 24, "device_prefill_tok", DI.COST_D,
                                       num * total / den)
        assert np.float32(so["param"][j]) == w == np.float32(found[j].w_tail), j
        assert (so["hist_param"][j][:24].astype(np.float32) == hp).all() and (so["hist_acc"][j][:24] == ha).all(), j
        waits.append(float(w))
    if levels[0][0] == 0:                                                    # no budget: wait out every server, and no longer
        assert abs(waits[0] - float(tr["srv_ttft"].max())) <= 128.0 / 2 ** 20
    assert all(a >= b for a, b in zip(waits, waits[1:])) and waits[-1] < 1e-4    # full budget: start (almost) at once
    pol_specs = [dict(mode=1, l_th=-1, w_tail=w, mig_mode=1) for w in waits]
    tr_host = dict(tr, tok_arr=None)
    got, want = check_stats(B, oracle, tr_host, pol_specs, DI.COST_D, tau=cfg["tau"], kappa=cfg["kappa"])
    assert all(want[j]["d_pre"] <= num * total / den for j, (num, den) in enumerate(levels))
    assert oracle.policy_type(DI.COST_D) == 1


# ----------------------------------------------------------- budget search

def test_wait_search_history_is_bit_identical(B, oracle):
    print("search parity wait", flush=True)
    cfg = DI.config(3, n_req=50_003)
    tr = oracle.gen_trace(cfg["gen"])
    dt = B.upload_trace(tr)
    cost = cfg["cost"]
    c_all = cost["cs_pre"] * (int(tr["prompt_len"].astype(np.int64).sum()) + int(tr["output_len"].astype(np.int64).sum()))
    cases = [("device_cost", 0.30 * c_all), ("device_prefill_tok", 0.2 * int(tr["prompt_len"].astype(np.int64).sum())),
             ("total_cost", 1.30 * c_all)]
    templ = [B.Policy(mode=1, l_th=-1) for _ in cases]
    specs = [dict(which_param=B.PARAM_W_TAIL, which_acc=a, n_steps=32, lo=0.0, hi=5.0, target=t) for a, t in cases]
    res = B.disco_budget_search(dt, cost, templ, specs)
    so = B.search_to_host(res["out"], len(cases))
    pol = B.policies_to_host(res["pol_out"], len(cases))
    for j, (a, t) in enumerate(cases):
        w, hp, ha = oracle.search_wait(tr, oracle.Policy(mode=1, l_th=-1), 0.0, 5.0, 32, a, cost, t)
        assert np.float32(so["param"][j]) == w == np.float32(pol[j].w_tail), (a, so["param"][j], w)
        assert (so["hist_param"][j][:32].astype(np.float32) == hp).all(), a
        assert (so["hist_acc"][j][:32] == ha).all(), a
        d = oracle.dispatch(tr, [oracle.Policy(mode=1, l_th=-1, w_tail=float(w))], materialise=False)
        at = so["at_param"][j]
        assert int(at["d_pre"]) == int(d["d_pre"][0]) and int(at["d_dec"]) == int(d["d_dec"][0])
        assert int(at["s_dec"]) == int(d["s_dec"][0])


def test_single_search_single_step(B, oracle):
    print("search parity single", flush=True)
    tr = DI.handmade_trace(77, 999, tokens=False)
    dt = B.upload_trace(tr)
    res = B.disco_budget_search(dt, DI.COST_D, [B.Policy(mode=1, l_th=50)],
                                [dict(which_param=B.PARAM_W_TAIL, which_acc="device_prefill_tok", n_steps=1, lo=0.0,
                                      hi=1.0, target=1e5)])
    so = B.search_to_host(res["out"], 1)
    w, hp, ha = oracle.search_wait(tr, oracle.Policy(mode=1, l_th=50), 0.0, 1.0, 1, "device_prefill_tok", DI.COST_D, 1e5)
    assert np.float32(so["param"][0]) == w and so["hist_acc"][0][0] == ha[0]


def test_device_resident_policy_table(B, oracle):
    """search -> dispatch -> statistics with the found columns never leaving the device."""
    print("device policy table", flush=True)
    cfg = DI.config(1, n_req=30_011, seed=2)
    tr = oracle.gen_trace(cfg["gen"])
    dt = B.disco_gen_trace(cfg["gen"])
    levels = DI.budget_levels(8)
    total = int(tr["prompt_len"].astype(np.int64).sum())
    lmax = int(tr["prompt_len"].max())
    specs = [dict(which_param=B.PARAM_L_TH, which_acc="server_prefill_tok", n_steps=13, lo=0, hi=lmax + 1,
                  target=num * total / den) for num, den in levels]
    res = B.disco_budget_search(dt, cfg["cost"], [B.Policy(mode=0) for _ in levels], specs)
    r = B.disco_eval_dispatch(dt, res["policies"])
    got = B.stats_to_host(B.disco_reduce_stats(dt, cfg["cost"], res["policies"], r["acc"]), len(levels))
    opol = [oracle.Policy(mode=0, l_th=oracle.search_lth(tr, oracle.Policy(mode=0), 0, lmax + 1, 13, "server_prefill_tok",
                                                        cfg["cost"], num * total / den)[0]) for num, den in levels]
    want = oracle.stats(tr, opol, cfg["cost"])
    for j, w in enumerate(want):
        assert int(got[j]["s_pre"]) == w["s_pre"] and int(got[j]["d_dec"]) == w["d_dec"]
        for qi in range(2):
            assert int(got[j]["ttft_rank"][qi]) == w["ttft_rank"][qi]
            assert np.float32(got[j]["ttft_q"][qi]) == np.float32(w["ttft_q"][qi])


def test_stats_timelines_many_column_sets(B, oracle):
    """Tables whose winner sets are not nested: more distinct column sets than the class table holds
    (per-column histograms), and a few sets with several distinct prefixes."""
    print("stats parity irregular column sets", flush=True)
    rng = np.random.default_rng(5)
    tr = DI.handmade_trace(91, 900, tokens=True, max_out=150, stall_p=0.04)
    specs = []
    for j in range(12):
        if j % 3 == 0:
            specs.append(dict(mode=0, l_th=int(rng.integers(0, 3000)), mig_mode=int(rng.integers(0, 2))))
        elif j % 3 == 1:
            specs.append(dict(mode=1, l_th=int(rng.integers(-1, 2000)), w_tail=DI.f32(rng.uniform(0, 1.5)),
                              mig_mode=int(rng.integers(0, 2))))
        else:
            specs.append(dict(mode=1, l_th=-1, beta=DI.f32(rng.uniform(1e-4, 2e-3)), w_tail=DI.f32(rng.uniform(0.2, 2.0)),
                              mig_mode=1))
    check_stats(B, oracle, tr, specs, DI.COST_S, tau=DI.TAU, kappa=DI.KAPPA_LAG,
                quantiles=((50, 100), (99, 100), (1, 100), (999, 1000)))
    # slow devices (gap above the pacing interval): the device timeline needs the scan as well
    tr2 = DI.handmade_trace(92, 400, tokens=True, max_out=300, stall_p=0.03)
    tr2["dev_dec_spt"] = (tr2["dev_dec_spt"] * np.float32(2.5)).astype(np.float32)
    check_stats(B, oracle, tr2, mixed_policies(lag=True), DI.COST_S, tau=DI.TAU, kappa=DI.KAPPA_LAG)


def test_stats_timelines_more_classes_than_counted_in_lds(B, oracle):
    """24 length-threshold columns with alternating hand-off kinds: up to 50 nested column sets, i.e. more classes
    than the selection counts per workgroup in LDS (the rest is counted in device memory), most of them analytic."""
    print("stats parity timelines 24 threshold columns", flush=True)
    tr = DI.handmade_trace(77, 3000, tokens=True, max_out=200, stall_p=0.004)
    lths = np.unique(np.quantile(tr["prompt_len"], np.linspace(0.02, 0.98, 24)).astype(np.int64))
    specs = [dict(mode=0, l_th=int(l), mig_mode=j % 2) for j, l in enumerate(lths)]
    assert len(specs) > 16
    check_stats(B, oracle, tr, specs, DI.COST_S, tau=DI.TAU, kappa=DI.KAPPA_LAG)


def test_stats_timelines_under_shrunk_grids(B, oracle):
    """The same statistics with every grid shrunk (testing aid of the library): few workgroups take many rounds each,
    and the selection counts its analytic timelines in device memory instead of LDS."""
    print("stats parity timelines, grids / 16", flush=True)
    tr = DI.handmade_trace(78, 5000, tokens=True, max_out=160, stall_p=0.01)
    try:
        assert B._lib.disco_set_grid_divisor(16) == 0
        check_stats(B, oracle, tr, mixed_policies(lag=True), DI.COST_S, tau=DI.TAU, kappa=DI.KAPPA_LAG)
    finally:
        assert B._lib.disco_set_grid_divisor(1) == 0


@pytest.mark.parametrize("hi_extra,which", [(1, "server_prefill_tok"), (60_000, "server_prefill_tok"),
                                            (1, "device_prefill_tok"), (1, "total_cost")])
def test_threshold_search_paths(B, oracle, hi_extra, which):
    """Length-threshold searches through the tabulated path (brackets inside the length table, prompt-token
    accumulators) and through the generic passes (bracket beyond the table, cost accumulator): same history."""
    print(f"search parity thresholds hi_extra={hi_extra} acc={which}", flush=True)
    tr = DI.handmade_trace(123, 6_001, tokens=False)
    dt = B.upload_trace(tr)
    total = int(tr["prompt_len"].astype(np.int64).sum())
    lmax = int(tr["prompt_len"].max())
    hi = lmax + hi_extra
    steps = max(1, hi.bit_length())
    fracs = [0.0, 0.13, 0.5, 0.77, 1.0]
    if which == "total_cost":
        c_all = DI.COST_S["cs_pre"] * (total + int(tr["output_len"].astype(np.int64).sum()))
        targets = [f * c_all for f in fracs]
    else:
        targets = [f * total for f in fracs]
    specs = [dict(which_param=B.PARAM_L_TH, which_acc=which, n_steps=steps, lo=0, hi=hi, target=t) for t in targets]
    res = B.disco_budget_search(dt, DI.COST_S, [B.Policy(mode=0) for _ in targets], specs)
    so = B.search_to_host(res["out"], len(targets))
    pol = B.policies_to_host(res["pol_out"], len(targets))
    for j, t in enumerate(targets):
        l_th, hp, ha = oracle.search_lth(tr, oracle.Policy(mode=0), 0, hi, steps, which, DI.COST_S, t)
        assert pol[j].l_th == l_th == int(so["param"][j]), (j, pol[j].l_th, l_th)
        assert (so["hist_param"][j][:steps] == hp).all(), j
        if which == "total_cost":
            assert np.allclose(so["hist_acc"][j][:steps], ha, rtol=1e-12, atol=0), j
        else:
            assert (so["hist_acc"][j][:steps] == ha).all(), j
        d = oracle.dispatch(tr, [oracle.Policy(mode=0, l_th=l_th)], materialise=False)
        at = so["at_param"][j]
        for f in ("s_pre", "s_dec", "d_pre", "d_dec", "n_dev_win"):
            assert int(at[f]) == int(d[f][0]), (f, j)


def test_threshold_search_device_constrained_template(B, oracle):
    """A length threshold searched on a device-constrained template (Eq. 1: no wait up to l_th) takes the generic passes."""
    print("search parity threshold on a wait-time template", flush=True)
    tr = DI.handmade_trace(124, 3_000, tokens=False)
    dt = B.upload_trace(tr)
    total = int(tr["prompt_len"].astype(np.int64).sum())
    lmax = int(tr["prompt_len"].max())
    steps = (lmax + 1).bit_length()
    templ = dict(mode=1, w_tail=DI.f32(0.4))
    res = B.disco_budget_search(dt, DI.COST_D, [B.Policy(**templ)],
                                [dict(which_param=B.PARAM_L_TH, which_acc="device_prefill_tok", n_steps=steps, lo=0,
                                      hi=lmax + 1, target=0.6 * total)])
    so = B.search_to_host(res["out"], 1)
    l_th, hp, ha = oracle.search_lth(tr, oracle.Policy(**templ), 0, lmax + 1, steps, "device_prefill_tok", DI.COST_D,
                                     0.6 * total)
    assert int(so["param"][0]) == l_th
    assert (so["hist_param"][0][:steps] == hp).all() and (so["hist_acc"][0][:steps] == ha).all()


@pytest.mark.parametrize("kappa,tau", [(3.0, 0.2), (0.0, 0.2), (1e-4, 0.2), (3.0, 0.05), (8.0, 0.02), (40.0, 0.01)])
def test_migration_late_handoffs(B, oracle, kappa, tau):
    """A server whose gaps hover around the pacing interval keeps the buffer near empty, so stalls trigger the
    hand-off deep inside long requests (chunks after the first), also for degenerate trigger thresholds."""
    print(f"migration parity late hand-offs kappa={kappa} tau={tau}", flush=True)
    rng = np.random.default_rng(17)
    tr = DI.handmade_trace(200, 700, tokens=True, max_out=1500, stall_p=0.0)
    n = tr["output_len"]
    off = tr["tok_off"]
    gaps = rng.lognormal(math.log(tau) + 0.05, 0.5, int(off[-1])).astype(np.float32)
    stall = rng.random(gaps.size) < 0.002
    gaps[stall] = rng.uniform(2.0 * tau, 12.0 * tau, int(stall.sum())).astype(np.float32)
    arr = np.empty(int(off[-1]), np.float32)
    for i in range(len(n)):
        a, b = int(off[i]), int(off[i + 1])
        arr[a] = 0
        arr[a + 1:b] = np.cumsum(gaps[a + 1:b], dtype=np.float32)
    tr = dict(tr, tok_arr=arr)
    specs = [dict(mode=1, l_th=-1, w_tail=math.inf, mig_mode=1), dict(mode=0, l_th=0, mig_mode=1),
             dict(mode=1, l_th=-1, w_tail=math.inf, mig_mode=0)]
    _, acc, want = check_migration(B, oracle, tr, specs, tau, kappa, delivered_col=0)
    m = want["mig_idx"][0]
    if kappa >= 1.0 and tau >= 0.05:
        assert (m >= 256).sum() > 10 and (m >= 512).sum() > 3, ((m >= 256).sum(), (m >= 512).sum())
    check_stats(B, oracle, tr, specs, DI.COST_S, tau=tau, kappa=kappa)


@pytest.mark.parametrize("kind", ["thresholds", "mixed"])
def test_stats_heavy_ties_keep_the_histogram_passes(B, oracle, kind):
    """Most TTFTs are one and the same value while a few outliers keep the key range wide: the values that still
    match a slot after two radix passes are too many for the candidate list (its bound adds up over 128 slots),
    so the selection has to go on with histogram passes."""
    print(f"stats parity heavy ties {kind}", flush=True)
    rng = np.random.default_rng(23)
    n = 60_000                   # 64 median slots x 0.9 n tied values: 3.4 M against a list of 2 M entries
    tr = DI.handmade_trace(61, n, tokens=False)
    tr["srv_ttft"] = np.where(rng.random(n) < 0.9, np.float32(0.5), tr["srv_ttft"]).astype(np.float32)
    tr["dev_pre_spt"] = (tr["dev_pre_spt"] * np.float32(50)).astype(np.float32)       # the server wins nearly every race
    if kind == "thresholds":
        specs = [dict(mode=0, l_th=int(t)) for t in np.linspace(0, 400, 64)]
    else:
        specs = [dict(mode=0, l_th=int(t)) for t in np.linspace(0, 400, 32)] + \
                [dict(mode=1, l_th=-1, w_tail=DI.f32(w)) for w in np.linspace(0.6, 3.0, 32)]
    got, want = check_stats(B, oracle, tr, specs, DI.COST_S)
    assert sum(1 for w in want if np.float32(w["ttft_q"][0]) == np.float32(0.5)) > 32


@pytest.mark.parametrize("kind", ["band", "ties"])
def test_stats_threshold_table_too_large_for_buckets(B, oracle, kind):
    """Threshold table (selection by classes) on 2.3 M requests whose server TTFTs nearly all carry one first radix
    digit: the values with the digits of the wanted order statistics outnumber the candidate list (2^21 entries),
    so the second pass is a histogram pass again.  'band': the values spread over the second digit and the list
    takes over after that pass; 'ties': one value dominates and the histogram passes go on to the end."""
    print(f"stats parity threshold table beyond the bucket capacity: {kind}", flush=True)
    rng = np.random.default_rng(29)
    n = 2_300_000
    tr = DI.handmade_trace(67, n, tokens=False)
    common = rng.random(n) < 0.96
    if kind == "band":
        near = (np.uint32(0x3F000000) + rng.integers(0, 1 << 17, n).astype(np.uint32)).view(np.float32)   # 2^17 bit patterns in a row from 0.5
    else:
        near = np.full(n, 0.5, np.float32)
    tr["srv_ttft"] = np.where(common, near, tr["srv_ttft"]).astype(np.float32)
    tr["dev_pre_spt"] = (tr["dev_pre_spt"] * np.float32(50)).astype(np.float32)       # the server wins nearly every race
    specs = [dict(mode=0, l_th=int(t)) for t in np.linspace(0, 400, 8)]
    got, want = check_stats(B, oracle, tr, specs, DI.COST_S)
    assert sum(1 for w in want if 0.5 <= float(w["ttft_q"][0]) < 0.53) >= 6


def test_stats_threshold_table_smallest_workspace(B, oracle):
    """A workspace without the byte per request: the later passes of the selection by classes look the first racing
    column of a request up again instead of reading it back."""
    print("stats parity threshold table, workspace for zero requests", flush=True)
    tr = DI.handmade_trace(71, 50_000, tokens=False)
    specs = [dict(mode=0, l_th=int(t)) for t in np.linspace(0, 3100, 24)]
    check_stats(B, oracle, tr, specs, DI.COST_S, ws_requests=0, quantiles=((50, 100), (99, 100), (999, 1000)))


def test_stats_threshold_table_buckets_in_two_rounds(B, oracle):
    """1.5 M requests: a workgroup of the scatter pass takes its requests in two rounds, each with its own share
    of the buckets."""
    print("stats parity threshold table, 1.5 M requests", flush=True)
    tr = DI.handmade_trace(73, 1_500_000, tokens=False)
    specs = [dict(mode=0, l_th=int(t)) for t in np.linspace(0, 3100, 8)]
    check_stats(B, oracle, tr, specs, DI.COST_S)


@pytest.mark.parametrize("n_search,n_steps", [(9, 7), (10, 5), (21, 32), (22, 3), (64, 4)])
def test_wait_searches_side_by_side(B, oracle, n_search, n_steps):
    """Many wait-time searches in one call: the number of searches decides how many levels of the bisection a pass
    evaluates (three for up to 9 searches, two for up to 21, else one) and the steps need not fill the last pass;
    the recorded history is that of the plain bisection for every one of them."""
    print(f"search parity {n_search} searches x {n_steps} steps", flush=True)
    tr = DI.handmade_trace(79, 20_011, tokens=False)
    dt = B.upload_trace(tr)
    total = int(tr["prompt_len"].astype(np.int64).sum())
    targets = [total * (j + 1) / (n_search + 2) for j in range(n_search)]
    templ = [B.Policy(mode=1, l_th=(j % 5) * 100 - 1) for j in range(n_search)]
    specs = [dict(which_param=B.PARAM_W_TAIL, which_acc="device_prefill_tok", n_steps=n_steps, lo=0.0, hi=4.0, target=t)
             for t in targets]
    res = B.disco_budget_search(dt, DI.COST_D, templ, specs)
    so = B.search_to_host(res["out"], n_search)
    pol = B.policies_to_host(res["pol_out"], n_search)
    for j in range(n_search):
        op = oracle.Policy(mode=1, l_th=(j % 5) * 100 - 1)
        w, hp, ha = oracle.search_wait(tr, op, 0.0, 4.0, n_steps, "device_prefill_tok", DI.COST_D, targets[j])
        assert np.float32(so["param"][j]) == w == np.float32(pol[j].w_tail), (j, so["param"][j], w)
        assert (so["hist_param"][j][:n_steps].astype(np.float32) == hp).all(), j
        assert (so["hist_acc"][j][:n_steps] == ha).all(), j
        assert pol[j].l_th == (j % 5) * 100 - 1


def test_slope_search_history_is_bit_identical(B, oracle):
    """Bisection on the ramp slope beta (Eq. 2 on the trace), next to wait and threshold searches in one call."""
    print("search parity ramp slope", flush=True)
    tr = oracle.gen_trace(DI.config(3, n_req=30_011)["gen"])
    dt = B.upload_trace(tr)
    total = int(tr["prompt_len"].astype(np.int64).sum())
    lmax = int(tr["prompt_len"].max())
    templ = [B.Policy(mode=1, l_th=40, w_tail=2.0, beta=0.0), B.Policy(mode=1, l_th=-1, w_tail=1.0, beta=0.0),
             B.Policy(mode=1, l_th=-1), B.Policy(mode=0)]
    specs = [dict(which_param=B.PARAM_BETA, which_acc="device_prefill_tok", n_steps=20, lo=0.0, hi=0.02, target=0.55 * total),
             dict(which_param=B.PARAM_BETA, which_acc="device_cost", n_steps=20, lo=0.0, hi=0.05, target=0.2 * DI.COST_D["lam"] * DI.COST_D["e_pre"] * total),
             dict(which_param=B.PARAM_W_TAIL, which_acc="device_prefill_tok", n_steps=20, lo=0.0, hi=5.0, target=0.3 * total),
             dict(which_param=B.PARAM_L_TH, which_acc="server_prefill_tok", n_steps=20, lo=0, hi=lmax + 1, target=0.5 * total)]
    res = B.disco_budget_search(dt, DI.COST_D, templ, specs)
    so = B.search_to_host(res["out"], 4)
    pol = B.policies_to_host(res["pol_out"], 4)
    for j in (0, 1):
        op = oracle.Policy(mode=1, l_th=templ[j].l_th, w_tail=templ[j].w_tail, beta=0.0)
        b, hp, ha = oracle.search_slope(tr, op, specs[j]["lo"], specs[j]["hi"], 20, specs[j]["which_acc"], DI.COST_D,
                                        specs[j]["target"])
        assert np.float32(so["param"][j]) == b == np.float32(pol[j].beta), (j, so["param"][j], b)
        assert (so["hist_param"][j][:20].astype(np.float32) == hp).all(), j
        assert (so["hist_acc"][j][:20] == ha).all(), j
        assert len(set(ha)) > 3                    # the slope really moves the accumulator
    w, hp, ha = oracle.search_wait(tr, oracle.Policy(mode=1, l_th=-1), 0.0, 5.0, 20, "device_prefill_tok", DI.COST_D, 0.3 * total)
    assert np.float32(so["param"][2]) == w and (so["hist_acc"][2][:20] == ha).all()
    lth, hp, ha = oracle.search_lth(tr, oracle.Policy(mode=0), 0, lmax + 1, 20, "server_prefill_tok", DI.COST_D, 0.5 * total)
    assert int(so["param"][3]) == lth == pol[3].l_th and (so["hist_acc"][3][:20] == ha).all()


def test_step_replayed_from_a_hip_graph(B, oracle):
    """The entry points only enqueue kernels on the caller's stream (no memset or copy nodes, no synchronisation), so a
    search + statistics step can be captured into a HIP graph: every replay, with eager steps in between, gives what
    the eager step gives."""
    print("graph replay of a search + statistics step", flush=True)
    cfg = DI.config(1, n_req=60_000)
    tr = oracle.gen_trace(cfg["gen"])
    dt = B.upload_trace(tr)
    P = 16
    total = int(tr["prompt_len"].astype(np.int64).sum())
    lmax = int(tr["prompt_len"].max())
    templ = B.prepare_policies([B.Policy(mode=B.MODE_S) for _ in range(P)])
    specs = B.prepare_specs([dict(which_param=B.PARAM_L_TH, which_acc="server_prefill_tok", n_steps=13, lo=0, hi=lmax + 1,
                                  target=j * total / (P - 1)) for j in range(P)])
    ws = B.workspace(tr["n_req"], P)
    acc = torch.zeros(P * 128, dtype=torch.uint8, device="cuda")
    sout = torch.zeros(P * B.SEARCH_DTYPE.itemsize, dtype=torch.uint8, device="cuda")
    pol_out = torch.zeros(P * 32, dtype=torch.uint8, device="cuda")
    stats = torch.zeros(P * 256, dtype=torch.uint8, device="cuda")

    def step():
        res = B.disco_budget_search(dt, cfg["cost"], templ, specs, ws=ws, out=sout, pol_out=pol_out, acc=acc)
        B.disco_reduce_stats(dt, cfg["cost"], res["policies"], acc, ws=ws, out=stats)

    step()
    torch.cuda.synchronize()
    want = B.stats_to_host(stats, P).copy()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                        # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for _ in range(3):
        stats.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = B.stats_to_host(stats, P)
        for f in want.dtype.names:
            if want[f].dtype.kind in "iu":
                assert (got[f] == want[f]).all(), f
            else:
                assert np.allclose(got[f], want[f], rtol=1e-9, atol=0, equal_nan=True), f
        assert (got["ttft_q"].view(np.uint32) == want["ttft_q"].view(np.uint32)).all()
        step()                                        # eager work between the replays
        torch.cuda.synchronize()


def test_searches_on_an_empty_trace(B, oracle):
    """No requests: every accumulator is zero, the bisection still walks its steps (never above the target, so the
    bracket closes in on its lower end) and the answers' totals are zero."""
    print("search parity empty trace", flush=True)
    tr = DI.handmade_trace(81, 0, tokens=False)
    dt = B.upload_trace(tr)
    templ = [B.Policy(mode=1, l_th=-1), B.Policy(mode=0), B.Policy(mode=1, l_th=10, w_tail=1.0, beta=0.0)]
    specs = [dict(which_param=B.PARAM_W_TAIL, which_acc="device_cost", n_steps=9, lo=0.0, hi=5.0, target=1.0),
             dict(which_param=B.PARAM_L_TH, which_acc="server_prefill_tok", n_steps=9, lo=0, hi=100, target=0.0),
             dict(which_param=B.PARAM_BETA, which_acc="device_prefill_tok", n_steps=9, lo=0.0, hi=1.0, target=0.0)]
    res = B.disco_budget_search(dt, DI.COST_D, templ, specs)
    so = B.search_to_host(res["out"], 3)
    w, hp, ha = oracle.search_wait(tr, oracle.Policy(mode=1, l_th=-1), 0.0, 5.0, 9, "device_cost", DI.COST_D, 1.0)
    assert np.float32(so["param"][0]) == w and (so["hist_param"][0][:9].astype(np.float32) == hp).all()
    lth, hp, ha = oracle.search_lth(tr, oracle.Policy(mode=0), 0, 100, 9, "server_prefill_tok", DI.COST_D, 0.0)
    assert int(so["param"][1]) == lth and (so["hist_param"][1][:9].astype(np.int32) == hp).all()
    b, hp, ha = oracle.search_slope(tr, oracle.Policy(mode=1, l_th=10, w_tail=1.0, beta=0.0), 0.0, 1.0, 9,
                                    "device_prefill_tok", DI.COST_D, 0.0)
    assert np.float32(so["param"][2]) == b and (so["hist_param"][2][:9].astype(np.float32) == hp).all()
    assert (so["hist_acc"][:, :9] == 0).all()
    for j in range(3):
        assert int(so["at_param"][j]["s_pre"]) == 0 and int(so["at_param"][j]["d_dec"]) == 0
