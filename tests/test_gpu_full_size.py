"""GPU parity at the full sizes of the five workloads, with the same sequence
of calls the benchmark times (search -> dispatch -> timelines -> statistics,
policy columns resident on the device).

Workloads 1, 2 and 3 are small enough for the oracle to evaluate whole.  For
workload 4 (4.9e8 token events) the oracle evaluates every request-level
quantity whole and the token-level ones on a sample of requests; the totals
and the selected TBT order statistics are then tied to the per-pair and
per-token outputs (which the sample checks bit for bit) by properties that
hold at any size: a total is the sum of its per-pair terms, and a value v is
the k-th smallest iff  #{x < v} < k <= #{x <= v}."""
import math

import numpy as np
import pytest
import torch

import disco_inputs as DI
from test_gpu_parity import REL, assert_same_bits, close

pytestmark = pytest.mark.gpu


def _levels_search(B, oracle, cfg, tr, dt, mig_mode):
    """Budget levels -> thresholds on both sides; returns (device policies, oracle policies, the accumulators the
    search leaves for the found columns: its last pass is their evaluation, as in the benchmark's step)."""
    P = cfg["levels"]
    levels = DI.budget_levels(P)
    total = int(tr["prompt_len"].astype(np.int64).sum())
    lmax = int(tr["prompt_len"].max())
    steps = max(1, (lmax + 1).bit_length())
    templ = [B.Policy(mode=0, mig_mode=mig_mode) for _ in levels]
    specs = [dict(which_param=B.PARAM_L_TH, which_acc="server_prefill_tok", n_steps=steps, lo=0, hi=lmax + 1,
                  target=num * total / den) for num, den in levels]
    acc = torch.zeros(P * 128, dtype=torch.uint8, device="cuda")
    res = B.disco_budget_search(dt, cfg["cost"], templ, specs, acc=acc)
    found = B.policies_to_host(res["pol_out"], P)
    so = B.search_to_host(res["out"], P)
    opol = []
    for j, (num, den) in enumerate(levels):
        l_th, hp, ha = oracle.search_lth(tr, oracle.Policy(mode=0), 0, lmax + 1, steps, "server_prefill_tok",
                                         cfg["cost"], num * total / den)
        assert found[j].l_th == l_th == int(so["param"][j]), j
        assert (so["hist_param"][j][:steps] == hp).all() and (so["hist_acc"][j][:steps] == ha).all(), j
        opol.append(oracle.Policy(mode=0, l_th=l_th, mig_mode=mig_mode))
    return res["policies"], opol, acc


def _compare_stats(got, want, with_tbt):
    for j, w in enumerate(want):
        g = got[j]
        for f in ("s_pre", "s_dec", "d_pre", "d_dec", "n_dev_started", "n_dev_win", "n_req"):
            assert int(g[f]) == int(w[f]), (f, j)
        for f in ("server_cost", "device_energy", "device_cost", "total_cost"):
            assert close(float(g[f]), float(w[f]), 1e-12), (f, j)
        assert close(float(g["mean_ttft"]), w["mean_ttft"]), j
        for qi in range(2):
            assert int(g["ttft_rank"][qi]) == w["ttft_rank"][qi], (j, qi)
            assert np.float32(g["ttft_q"][qi]).view(np.uint32) == np.float32(w["ttft_q"][qi]).view(np.uint32), (j, qi)
            if with_tbt:
                assert int(g["tbt_rank"][qi]) == w["tbt_rank"][qi], (j, qi)
                assert np.float32(g["tbt_q"][qi]).view(np.uint32) == np.float32(w["tbt_q"][qi]).view(np.uint32), (j, qi)
        if with_tbt:
            assert int(g["n_migrated"]) == w["n_migrated"] and int(g["tbt_count"]) == w["tbt_count"], j
            assert close(float(g["mean_tbt"]), w["mean_tbt"]), j


@pytest.mark.timeout(300)
def test_workload1_full_size(B, oracle):
    """10^6 requests x 64 budget levels, dispatch only: thresholds, totals, mean/p50/p99 TTFT, cost."""
    print("full size: workload 1", flush=True)
    cfg = DI.config(1)
    tr = oracle.gen_trace(cfg["gen"])
    dt = B.disco_gen_trace(cfg["gen"])
    for name in ("prompt_len", "output_len", "srv_ttft"):
        assert_same_bits(getattr(dt, name).cpu().numpy(), tr[name], name)
    dpol, opol, acc = _levels_search(B, oracle, cfg, tr, dt, 0)
    ws = B.workspace(dt.n_req, cfg["levels"])
    got = B.stats_to_host(B.disco_reduce_stats(dt, cfg["cost"], dpol, acc, ws=ws), cfg["levels"])
    # a separate evaluation of the found columns leaves the same accumulators
    a0, a1 = B.accum_to_host(acc, cfg["levels"]), B.accum_to_host(B.disco_eval_dispatch(dt, dpol, ws=ws)["acc"], cfg["levels"])
    for f in ("s_pre", "s_dec", "d_pre", "d_dec", "n_dev_started", "n_dev_win", "ttft_min_bits", "ttft_max_bits"):
        assert (a0[f] == a1[f]).all(), f
    assert np.allclose(a0["ttft_sum"], a1["ttft_sum"], rtol=1e-12, atol=0)
    print("full size: workload 1 oracle statistics", flush=True)
    want = oracle.stats(tr, opol, cfg["cost"])
    _compare_stats(got, want, False)
    assert want[0]["s_pre"] == 0 and want[-1]["d_dec"] < want[0]["d_dec"]


@pytest.mark.timeout(300)
def test_workload2_full_size(B, oracle):
    """10^5 requests, 3.1e7 token events, one column with the lag-triggered hand-off."""
    print("full size: workload 2", flush=True)
    cfg = DI.config(2)
    tr = oracle.gen_trace(cfg["gen"])
    dt = B.disco_gen_trace(cfg["gen"])
    assert dt.n_tok == tr["n_tok"]
    assert_same_bits(dt.tok_arr.cpu().numpy(), tr["tok_arr"], "tok_arr")
    dpol, opol, acc = _levels_search(B, oracle, cfg, tr, dt, 1)
    ws = B.workspace(dt.n_req, 1)
    r = {"acc": acc}
    mg = B.disco_eval_migration(dt, cfg["tau"], cfg["kappa"], dpol, materialise=True, delivered_col=0, ws=ws, acc=r["acc"])
    got = B.stats_to_host(B.disco_reduce_stats(dt, cfg["cost"], dpol, r["acc"], tau=cfg["tau"], kappa=cfg["kappa"], ws=ws), 1)
    print("full size: workload 2 oracle", flush=True)
    want_m = oracle.migration(tr, opol, cfg["tau"], cfg["kappa"], materialise=True, tbt_col=0, want_delivered=True)
    assert_same_bits(mg["mig_idx"].cpu().numpy(), want_m["mig_idx"], "mig_idx")
    assert_same_bits(mg["n_src_tok"].cpu().numpy(), want_m["n_src_tok"], "n_src_tok")
    assert_same_bits(mg["t_last"].cpu().numpy(), want_m["t_last"], "t_last")
    assert_same_bits(mg["delivered"].cpu().numpy(), want_m["delivered"], "delivered")
    want = oracle.stats(tr, opol, cfg["cost"], tau=cfg["tau"], kappa=cfg["kappa"])
    _compare_stats(got, want, True)
    assert want[0]["n_migrated"] > 500


@pytest.mark.timeout(300)
def test_workload3_full_size(B, oracle):
    """4x10^6 requests, 32 bisection steps on the wait time: the whole history bit for bit."""
    print("full size: workload 3", flush=True)
    cfg = DI.config(3)
    tr = oracle.gen_trace(cfg["gen"])
    dt = B.disco_gen_trace(cfg["gen"])
    for name in ("prompt_len", "output_len", "srv_ttft"):
        assert_same_bits(getattr(dt, name).cpu().numpy(), tr[name], name)
    s = cfg["search"]
    c_all = cfg["cost"]["cs_pre"] * (int(tr["prompt_len"].astype(np.int64).sum()) + int(tr["output_len"].astype(np.int64).sum()))
    res = B.disco_budget_search(dt, cfg["cost"], [B.Policy(mode=1, l_th=-1)],
                                [dict(which_param=B.PARAM_W_TAIL, which_acc="device_cost", n_steps=s["steps"], lo=s["lo"],
                                      hi=s["hi"], target=s["budget_frac"] * c_all)])
    so = B.search_to_host(res["out"], 1)
    w, hp, ha = oracle.search_wait(tr, oracle.Policy(mode=1, l_th=-1), s["lo"], s["hi"], s["steps"], "device_cost",
                                   cfg["cost"], s["budget_frac"] * c_all)
    assert np.float32(so["param"][0]) == w
    assert (so["hist_param"][0][:32].astype(np.float32) == hp).all()
    assert (so["hist_acc"][0][:32] == ha).all()
    d = oracle.dispatch(tr, [oracle.Policy(mode=1, l_th=-1, w_tail=float(w))], materialise=False)
    at = so["at_param"][0]
    for f in ("s_pre", "s_dec", "d_pre", "d_dec", "n_dev_started", "n_dev_win"):
        assert int(at[f]) == int(d[f][0]), f
    # the bracket has closed to 5 * 2^-32 and the found wait is on the feasible side
    spend = cfg["cost"]["lam"] * oracle.device_energy(cfg["cost"], int(d["d_pre"][0]), int(d["d_dec"][0]))
    assert spend <= s["budget_frac"] * c_all


@pytest.mark.timeout(600)
def test_workload4_full_size(B, oracle):
    """10^6 requests x 8 levels, 4.9e8 token events, in the benchmark's launch configuration.  Request-level results
    against the oracle in full; token-level results against the oracle on sampled requests (hand-off index, source
    tokens and last delivery in all eight columns, every delivery of the all-race column), totals and order
    statistics by properties.  The class-mode TBT selection is compared with the oracle itself on a contiguous slice
    of the same recipe in test_workload4_slice_against_the_oracle."""
    print("full size: workload 4", flush=True)
    cfg = DI.config(4)
    tau, kappa, P = cfg["tau"], cfg["kappa"], cfg["levels"]
    tr = oracle.gen_requests(cfg["gen"])
    dt = B.disco_gen_trace(cfg["gen"])
    N, T = dt.n_req, dt.n_tok
    assert T == tr["n_tok"]
    for name in ("prompt_len", "output_len", "srv_ttft", "dev_pre_spt", "dev_dec_spt", "tok_off"):
        assert_same_bits(getattr(dt, name).cpu().numpy(), tr[name], name)
    dpol, opol, sacc = _levels_search(B, oracle, cfg, tr, dt, 1)
    ws = B.workspace(N, P)
    r = {"acc": sacc}
    # the benchmark's launch configuration: streaming token walk (per-pair outputs from its summaries), then the
    # statistics starting from what the walk left in the workspace
    mg = B.disco_eval_migration(dt, tau, kappa, dpol, materialise=True, ws=ws, acc=r["acc"])
    acc = B.accum_to_host(r["acc"], P)
    got = B.stats_to_host(B.disco_reduce_stats(dt, cfg["cost"], dpol, r["acc"], tau=tau, kappa=kappa, ws=ws, reuse_walk=True), P)
    # ... and once more walking the tokens again: the same statistics
    got2 = B.stats_to_host(B.disco_reduce_stats(dt, cfg["cost"], dpol, r["acc"], tau=tau, kappa=kappa, ws=ws), P)
    assert got.tobytes() == got2.tobytes()
    # per-token deliveries of the all-race column (the general kernel): server-sourced and migrated timelines
    mg["delivered"] = B.disco_eval_migration(dt, tau, kappa, dpol, materialise=False, delivered_col=P - 1, ws=ws)["delivered"]
    torch.cuda.synchronize()

    # (1) request-level: dispatch totals and TTFT statistics of every column, whole
    print("full size: workload 4 oracle dispatch", flush=True)
    want_d = oracle.stats(tr, opol, cfg["cost"])
    for j, w in enumerate(want_d):
        g = got[j]
        for f in ("s_pre", "n_dev_started", "n_dev_win", "n_req"):
            assert int(g[f]) == int(w[f]), (f, j)
        assert close(float(g["mean_ttft"]), w["mean_ttft"]), j
        for qi in range(2):
            assert int(g["ttft_rank"][qi]) == w["ttft_rank"][qi]
            assert np.float32(g["ttft_q"][qi]).view(np.uint32) == np.float32(w["ttft_q"][qi]).view(np.uint32), (j, qi)
    dec = oracle.dispatch(tr, opol, materialise=True)["decision"]

    # (2) token-level on sampled requests: generator, hand-off index, source tokens, last delivery, deliveries
    print("full size: workload 4 sampled timelines", flush=True)
    rng = np.random.default_rng(4)
    mig0 = mg["mig_idx"][P - 1].cpu().numpy()
    picks = np.unique(np.concatenate([
        rng.integers(0, N, 1500), [0, 1, N - 2, N - 1], np.argsort(tr["output_len"])[-40:],
        np.flatnonzero(tr["output_len"] == 1)[:40], np.flatnonzero(mig0 >= 0)[:300]]))
    n_s = tr["output_len"][picks]
    off_s = np.zeros(len(picks) + 1, np.int64)
    np.cumsum(n_s, out=off_s[1:])
    arr_s = np.empty(int(off_s[-1]), np.float32)
    gpu_arr = dt.tok_arr
    for a, i in enumerate(picks):
        seg = oracle.gen_tokens(cfg["gen"], tr["tok_off"], int(i), int(i) + 1)
        arr_s[off_s[a]:off_s[a + 1]] = seg
        lo = int(tr["tok_off"][i])
        assert_same_bits(gpu_arr[lo:lo + seg.size].cpu().numpy(), seg, f"tok_arr of request {i}")
    sub = {"n_req": len(picks), "n_tok": int(off_s[-1]), "tok_off": off_s, "tok_arr": arr_s,
           "dev_pre_spt_s": 0.0, "dev_dec_spt_s": 0.0, "dev_ttft_c": 0.0}
    for name in ("prompt_len", "output_len", "srv_ttft", "srv_tbt", "dev_pre_spt", "dev_dec_spt"):
        sub[name] = np.ascontiguousarray(tr[name][picks])
    want_m = oracle.migration(sub, opol, tau, kappa, materialise=True, tbt_col=P - 1, want_delivered=True)
    sub_dec = oracle.dispatch(sub, opol, materialise=True)["decision"][P - 1]
    assert ((sub_dec & 4) == 0).sum() > 500, "the sampled deliveries must cover server-sourced timelines"
    pk = torch.from_numpy(picks).cuda()
    for name in ("mig_idx", "n_src_tok", "t_last"):
        assert_same_bits(mg[name][:, pk].cpu().numpy(), want_m[name], name)
    assert (want_m["mig_idx"] >= 0).sum() > 100
    deliv = mg["delivered"]
    for a, i in enumerate(picks):
        lo = int(tr["tok_off"][i])
        assert_same_bits(deliv[lo:lo + int(n_s[a])].cpu().numpy(), want_m["delivered"][off_s[a]:off_s[a + 1]],
                         f"delivered of request {i}")

    # (3) totals = sums of the per-pair outputs checked above
    print("full size: workload 4 totals", flush=True)
    n_all = torch.from_numpy(tr["output_len"]).cuda().to(torch.int64)
    l_all = torch.from_numpy(tr["prompt_len"]).cuda().to(torch.int64)
    dev_src = (torch.from_numpy(dec).cuda() & 4) != 0
    sum_n = int(n_all.sum().item())
    for j in range(P):
        m = mg["mig_idx"][j].to(torch.int64)
        ns = mg["n_src_tok"][j].to(torch.int64)
        srv = ~dev_src[j]
        s_dec = int(ns[srv].sum().item())
        migd = m >= 0
        assert int(acc["m_s_dec"][j]) == s_dec and int(acc["m_d_dec"][j]) == sum_n - s_dec, j
        assert int(acc["n_migrated"][j]) == int(migd.sum().item()), j
        assert int(acc["m_d_repre"][j]) == int((l_all[migd] + m[migd]).sum().item()), j
        assert int(acc["tbt_count"][j]) == sum_n - N, j
        assert not bool((migd & dev_src[j]).any().item()), "a device-sourced timeline never hands off"
        tl_sum = float(mg["t_last"][j].to(torch.float64).sum().item())
        assert close(float(acc["tlast_sum"][j]), tl_sum), j
        assert close(float(got[j]["mean_tbt"]), tl_sum / (sum_n - N)), j
        assert int(got[j]["s_dec"]) == s_dec and int(got[j]["d_dec"]) == sum_n - s_dec, j
        assert int(got[j]["d_pre"]) == int(acc["d_pre"][j]) + int(acc["m_d_repre"][j]), j
        w = oracle.total_cost(cfg["cost"], int(got[j]["s_pre"]), s_dec, int(got[j]["d_pre"]), sum_n - s_dec)
        assert close(float(got[j]["total_cost"]), w, 1e-12), j

    # (4) TBT order statistics of every column: rank by the nearest-rank rule, value by counting
    print("full size: workload 4 order statistics", flush=True)
    starts = torch.from_numpy(tr["tok_off"][:-1]).cuda()
    for j in range(P):
        if j < P - 1:
            mj = B.disco_eval_migration(dt, tau, kappa, dpol, materialise=False, delivered_col=j, ws=ws)
            deliv = mj["delivered"]
        else:
            deliv = mg["delivered"]
        gaps = deliv[1:] - deliv[:-1]
        keep = torch.ones(T - 1, dtype=torch.bool, device="cuda")
        keep[starts[1:] - 1] = False          # the difference across a request boundary is no gap
        for qi, (num, den) in enumerate(((50, 100), (99, 100))):
            k = (num * (sum_n - N) + den - 1) // den
            k = max(k, 1)
            assert int(got[j]["tbt_rank"][qi]) == k, (j, qi)
            v = torch.tensor(float(got[j]["tbt_q"][qi]), dtype=torch.float32, device="cuda")
            below = int(((gaps < v) & keep).sum().item())
            upto = int(((gaps <= v) & keep).sum().item())
            assert below < k <= upto, (j, qi, below, k, upto)
        del gaps, keep
        print(f"full size: workload 4 column {j} done", flush=True)


@pytest.mark.timeout(600)
def test_workload4_slice_against_the_oracle(B, oracle):
    """The first 50 000 requests of workload 4 (2.4e7 token events: requests of many 256-token iterations, the
    two-round TTFT buckets, eight columns of nested classes), evaluated whole by the oracle: thresholds, every
    total, and the rank and bit pattern of every TTFT and TBT order statistic of all eight columns, through the
    same sequence of calls as the benchmark's step."""
    print("workload 4, 50k-request slice: GPU", flush=True)
    cfg = DI.config(4, n_req=50_000)
    tau, kappa, P = cfg["tau"], cfg["kappa"], cfg["levels"]
    tr = oracle.gen_trace(cfg["gen"])
    dt = B.disco_gen_trace(cfg["gen"])
    assert dt.n_tok == tr["n_tok"]
    assert_same_bits(dt.tok_arr.cpu().numpy(), tr["tok_arr"], "tok_arr")
    dpol, opol, acc = _levels_search(B, oracle, cfg, tr, dt, 1)
    ws = B.workspace(dt.n_req, P)
    mg = B.disco_eval_migration(dt, tau, kappa, dpol, materialise=True, ws=ws, acc=acc)
    got = B.stats_to_host(B.disco_reduce_stats(dt, cfg["cost"], dpol, acc, tau=tau, kappa=kappa, ws=ws, reuse_walk=True), P)
    print("workload 4, 50k-request slice: oracle", flush=True)
    want_m = oracle.migration(tr, opol, tau, kappa, materialise=True)
    for name in ("mig_idx", "n_src_tok", "t_last"):
        assert_same_bits(mg[name].cpu().numpy(), want_m[name], name)
    want = oracle.stats(tr, opol, cfg["cost"], tau=tau, kappa=kappa)
    _compare_stats(got, want, True)
    assert want[P - 1]["n_migrated"] > 300 and want[0]["n_migrated"] == 0
    for j in range(P):
        assert int(got[j]["s_dec"]) == want[j]["s_dec"] and int(got[j]["d_dec"]) == want[j]["d_dec"], j
        assert int(got[j]["d_pre"]) == want[j]["d_pre"], j
