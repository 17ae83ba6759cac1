"""GPU parity of the closed-form policy solves (Alg. 2, Alg. 3 / Eq. 3) against
the oracle's exact-rational solve: thresholds, partial lengths, ranks and token
masses exactly, the selected waits bit for bit; then the solved table is
evaluated end to end (device-resident, never visiting the host)."""
from fractions import Fraction as F
import math

import numpy as np
import pytest

import disco_inputs as DI
from oracle import disco_solve as S

pytestmark = pytest.mark.gpu


def check_solve(B, tr, specs):
    dt = B.upload_trace(tr)
    res = B.disco_solve_policy(dt, specs)
    pol = np.frombuffer(res["pol_out"].cpu().numpy().tobytes(), dtype=B.POLICY_DTYPE, count=len(specs))
    out = B.solve_to_host(res["out"], len(specs))
    for j, sp in enumerate(specs):
        b = F(*sp["b"])
        assert int(out["status"][j]) == 0
        if sp["mode"] == 0:
            w = S.solve_server_constrained(tr["prompt_len"], b)
            assert int(pol["mode"][j]) == 0 and int(pol["l_th"][j]) == w["l_th"], (j, sp, int(pol["l_th"][j]), w)
            assert int(out["total_tokens"][j]) == w["total_tokens"]
            assert int(out["total_tokens"][j]) - int(out["zero_wait_tokens"][j]) == w["server_tokens"]
        else:
            w = S.solve_device_constrained(tr["prompt_len"], tr["srv_ttft"], b, F(*sp["alpha"]))
            got = (int(pol["l_th"][j]), int(pol["l_mid"][j]), int(out["rank_tail"][j]), int(out["rank_mid"][j]),
                   int(out["zero_wait_tokens"][j]), int(out["total_tokens"][j]))
            want = (w["l_th"], w["l_mid"], w["rank_tail"], w["rank_mid"], w["zero_wait_tokens"], w["total_tokens"])
            assert got == want, (j, sp, got, want)
            assert np.float32(pol["w_tail"][j]).view(np.uint32) == np.float32(w["w_tail"]).view(np.uint32), (j, sp)
            assert np.float32(pol["w_mid"][j]).view(np.uint32) == np.float32(w["w_mid"]).view(np.uint32), (j, sp)
            assert int(pol["mode"][j]) == 1 and math.isinf(pol["beta"][j])
        assert int(pol["mig_mode"][j]) == sp.get("mig_mode", 0)
    return dt, res


def level_specs(P, alphas=((1, 10),)):
    specs = []
    for j in range(P):
        specs.append(dict(mode=0, b=(j, P - 1)))
        for a in alphas:
            specs.append(dict(mode=1, b=(j, P - 1), alpha=a, mig_mode=1))
    return specs


@pytest.mark.parametrize("n_req", [0, 1, 2, 65, 1000, 20_011])
def test_solve_matches_oracle_on_handmade_traces(B, n_req):
    print(f"policy solve parity n_req={n_req}", flush=True)
    tr = DI.handmade_trace(500 + n_req, n_req, tokens=False, ties=True)
    check_solve(B, tr, level_specs(9, alphas=((1, 10), (1, 3)))[:64])
    check_solve(B, tr, [dict(mode=1, b=(1, 1), alpha=(1, 10)), dict(mode=1, b=(0, 1), alpha=(1, 2)),
                        dict(mode=1, b=(1, 10), alpha=(1, 10)), dict(mode=1, b=(32767, 32768), alpha=(1, 32768)),
                        dict(mode=0, b=(1, 32768)), dict(mode=0, b=(32767, 32768))])


def test_solve_few_lengths_and_tied_ttfts(B):
    """Coarse supports: the partial length carries most of the mass and many server TTFTs are equal."""
    print("policy solve parity coarse support", flush=True)
    rng = np.random.default_rng(8)
    n = 5000
    tr = DI.handmade_trace(9, n, tokens=False)
    tr["prompt_len"] = rng.choice([7, 300, 301, 32771], n, p=[0.4, 0.3, 0.2, 0.1]).astype(np.int32)
    tr["srv_ttft"] = (rng.integers(1, 40, n).astype(np.float32) / np.float32(16))
    check_solve(B, tr, level_specs(16, alphas=((1, 20), (2, 5)))[:64])


def test_solve_reports_lengths_beyond_the_table(B):
    tr = DI.handmade_trace(10, 100, tokens=False)
    tr["prompt_len"][17] = 40_000
    dt = B.upload_trace(tr)
    res = B.disco_solve_policy(dt, [dict(mode=0, b=(1, 2)), dict(mode=1, b=(1, 2), alpha=(1, 10))])
    assert (B.solve_to_host(res["out"], 2)["status"] == 1).all()


def test_solved_table_evaluates_end_to_end(B, oracle):
    """Workload-0-like trace: 16 levels of Alg. 3 and of Alg. 2 solved on the device, evaluated from the device table."""
    print("policy solve end to end", flush=True)
    cfg = DI.config(0, n_req=30_011, seed=6)
    tr = oracle.gen_trace(cfg["gen"])
    specs = level_specs(16)
    dt, res = check_solve(B, tr, specs)
    r = B.disco_eval_dispatch(dt, res["policies"])
    got = B.stats_to_host(B.disco_reduce_stats(dt, cfg["cost"], res["policies"], r["acc"]), len(specs))
    opol = []
    for sp in specs:
        if sp["mode"] == 0:
            opol.append(oracle.Policy(mode=0, l_th=S.solve_server_constrained(tr["prompt_len"], F(*sp["b"]))["l_th"]))
        else:
            w = S.solve_device_constrained(tr["prompt_len"], tr["srv_ttft"], F(*sp["b"]), F(*sp["alpha"]))
            opol.append(oracle.Policy(mode=1, l_th=w["l_th"], l_mid=w["l_mid"], w_mid=float(w["w_mid"]), w_tail=float(w["w_tail"])))
    want = oracle.stats(tr, opol, cfg["cost"])
    total = int(tr["prompt_len"].astype(np.int64).sum())
    for j, (sp, w) in enumerate(zip(specs, want)):
        assert int(got[j]["s_pre"]) == w["s_pre"] and int(got[j]["d_pre"]) == w["d_pre"] and int(got[j]["d_dec"]) == w["d_dec"]
        for qi in range(2):
            assert np.float32(got[j]["ttft_q"][qi]).view(np.uint32) == np.float32(w["ttft_q"][qi]).view(np.uint32)
        # the budget of the constrained endpoint is met: exactly for Alg. 3, up to sampling noise for Alg. 2
        b = sp["b"][0] / sp["b"][1]
        if sp["mode"] == 0:
            assert w["s_pre"] <= b * total + 1e-9
        else:
            assert abs(w["d_pre"] / total - b) < 0.01, (j, w["d_pre"] / total, b)
