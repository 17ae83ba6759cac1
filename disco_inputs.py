"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds workload *descriptions* (distribution parameters, sizes,
policy grids, cost rates) and small hand-made traces drawn with numpy's own
generator.  It contains none of the method's arithmetic: it imports neither the
CPU oracle nor the GPU library; both consume what it describes.

The five workloads stand in for the paper's measured inputs (server traces of
four commercial APIs, device profiles of three phone/model pairs, Alpaca
prompts), none of which can be shipped.  The recipe follows the paper's own
scalability study, which fits log-normal laws to prompt length and server TTFT
(Sec. 5.3), keeps server TTFT independent of prompt length (Sec. 3, Pearson
table) and device TTFT linear in it, and adds a heavy server tail for the
TTFT spikes reported in Sec. 2.2.
"""
from __future__ import annotations

import math

import numpy as np

# Cost rates: 2e-6 $ per server token; device energy 2e9 FLOPs/token at
# 1e-12 J/FLOP = 2e-3 J per token (App. E: energy linear in FLOPs).
COST_S = {"cs_pre": 2e-6, "cs_dec": 2e-6, "e_pre": 2e-3, "e_dec": 2e-3, "lam": 3e-4}
# lam = 3e-4 $/J makes a device token cost 0.3 server tokens (server-constrained
# by Alg. 1); lam = 5e-3 $/J makes it 5 server tokens (device-constrained).
COST_D = dict(COST_S, lam=5e-3)

TAU = 0.2        # pacing interval, 5 tokens/s reading speed (Sec. 2.1)
KAPPA_LAG = 3.0  # hand-off when a token is more than 3 pacing intervals overdue


def _gen(n_req, *, prompt_hi=4096, out=(5.0, 0.8, 1, 1024), pareto_alpha=1.5,
         dev=(0, 1.0 / 20.0, 1.0 / 800.0, 0.0, 40.0), tokens=False, seed=0):
    return {
        "seed": seed, "n_req": int(n_req),
        "prompt_mu": 5.5, "prompt_sigma": 1.0, "prompt_lo": 8, "prompt_hi": prompt_hi,
        "out_mu": out[0], "out_sigma": out[1], "out_lo": out[2], "out_hi": out[3],
        "ttft_mu": -1.2, "ttft_sigma": 0.5, "ttft_pareto_p": 0.1,
        "ttft_pareto_xm": 0.5, "ttft_pareto_alpha": pareto_alpha,
        "tbt_mu": -3.5, "tbt_sigma": 0.3,
        "dev_mode": dev[0], "dev_a": dev[1], "dev_b": dev[2], "dev_p": dev[3], "dev_pre_ratio": dev[4],
        "gap_mu": -3.5, "gap_sigma": 0.6, "gap_stall_p": 0.01, "gap_stall_lo": 0.5, "gap_stall_hi": 2.0,
        "tokens": tokens, "dev_ttft_c": 0.0,
    }


def config(idx: int, n_req: int | None = None, seed: int = 0) -> dict:
    """Workload `idx` (0..4).  `n_req` overrides the request count (scaled-down
    runs keep every distribution)."""
    if idx == 0:
        return {"name": "config0", "gen": _gen(n_req or 10_000, seed=seed), "levels": 16,
                "cost": COST_S, "timelines": True, "tau": TAU, "kappa": KAPPA_LAG}
    if idx == 1:
        return {"name": "config1", "gen": _gen(n_req or 1_000_000, seed=seed), "levels": 64,
                "cost": COST_S, "timelines": False, "tau": TAU, "kappa": KAPPA_LAG}
    if idx == 2:
        return {"name": "config2",
                "gen": _gen(n_req or 100_000, out=(5.5, 0.7, 1, 2048),
                            dev=(1, 15.0, 40.0, 0.0, 40.0), tokens=True, seed=seed),
                "levels": 1, "cost": COST_S, "timelines": True, "tau": TAU, "kappa": KAPPA_LAG}
    if idx == 3:
        return {"name": "config3", "gen": _gen(n_req or 4_000_000, pareto_alpha=1.2, seed=seed),
                "levels": 1, "cost": COST_D, "timelines": False, "tau": TAU, "kappa": KAPPA_LAG,
                "search": {"lo": 0.0, "hi": 5.0, "steps": 32, "budget_frac": 0.30}}
    if idx == 4:
        return {"name": "config4",
                "gen": _gen(n_req or 1_000_000, prompt_hi=32768, out=(5.8, 0.9, 1, 4096),
                            dev=(2, 8.0, 40.0, 0.5, 40.0), tokens=True, seed=seed),
                "levels": 8, "cost": COST_S, "timelines": True, "tau": TAU, "kappa": KAPPA_LAG}
    raise ValueError(idx)


def budget_levels(P: int):
    """Budget ratios b_j = j / (P-1) as exact fractions (num, den); a single
    level is the full budget."""
    if P == 1:
        return [(1, 1)]
    return [(j, P - 1) for j in range(P)]


def handmade_trace(seed: int, n_req: int, *, tokens: bool, max_out: int = 300,
                   per_request_device: bool = True, stall_p: float = 0.02,
                   ties: bool = False) -> dict:
    """Small irregular trace from numpy's PCG64 (not the method's generator):
    ragged output lengths including 1, occasional stalls, optional exact ties
    between server and device TTFT."""
    rng = np.random.default_rng(seed)
    prompt_len = rng.integers(1, 3000, n_req).astype(np.int32)
    output_len = rng.integers(1, max_out + 1, n_req).astype(np.int32)
    if n_req:
        output_len[rng.integers(0, n_req, max(1, n_req // 10))] = 1
    srv_ttft = rng.lognormal(-1.2, 0.7, n_req).astype(np.float32)
    srv_tbt = rng.lognormal(-3.5, 0.3, n_req).astype(np.float32)
    k_s, g_s = np.float32(1.0 / 800.0), np.float32(0.05)
    if per_request_device:
        dec = (1.0 / rng.uniform(4.0, 40.0, n_req)).astype(np.float32)
        pre = (dec / np.float32(40.0)).astype(np.float32)
    else:
        dec = pre = None
    if ties and n_req:
        k = pre if pre is not None else np.full(n_req, k_s, np.float32)
        idx = rng.integers(0, n_req, max(1, n_req // 5))
        # server TTFT exactly equal to k*l (one rounding, same as the fused form when c = 0)
        srv_ttft[idx] = (prompt_len[idx].astype(np.float32) * k[idx]).astype(np.float32)
    tok_off = np.zeros(n_req + 1, np.int64)
    np.cumsum(output_len, out=tok_off[1:])
    tok_arr = None
    if tokens:
        total = int(tok_off[-1])
        gaps = rng.lognormal(-3.5, 0.6, total).astype(np.float32)
        stall = rng.random(total) < stall_p
        gaps[stall] = rng.uniform(0.5, 2.0, int(stall.sum())).astype(np.float32)
        tok_arr = np.empty(total, np.float32)
        for i in range(n_req):
            a, b = int(tok_off[i]), int(tok_off[i + 1])
            tok_arr[a] = 0.0
            tok_arr[a + 1:b] = np.cumsum(gaps[a + 1:b], dtype=np.float32)
    return {"n_req": n_req, "n_tok": int(tok_off[-1]), "prompt_len": prompt_len,
            "output_len": output_len, "srv_ttft": srv_ttft, "srv_tbt": srv_tbt,
            "dev_pre_spt": pre, "dev_dec_spt": dec, "tok_off": tok_off, "tok_arr": tok_arr,
            "dev_pre_spt_s": float(k_s), "dev_dec_spt_s": float(g_s), "dev_ttft_c": 0.0}


def f32(x: float) -> float:
    """Round a Python float to the nearest fp32 (what both sides receive)."""
    return float(np.float32(x))


INF = math.inf
