#!/usr/bin/env python3
"""Benchmark of the DiSCo policy-evaluation path on one MI355X.

A step is one pass of the whole path over one resident batch: budget search
(one length threshold per budget level), fused dispatch + reduction, order
statistics -- and, for workloads with token timelines, the timeline pass and
the TBT order statistics.  The headline workload is configuration 1
(10^6 requests x 64 budget levels, dispatch only); the other configurations
are reported as extra fields of the same JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload config1] [--extras config2,config3,config4,config4buffer,config1stoch]
    python bench.py --copy-calibration BYTES     # one plain device copy of known size, for scaling HBM counters
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E peak
# Vector-ALU peak for the non-packed fp32 / fp64 / integer / compare instructions this path is made of:
# 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz, one operation per lane and clock
ALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# Operations per evaluated (request, column) pair of a length-threshold column (Alg. 3), with what a race decides
# computed once per request: the comparison l < l_th; three selections (server prefill tokens, device decode
# tokens and win count as one packed word, the TTFT); two integer adds; the fp64 TTFT sum (convert + add); minimum
# and maximum of the TTFT bits.  It is also the number of vector instructions per pair that the kernel issues.
OPS_PER_PAIR = 10


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="config1")
    ap.add_argument("--extras", default="config2,config3,config4,config4buffer,config1stoch")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-reps", type=int, default=20)
    ap.add_argument("--copy-calibration", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on one GPU; --gpus must be 1 (requests are independent and would shard by request)",
              file=sys.stderr)
        return 2

    import torch

    import disco_inputs as DI
    import paper_2502_11417_amd as D

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    if args.copy_calibration:
        # a plain copy kernel of known size: what FETCH_SIZE / WRITE_SIZE read for it scales the other kernels' counters
        n = args.copy_calibration // 4
        src = torch.arange(n, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": n * 4, "launches": 3}))
        return 0

    def sync():
        torch.cuda.synchronize()

    class Workload:
        """Resident trace + everything a step needs, allocated once."""

        def __init__(self, idx, buffer=False, stoch=False):
            self.idx = idx
            self.stoch = stoch
            self.cfg = DI.config(idx)
            g = self.cfg["gen"]
            t0 = time.perf_counter()
            self.trace = D.disco_gen_trace(g)
            sync()
            self.gen_s = time.perf_counter() - t0
            self.N = self.trace.n_req
            self.T = self.trace.n_tok
            self.P = self.cfg["levels"]
            self.ws = D.workspace(self.N, max(self.P, 1))
            self.acc = torch.zeros(self.P * 128, dtype=torch.uint8, device="cuda")
            self.stats = torch.zeros(self.P * 256, dtype=torch.uint8, device="cuda")
            self.sum_l = int(self.trace.prompt_len.sum(dtype=torch.int64).item())
            self.sum_n = int(self.trace.output_len.sum(dtype=torch.int64).item())
            self.lmax = int(self.trace.prompt_len.max().item())
            self.levels = DI.budget_levels(self.P)
            self.lth_steps = max(1, (self.lmax + 1).bit_length())
            # buffer: the cost-triggered hand-off of Sec. 4.3 in place of the lag trigger
            mig = (D.MIG_BUFFER if buffer else D.MIG_LAG) if self.cfg["timelines"] else D.MIG_NONE
            self.templ = [D.Policy(mode=D.MODE_S, mig_mode=mig) for _ in self.levels]
            self.specs = [dict(which_param=D.PARAM_L_TH, which_acc="server_prefill_tok", n_steps=self.lth_steps,
                               lo=0, hi=self.lmax + 1, target=num * self.sum_l / den) for num, den in self.levels]
            # the same table and specs every step: marshalled once
            self.templ_c, self.specs_c = D.prepare_policies(self.templ), D.prepare_specs(self.specs)
            self.sout = torch.zeros(self.P * D.binding.SEARCH_DTYPE.itemsize, dtype=torch.uint8, device="cuda")
            self.pol_out = torch.zeros(self.P * 32, dtype=torch.uint8, device="cuda")
            self.pols = None
            if stoch:
                # the Stoch-S baseline of Sec. 5.1 on the same budget grid: 8 levels x 8 runs, averaged over the runs
                self.runs = 8
                self.levels = DI.budget_levels(self.P // self.runs)
                self.pols = [D.Policy(mode=D.MODE_STOCH_S, beta=num / den, l_mid=run, mig_mode=mig)
                             for num, den in self.levels for run in range(self.runs)]
                self.avg = torch.zeros(len(self.levels) * 256, dtype=torch.uint8, device="cuda")

        def search(self):
            """Budget levels -> length thresholds; the found columns stay on the device."""
            res = D.disco_budget_search(self.trace, self.cfg["cost"], self.templ_c, self.specs_c, ws=self.ws,
                                        out=self.sout, pol_out=self.pol_out, acc=self.acc)
            self.pols = res["policies"]

        def step(self):
            cfg = self.cfg
            if self.idx == 3:
                c_all = cfg["cost"]["cs_pre"] * (self.sum_l + self.sum_n)
                s = cfg["search"]
                return D.disco_budget_search(
                    self.trace, cfg["cost"], [D.Policy(mode=D.MODE_D, l_th=-1)],
                    [dict(which_param=D.PARAM_W_TAIL, which_acc="device_cost", n_steps=s["steps"], lo=s["lo"],
                          hi=s["hi"], target=s["budget_frac"] * c_all)], ws=self.ws)
            # budget levels -> thresholds (device-resident bisection), then evaluate the found columns
            # straight from the device-resident policy table: no host round trip inside a step
            if not self.stoch:
                self.search()
            # (the search's last pass is the evaluation of the found columns: it leaves their accumulators in acc)
            tau = cfg["tau"] if cfg["timelines"] else None
            if self.stoch:
                D.disco_eval_dispatch(self.trace, self.pols, ws=self.ws, acc=self.acc)
            if tau is not None:
                D.disco_eval_migration(self.trace, tau, cfg["kappa"], self.pols, ws=self.ws, acc=self.acc,
                                       cost=cfg["cost"])
            # (the statistics start from what the evaluation's token walk left in the workspace)
            st = D.disco_reduce_stats(self.trace, cfg["cost"], self.pols, self.acc, tau=tau, kappa=cfg["kappa"],
                                      ws=self.ws, out=self.stats, mig_cost=cfg["cost"], reuse_walk=tau is not None)
            if self.stoch:
                return D.disco_average_runs(st, len(self.levels), self.runs, out=self.avg)
            return st

        def time_steps(self, steps, warmup):
            if self.idx != 3 and not self.stoch:
                self.search()
            for _ in range(warmup):
                self.step()
            sync()
            t0 = time.perf_counter()
            for _ in range(steps):
                self.step()
            sync()
            return (time.perf_counter() - t0) / steps

    def event_time(fn, reps):
        """Average duration of `fn` over `reps` back-to-back calls, HIP events on the launch stream."""
        fn()
        sync()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        sync()
        return e0.elapsed_time(e1) / reps * 1e-3

    idx = int(args.workload.replace("config", ""))
    log(f"[bench] generating {args.workload} ...")
    w = Workload(idx)
    log(f"[bench] {args.workload}: N={w.N} P={w.P} T={w.T} gen {w.gen_s * 1e3:.1f} ms; timing {args.steps} steps")
    sec = w.time_steps(args.steps, args.warmup)
    pairs = w.N * (w.cfg["search"]["steps"] if idx == 3 else w.P)
    value = pairs / sec

    # Kernel of the headline path that the roofline is quoted for: the fused dispatch-and-reduce pass (it runs once
    # inside the budget search and once for the evaluation).  With many columns it is bound by vector arithmetic
    # (OPS_PER_PAIR operations per pair against 12 B per request: prompt length, server TTFT, output length,
    # independent of the number of columns); with one column by memory.  The timed call also launches the 5-us
    # kernel that stages the policy table, so the figures are slightly conservative.
    bytes_per_launch = 12.0 * w.N
    if idx == 3:
        one = [D.Policy(mode=D.MODE_D, l_th=-1, w_tail=0.6)]
        t_k = event_time(lambda: D.disco_eval_dispatch(w.trace, one, ws=w.ws, acc=w.acc), args.kernel_reps)
        pairs_per_launch = w.N
    else:
        t_k = event_time(lambda: D.disco_eval_dispatch(w.trace, w.pols, ws=w.ws, acc=w.acc), args.kernel_reps)
        pairs_per_launch = w.N * w.P
    gbs = bytes_per_launch / t_k / 1e9
    tops = OPS_PER_PAIR * pairs_per_launch / t_k / 1e12
    common = {"kernel": "k_dispatch_acc", "traffic": measured_traffic("k_dispatch_acc", args.workload),
              "launch_us": round(t_k * 1e6, 2), "pairs_per_s_in_kernel": pairs_per_launch / t_k}
    if idx == 3:
        roofline = {"bound": "hbm", "achieved": round(gbs, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(gbs / HBM_PEAK_GBS, 4), **common}
    else:
        roofline = {"bound": "alu", "achieved": round(tops, 3), "peak": round(ALU_PEAK_TOPS, 2), "unit": "Top/s",
                    "frac": round(tops / ALU_PEAK_TOPS, 4), **common,
                    "hbm": {"achieved": round(gbs, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4)}}

    result = {
        "metric": "request x policy evaluations/s", "value": value, "unit": "pairs/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": sec * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "n_req": w.N, "policy_columns": w.P, "token_events": w.T,
                   "step": "budget search + fused dispatch/reduce + order statistics"},
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(idx)

    extras = {}
    if idx != 3:
        # closed-form policy solves (Alg. 3 and Alg. 2) for the budget grid of the timed workload: half the columns each
        half = max(1, w.P // 2)
        sspecs = [dict(mode=D.MODE_S, b=(j, max(half - 1, 1))) for j in range(half)] + \
                 [dict(mode=D.MODE_D, b=(j, max(half - 1, 1)), alpha=(1, 10)) for j in range(half)]
        spol = torch.zeros(len(sspecs) * 32, dtype=torch.uint8, device="cuda")
        sout = torch.zeros(len(sspecs) * D.binding.SOLVE_DTYPE.itemsize, dtype=torch.uint8, device="cuda")
        t_s = event_time(lambda: D.disco_solve_policy(w.trace, sspecs, ws=w.ws, pol_out=spol, out=sout), 10)
        extras["policy_solve"] = {"workload": args.workload, "columns": len(sspecs), "ms": t_s * 1e3,
                                  "what": "length table + per-column plan + 4-pass multi-rank selection over the server TTFTs"}
    for name in [e for e in args.extras.split(",") if e and e != args.workload]:
        if not name.startswith("config"):
            continue
        buffer, stoch = name.endswith("buffer"), name.endswith("stoch")
        k = int(name.replace("config", "").replace("buffer", "").replace("stoch", ""))
        del w
        torch.cuda.empty_cache()
        log(f"[bench] extra {name} ...")
        w = Workload(k, buffer=buffer, stoch=stoch)
        steps = 3 if k == 4 else 10
        s = w.time_steps(steps, 1)
        ex = {"n_req": w.N, "policy_columns": w.P, "token_events": w.T, "ms_per_step": s * 1e3}
        if k == 3:
            # 32 recorded bisection steps; the library takes three of them per pass over the trace (7 candidate
            # columns per pass), so the trace is read ceil(32 / 3) + 1 = 12 times
            steps_ = w.cfg["search"]["steps"]
            passes = (steps_ + 2) // 3 + 1
            ex["pairs_per_s"] = w.N * steps_ / s
            ex["passes_over_the_trace"] = passes
            ex["evaluated_pairs_per_s"] = w.N * (7 * (passes - 1) + 1) / s
            ex["hbm_frac_of_peak"] = 12.0 * w.N * passes / s / 1e9 / HBM_PEAK_GBS
        elif not w.cfg["timelines"]:
            ex["pairs_per_s"] = w.N * w.P / s
            if stoch:
                st = D.stats_to_host(w.step(), len(w.levels))
                ex["runs"] = w.runs
                ex["mean_ttft_by_level"] = [float(x) for x in st["mean_ttft"]]
                ex["p99_ttft_by_level"] = [float(x[1]) for x in st["ttft_q"]]
        else:
            ex["pairs_per_s"] = w.N * w.P / s
            ex["token_events_per_s_raw"] = w.T / s
            ex["token_events_per_s_pair_weighted"] = w.T * w.P / s
            # timeline statistics pass alone: 4 B per token event + 28 B per request, read once for all columns
            tau = w.cfg["tau"]
            t_tl = event_time(lambda: D.disco_eval_migration(w.trace, tau, w.cfg["kappa"], w.pols, ws=w.ws, acc=w.acc,
                                                             cost=w.cfg["cost"]), 3 if k == 4 else 10)
            gb = (4.0 * w.T + 28.0 * w.N) / 1e9
            kern = "k_tl_stats_buf" if buffer else "k_tl_stats"    # pairs with a buffer hand-off: their own statistics kernel
            ex["timeline_kernel"] = {"bound": "hbm", "kernel": kern, "launch_ms": t_tl * 1e3, "achieved_GBs": gb / t_tl,
                                     "frac": gb / t_tl / HBM_PEAK_GBS,
                                     "traffic": measured_traffic(kern, name)}
            if k == 4 and not buffer:
                # recorded-trace ingest at this size: wall-clock fp64 timestamps -> relative arrays, 8 B read and 4 B
                # written per token event (+ 28 B per request); the timestamps are rebuilt from the resident trace
                tr = w.trace
                base = torch.cumsum(torch.full((w.N,), 0.25, dtype=torch.float64, device="cuda"), 0) + 1.7e9
                first = base + tr.srv_ttft.double()
                t_token = torch.repeat_interleave(first, tr.output_len.long()) + tr.tok_arr.double()
                del first
                ing = {}
                t_in = event_time(lambda: ing.update(t=D.disco_ingest_trace(base, t_token, tr.tok_off, tr.prompt_len)), 3)
                gbi = (12.0 * w.T + 28.0 * w.N) / 1e9
                ex["ingest_kernel"] = {"bound": "hbm", "kernel": "k_ingest", "launch_ms": t_in * 1e3,
                                       "achieved_GBs": gbi / t_in, "frac": gbi / t_in / HBM_PEAK_GBS}
                t_fit = event_time(lambda: D.disco_fit_lognormal(tr.srv_ttft, ws=w.ws), 5)
                ex["lognormal_fit_ms"] = t_fit * 1e3
                del t_token, ing, base
            if buffer:
                st = D.stats_to_host(w.step(), w.P)
                ex["migrated_requests"] = [int(x) for x in st["n_migrated"]]
                ex["mean_delay_num"] = [None if x != x else float(x) for x in st["mean_delay_num"]]
        extras[name] = ex
        log(f"[bench] {name}: {json.dumps(ex)}")
    if extras:
        result["extras"] = extras
    print(json.dumps(result))
    return 0


def measured_traffic(kernel: str, workload: str):
    """HBM bytes per launch from the committed rocprofv3 counter summary, or None if there is none for this
    kernel and workload or the kernel sources have changed since the counters were taken."""
    import hashlib

    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        table = json.load(f)
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2502_11417_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        with open(os.path.join(csrc, name), "rb") as f:
            h.update(f.read())
    if table.get("csrc_sha256") != h.hexdigest():
        return None
    entry = table.get("kernels", {}).get(f"{kernel}/{workload}")
    return entry["hbm_bytes_per_launch"] if entry else None


def cpu_baseline(idx: int) -> dict:
    """The oracle as it stands, on a bounded sample of the same workload, on the host's cores."""
    import numpy as np

    import disco_inputs as DI
    from oracle import disco_oracle as O

    n_sample = {0: 10_000, 1: 1_000_000, 2: 100_000, 3: 4_000_000, 4: 20_000}[idx]
    cfg = DI.config(idx, n_req=n_sample)
    tr = O.gen_trace(cfg["gen"])
    t0 = time.perf_counter()
    if idx == 3:
        c_all = cfg["cost"]["cs_pre"] * (int(tr["prompt_len"].astype(np.int64).sum()) + int(tr["output_len"].astype(np.int64).sum()))
        s = cfg["search"]
        O.search_wait(tr, O.Policy(mode=1, l_th=-1), s["lo"], s["hi"], s["steps"], "device_cost", cfg["cost"],
                      s["budget_frac"] * c_all)
        pairs = n_sample * s["steps"]
    else:
        levels = DI.budget_levels(cfg["levels"])
        total = int(tr["prompt_len"].astype(np.int64).sum())
        lmax = int(tr["prompt_len"].max())
        steps = max(1, (lmax + 1).bit_length())
        mig = 1 if cfg["timelines"] else 0
        pols = []
        for num, den in levels:
            l_th, _, _ = O.search_lth(tr, O.Policy(mode=0), 0, lmax + 1, steps, "server_prefill_tok", cfg["cost"],
                                      num * total / den)
            pols.append(O.Policy(mode=0, l_th=l_th, mig_mode=mig))
        O.stats(tr, pols, cfg["cost"], tau=cfg["tau"] if cfg["timelines"] else None, kappa=cfg["kappa"])
        pairs = n_sample * len(levels)
    dt = time.perf_counter() - t0
    return {"value": pairs / dt, "unit": "pairs/s", "cores": 1, "kind": "oracle",
            "sample": f"first {n_sample} requests of config{idx} (same generator and seed), same step, {dt:.1f} s"}


if __name__ == "__main__":
    sys.exit(main())
