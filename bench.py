#!/usr/bin/env python3
"""Benchmark of the DiSCo policy-evaluation path on one MI355X.

A step is one pass of the whole path over one resident batch: budget search
(one length threshold per budget level), fused dispatch + reduction, TTFT order
statistics -- and, for workloads with token timelines, the token walk, the
per-column totals and the TBT order statistics.  The headline workload is the
largest one that fits the GPU, configuration 4 (10^6 requests x 8 budget
levels, 4.9e8 token events, lag-triggered hand-off); the other configurations
are reported as extra fields of the same JSON line, each with its own CPU
baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload config4]
                    [--extras config1,config2,config3,config4buffer,config1stoch]
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
# Vector-ALU peak for the non-packed fp32 / fp64 / integer / compare instructions the dispatch pass is made of:
# 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz, one operation per lane and clock
ALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
# Operations per evaluated (request, column) pair of a length-threshold column (Alg. 3), with what a race decides
# computed once per request: the comparison l < l_th; three selections (server prefill tokens, device decode
# tokens and win count as one packed word, the TTFT); two integer adds; the fp64 TTFT sum (convert + add); minimum
# and maximum of the TTFT bits.
OPS_PER_PAIR = 10
# Bytes per request that the streaming token walk moves besides the tokens: it reads the walk flags (1), the output
# length (4) and the token offset (8) and writes the 16-byte summary.
WALK_BYTES_PER_REQUEST = 29.0
READ_PROBE_BYTES = 4 << 30       # the streaming-read ceiling is measured over 4 GiB


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="config4")
    ap.add_argument("--extras", default="config1,config2,config3,config4buffer,config1stoch")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the step")
    ap.add_argument("--kernel-reps", type=int, default=20)
    ap.add_argument("--copy-calibration", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on one GPU; --gpus must be 1 (requests are independent and would shard by request)",
              file=sys.stderr)
        return 2

    # the CPU baselines of the timed workload first: the all-cores one forks, which must happen before the GPU is initialised
    cpu_pre = {}
    if not args.no_cpu_baseline and not args.copy_calibration:
        idx0 = int("".join(ch for ch in args.workload if ch.isdigit()) or 4)
        log(f"[bench] CPU baselines of config{idx0} (oracle) ...")
        cpu_pre["one"] = {a: b for a, b in cpu_baseline(idx0).items() if not a.startswith("_")}
        cpu_pre["all"] = cpu_baseline_all_cores(idx0)

    import numpy as np
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
            self.buffer = buffer
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
            self.mig = (D.MIG_BUFFER if buffer else D.MIG_LAG) if self.cfg["timelines"] else D.MIG_NONE
            self.templ = [D.Policy(mode=D.MODE_S, mig_mode=self.mig) for _ in self.levels]
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
                self.pols = [D.Policy(mode=D.MODE_STOCH_S, beta=num / den, l_mid=run, mig_mode=self.mig)
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
            """(seconds per step, host seconds per step spent enqueueing)."""
            if self.idx != 3 and not self.stoch:
                self.search()
            for _ in range(warmup):
                self.step()
            sync()
            t0 = time.perf_counter()
            for _ in range(steps):
                self.step()
            t_enq = time.perf_counter() - t0
            sync()
            return (time.perf_counter() - t0) / steps, t_enq / steps

        def time_graph_replay(self, steps):
            """The same step captured once into a HIP graph and replayed: what is left of a step when the host only
            issues one launch.  Returns (seconds per replayed step, the replay's statistics equal the eager step's)."""
            if self.idx != 3 and not self.stoch:
                self.search()
            self.step()
            sync()
            want = self.stats.clone() if self.idx != 3 else None
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                self.step()                               # warm-up on the capture stream
            torch.cuda.current_stream().wait_stream(side)
            sync()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                self.step()
            graph.replay()
            sync()
            same = None
            if want is not None:
                a = D.stats_to_host(self.stats, self.P)
                b = D.stats_to_host(want, self.P)
                same = all((a[f] == b[f]).all() if a[f].dtype.kind in "iu" else
                           bool(np.allclose(a[f], b[f], rtol=1e-9, atol=0, equal_nan=True)) for f in a.dtype.names)
            t0 = time.perf_counter()
            for _ in range(steps):
                graph.replay()
            sync()
            sec = (time.perf_counter() - t0) / steps
            del graph
            return sec, same

        # ---- what a step's throughput is quoted in
        def throughput(self, sec):
            out = {}
            if self.idx == 3:
                steps_ = self.cfg["search"]["steps"]
                passes = (steps_ + 2) // 3 + 1       # three recorded bisection steps per pass over the trace, + the evaluation
                out["pairs_per_s"] = self.N * steps_ / sec
                out["passes_over_the_trace"] = passes
                out["evaluated_pairs_per_s"] = self.N * (7 * (passes - 1) + 1) / sec
                out["hbm_frac_of_peak"] = 12.0 * self.N * passes / sec / 1e9 / HBM_PEAK_GBS
            else:
                out["pairs_per_s"] = self.N * self.P / sec
            if self.cfg["timelines"]:
                out["token_events_per_s_raw"] = self.T / sec
                out["token_events_per_s_pair_weighted"] = self.T * self.P / sec
            return out

        # ---- rooflines
        def must_read_tokens(self):
            """Token events the statistics pass has to read: the tokens of every request with a server-sourced column,
            up to and including the hand-off token where all such columns have the lag trigger and it fired."""
            pols = D.policies_to_host(self.pol_out, self.P) if not self.stoch else self.pols
            dec = D.disco_eval_dispatch(self.trace, self.pols, materialise=True, ws=self.ws)["decision"]
            mg = D.disco_eval_migration(self.trace, self.cfg["tau"], self.cfg["kappa"], self.pols, materialise=True, ws=self.ws,
                                        cost=self.cfg["cost"])
            srv = (dec & 4) == 0
            lag = torch.tensor([p.mig_mode == D.MIG_LAG for p in pols], device="cuda")
            any_lag = (srv & lag[:, None]).any(0)
            any_plain = (srv & ~lag[:, None]).any(0)
            m = torch.where(srv & lag[:, None], mg["mig_idx"], torch.full_like(mg["mig_idx"], -1)).max(0).values
            n = self.trace.output_len
            need = torch.where(any_plain, n, torch.where(any_lag, torch.where(m >= 0, torch.minimum(m + 1, n), n), torch.zeros_like(n)))
            return int(need.sum(dtype=torch.int64).item()), int((any_lag | any_plain).sum().item())

        def walk_roofline(self, name, reps):
            """The streaming token-walk kernel against the HBM roofline: algorithmic bytes per launch over the launch
            duration, HIP events around the kernel on its stream (taken inside the library)."""
            need, walked = self.must_read_tokens()
            mean_ms, min_ms = D.disco_time_token_walk(self.trace, self.cfg["tau"], self.cfg["kappa"], self.pols, self.ws, reps=reps)
            nbytes = 4.0 * need + WALK_BYTES_PER_REQUEST * self.N
            gbs = nbytes / (mean_ms * 1e-3) / 1e9
            traffic = measured_traffic("k_tl_walk", name)
            r = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                 "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": traffic, "kernel": "k_tl_walk",
                 "launch_us": round(mean_ms * 1e3, 2), "launch_us_min": round(min_ms * 1e3, 2),
                 "bytes_per_launch": nbytes, "token_events_read": need, "token_events_total": self.T,
                 "requests_walked": walked,
                 "per_unit": "4 B per token event that has to be read + 29 B per request (13 read, 16 written)"}
            if traffic is not None:
                r["traffic_over_algorithmic"] = round(traffic / nbytes, 3)
                r["traffic_within_10_percent"] = abs(traffic / nbytes - 1.0) <= 0.10
            return r

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

    def read_ceiling():
        """What this GPU sustains on a plain streaming read of 4 GiB (one read-and-reduce kernel)."""
        buf = torch.empty(READ_PROBE_BYTES // 4, dtype=torch.float32, device="cuda").fill_(1.0)
        out = torch.zeros(64, dtype=torch.int32, device="cuda")
        t = event_time(lambda: D.disco_read_probe(buf, out), 10)
        del buf
        torch.cuda.empty_cache()
        return {"GBs": round(READ_PROBE_BYTES / t / 1e9, 1), "bytes": READ_PROBE_BYTES,
                "frac_of_peak": round(READ_PROBE_BYTES / t / 1e9 / HBM_PEAK_GBS, 4), "kernel": "k_read_probe"}

    def dispatch_roofline(w, name, reps):
        """The fused dispatch-and-reduce pass (it runs once inside the budget search and once for an evaluation).  With
        many columns it is bound by vector arithmetic (OPS_PER_PAIR operations per pair against 12 B per request,
        independent of the number of columns); with one column by memory.  The timed call also launches the kernel
        that stages the policy table, so the figures are slightly conservative."""
        bytes_per_launch = 12.0 * w.N
        if w.idx == 3:
            one = [D.Policy(mode=D.MODE_D, l_th=-1, w_tail=0.6)]
            t_k = event_time(lambda: D.disco_eval_dispatch(w.trace, one, ws=w.ws, acc=w.acc), reps)
            pairs_per_launch = w.N
        else:
            t_k = event_time(lambda: D.disco_eval_dispatch(w.trace, w.pols, ws=w.ws, acc=w.acc), reps)
            pairs_per_launch = w.N * w.P
        gbs = bytes_per_launch / t_k / 1e9
        tops = OPS_PER_PAIR * pairs_per_launch / t_k / 1e12
        common = {"kernel": "k_dispatch_acc", "traffic": measured_traffic("k_dispatch_acc", name),
                  "launch_us": round(t_k * 1e6, 2), "pairs_per_s_in_kernel": pairs_per_launch / t_k}
        if w.idx == 3 or w.P == 1:
            return {"bound": "hbm", "achieved": round(gbs, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(gbs / HBM_PEAK_GBS, 4), **common}
        return {"bound": "alu", "achieved": round(tops, 3), "peak": round(ALU_PEAK_TOPS, 2), "unit": "Top/s",
                "frac": round(tops / ALU_PEAK_TOPS, 4), **common,
                "hbm": {"achieved": round(gbs, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4)}}

    def parse(name):
        buffer, stoch = name.endswith("buffer"), name.endswith("stoch")
        return int(name.replace("config", "").replace("buffer", "").replace("stoch", "")), buffer, stoch

    # ------------------------------------------------------------------ the headline workload
    idx, buffer, stoch = parse(args.workload)
    log(f"[bench] generating {args.workload} ...")
    w = Workload(idx, buffer=buffer, stoch=stoch)
    log(f"[bench] {args.workload}: N={w.N} P={w.P} T={w.T} gen {w.gen_s * 1e3:.1f} ms; timing {args.steps} steps")
    sec, host_sec = w.time_steps(args.steps, args.warmup)
    thr = w.throughput(sec)
    timelines = w.cfg["timelines"]
    if timelines:
        metric, unit, value = "token-events/s", "token-events/s", thr["token_events_per_s_raw"]
    else:
        metric, unit, value = "request x policy evaluations/s", "pairs/s", thr["pairs_per_s"]
    if timelines and not buffer:
        roofline = w.walk_roofline(args.workload, args.kernel_reps)
    else:
        roofline = dispatch_roofline(w, args.workload, args.kernel_reps)
    ceiling = read_ceiling()
    if roofline["bound"] == "hbm":
        roofline["read_ceiling"] = ceiling
        roofline["frac_of_read_ceiling"] = round(roofline["achieved"] / ceiling["GBs"], 4)

    result = {
        "metric": metric, "value": value, "unit": unit, "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": sec * 1e3, "host_ms_per_step": host_sec * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "n_req": w.N, "policy_columns": w.P, "token_events": w.T,
                   "step": "budget search + fused dispatch/reduce + TTFT order statistics"
                           + (" + token walk + per-column totals + TBT order statistics" if timelines else "")},
        **{k: v for k, v in thr.items()},
        "roofline": roofline,
    }
    if not args.no_graph and idx != 3 and not stoch:
        g_sec, g_same = w.time_graph_replay(args.steps)
        result["graph_replay"] = {"ms_per_step": g_sec * 1e3, "matches_eager_step": g_same,
                                  "what": "the step above captured once into a HIP graph and replayed (reported beside "
                                          "the eager step; `value` is the eager one)"}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_pre["one"]
        result["cpu_baseline_all_cores"] = cpu_pre["all"]

    # ------------------------------------------------------------------ the other workloads
    extras = {"read_ceiling": ceiling}
    for name in [e for e in args.extras.split(",") if e and e != args.workload]:
        if not name.startswith("config"):
            continue
        k, buffer, stoch = parse(name)
        del w
        torch.cuda.empty_cache()
        log(f"[bench] extra {name} ...")
        w = Workload(k, buffer=buffer, stoch=stoch)
        steps = 5 if k == 4 else 10
        s, hs = w.time_steps(steps, 1)
        ex = {"n_req": w.N, "policy_columns": w.P, "token_events": w.T, "ms_per_step": s * 1e3, "host_ms_per_step": hs * 1e3}
        ex.update(w.throughput(s))
        if not args.no_graph and not stoch and k != 3:
            g_sec, g_same = w.time_graph_replay(steps)
            ex["graph_replay_ms_per_step"] = g_sec * 1e3
            ex["graph_replay_matches_eager_step"] = g_same
        if w.cfg["timelines"] and not buffer:
            ex["roofline"] = w.walk_roofline(name, 10)
        elif not w.cfg["timelines"] and not stoch:
            ex["roofline"] = dispatch_roofline(w, name, args.kernel_reps)
        if k == 1 and not stoch:
            # closed-form policy solves (Alg. 3 and Alg. 2) for the budget grid: half the columns each
            half = max(1, w.P // 2)
            sspecs = [dict(mode=D.MODE_S, b=(j, max(half - 1, 1))) for j in range(half)] + \
                     [dict(mode=D.MODE_D, b=(j, max(half - 1, 1)), alpha=(1, 10)) for j in range(half)]
            spol = torch.zeros(len(sspecs) * 32, dtype=torch.uint8, device="cuda")
            sout = torch.zeros(len(sspecs) * D.binding.SOLVE_DTYPE.itemsize, dtype=torch.uint8, device="cuda")
            t_s = event_time(lambda: D.disco_solve_policy(w.trace, sspecs, ws=w.ws, pol_out=spol, out=sout), 10)
            ex["policy_solve"] = {"columns": len(sspecs), "ms": t_s * 1e3,
                                  "what": "length table + per-column plan + 4-pass multi-rank selection over the server TTFTs"}
            # the materialised dispatch variant (per-pair decision byte and TTFT written): the HBM-write-bound one
            dec = torch.empty((w.P, w.N), dtype=torch.uint8, device="cuda")
            ttft = torch.empty((w.P, w.N), dtype=torch.float32, device="cuda")
            # (the smaller of three measurements each: the difference of two short times is sensitive to a stray stall)
            t_fused = min(event_time(lambda: D.disco_eval_dispatch_static(w.trace, w.pols, w.acc), 10) for _ in range(3))
            t_mat = min(event_time(lambda: D.disco_eval_dispatch_static(w.trace, w.pols, w.acc, decision=dec, ttft=ttft), 10)
                        for _ in range(3))
            log(f"[bench] dispatch on the fixed scratch: fused {t_fused * 1e6:.1f} us, with per-pair outputs {t_mat * 1e6:.1f} us")
            mb = 5.0 * w.N * w.P + 12.0 * w.N
            t_k = t_mat - t_fused
            ex["materialised_dispatch"] = {"bound": "hbm", "kernel": "k_dispatch_mat", "bytes_per_launch": mb,
                                           "launch_us": t_k * 1e6 if t_k > 0 else None,
                                           "achieved_GBs": mb / t_k / 1e9 if t_k > 0 else None,
                                           "frac": mb / t_k / 1e9 / HBM_PEAK_GBS if t_k > 0 else None,
                                           "per_unit": "5 B written per pair (decision byte + TTFT) + 12 B read per request"}
            del dec, ttft
        if stoch:
            st = D.stats_to_host(w.step(), len(w.levels))
            ex["runs"] = w.runs
            ex["mean_ttft_by_level"] = [float(x) for x in st["mean_ttft"]]
            ex["p99_ttft_by_level"] = [float(x[1]) for x in st["ttft_q"]]
        if buffer:
            tau = w.cfg["tau"]
            t_tl = event_time(lambda: D.disco_eval_migration(w.trace, tau, w.cfg["kappa"], w.pols, ws=w.ws, acc=w.acc,
                                                             cost=w.cfg["cost"]), 5)
            ex["eval_migration_ms"] = t_tl * 1e3
            st = D.stats_to_host(w.step(), w.P)
            ex["migrated_requests"] = [int(x) for x in st["n_migrated"]]
            ex["mean_delay_num"] = [None if x != x else float(x) for x in st["mean_delay_num"]]
        if not args.no_cpu_baseline and not buffer and not stoch:
            ex["cpu_baseline"] = {a: b for a, b in cpu_baseline(k).items() if not a.startswith("_")}
        extras[name] = ex
        log(f"[bench] {name}: {json.dumps(ex)}")
    if idx == 4 and timelines and not buffer and "config4" not in extras:
        # recorded-trace ingest at the headline size: wall-clock fp64 timestamps -> relative arrays, 8 B read and 4 B
        # written per token event (+ 28 B per request); the timestamps are rebuilt from a resident trace
        del w
        torch.cuda.empty_cache()
        w = Workload(4)
        tr = w.trace
        base = torch.cumsum(torch.full((w.N,), 0.25, dtype=torch.float64, device="cuda"), 0) + 1.7e9
        first = base + tr.srv_ttft.double()
        t_token = torch.repeat_interleave(first, tr.output_len.long()) + tr.tok_arr.double()
        del first
        ing = {}
        t_in = event_time(lambda: ing.update(t=D.disco_ingest_trace(base, t_token, tr.tok_off, tr.prompt_len)), 3)
        gbi = (12.0 * w.T + 28.0 * w.N) / 1e9
        extras["ingest_config4"] = {"bound": "hbm", "kernel": "k_ingest", "launch_ms": t_in * 1e3,
                                    "achieved_GBs": gbi / t_in, "frac": gbi / t_in / HBM_PEAK_GBS}
        del t_token, ing, base
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


# Requests of each workload that the CPU baseline evaluates: the whole workload where the oracle finishes it in a
# few seconds, else its first requests (same generator and seed, so the same requests the GPU evaluates first).
CPU_SAMPLE = {0: 10_000, 1: 400_000, 2: 100_000, 3: 4_000_000, 4: 50_000}


def cpu_baseline(idx: int, n_sample: int | None = None, seed: int = 0) -> dict:
    """The oracle as it stands, on a bounded sample of the same workload, on one host core, in the workload's unit."""
    import numpy as np

    import disco_inputs as DI
    from oracle import disco_oracle as O

    n_sample = n_sample or CPU_SAMPLE[idx]
    cfg = DI.config(idx, n_req=n_sample, seed=seed)
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
    whole = n_sample == DI.config(idx)["gen"]["n_req"]
    sample = (f"all {n_sample} requests" if whole else f"first {n_sample} requests") + \
        f" of config{idx} (same generator and seed), same step, {dt:.1f} s"
    out = {"value": pairs / dt, "unit": "pairs/s", "cores": 1, "kind": "oracle", "sample": sample, "pairs_per_s": pairs / dt,
           "_pairs": pairs, "_tokens": int(tr["n_tok"]) if cfg["timelines"] else 0, "_seconds": dt}
    if cfg["timelines"]:
        out["value"], out["unit"] = int(tr["n_tok"]) / dt, "token-events/s"
    return out


def _cpu_worker(job):
    idx, n_sample, seed = job
    return cpu_baseline(idx, n_sample, seed)


def cpu_baseline_all_cores(idx: int) -> dict:
    """The same oracle step in one process per host core (at most 16), each on its own sample of the workload's recipe
    (seed = process number): what the host manages when every core evaluates a batch of its own.  Forks: call it
    before the GPU is initialised."""
    import multiprocessing as mp

    k = max(1, min(16, os.cpu_count() or 1))
    n_each = max(1, CPU_SAMPLE[idx] // 2)
    t0 = time.perf_counter()
    with mp.get_context("fork").Pool(k) as pool:
        parts = pool.map(_cpu_worker, [(idx, n_each, 1 + j) for j in range(k)])
    wall = time.perf_counter() - t0
    tokens, pairs = sum(p["_tokens"] for p in parts), sum(p["_pairs"] for p in parts)
    slowest = max(p["_seconds"] for p in parts)              # the processes run their steps side by side
    timelines = tokens > 0
    return {"value": (tokens if timelines else pairs) / slowest, "unit": "token-events/s" if timelines else "pairs/s", "cores": k,
            "kind": "oracle", "sample": f"{k} processes side by side, each the same step on {n_each} requests of config{idx}'s "
                                        f"recipe (seeds 1..{k}); slowest step {slowest:.1f} s, {wall:.1f} s wall with generating "
                                        f"the samples",
            "pairs_per_s": pairs / slowest}


if __name__ == "__main__":
    sys.exit(main())
