"""ctypes/numpy front end of the CPU oracle (``disco_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Importable from ``tests/``, the smoke check and the
CPU-baseline leg of the benchmark; the GPU library and its Python binding never
import this module, and this module never imports them.

Only marshalling happens here, plus the final assembly of per-column
statistics from the exact totals the C code returns (means are quotients of
those totals; costs go through the C cost functions).
"""
from __future__ import annotations

import ctypes as C
import math
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "disco_oracle.c")
_LIB = os.path.join(_HERE, "libdisco_oracle.so")

GCC_FLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a second or two)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(["gcc", *GCC_FLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _GenCfg(C.Structure):
    _fields_ = [
        ("seed", C.c_uint64), ("n_req", C.c_int64),
        ("prompt_mu", C.c_float), ("prompt_sigma", C.c_float),
        ("prompt_lo", C.c_int32), ("prompt_hi", C.c_int32),
        ("out_mu", C.c_float), ("out_sigma", C.c_float),
        ("out_lo", C.c_int32), ("out_hi", C.c_int32),
        ("ttft_mu", C.c_float), ("ttft_sigma", C.c_float), ("ttft_pareto_p", C.c_float),
        ("ttft_pareto_xm", C.c_float), ("ttft_pareto_alpha", C.c_float),
        ("tbt_mu", C.c_float), ("tbt_sigma", C.c_float),
        ("dev_mode", C.c_int32), ("dev_a", C.c_float), ("dev_b", C.c_float),
        ("dev_p", C.c_float), ("dev_pre_ratio", C.c_float),
        ("gap_mu", C.c_float), ("gap_sigma", C.c_float), ("gap_stall_p", C.c_float),
        ("gap_stall_lo", C.c_float), ("gap_stall_hi", C.c_float),
    ]


class _Policy(C.Structure):
    _fields_ = [
        ("mode", C.c_int32), ("l_th", C.c_int32), ("l_mid", C.c_int32),
        ("w_mid", C.c_float), ("beta", C.c_float), ("w_tail", C.c_float),
        ("mig_mode", C.c_int32),
    ]


@dataclass
class Policy:
    """One policy column (see ``orc_policy`` in the C source)."""
    mode: int = 0
    l_th: int = 0
    l_mid: int = -1
    w_mid: float = 0.0
    beta: float = math.inf
    w_tail: float = math.inf
    mig_mode: int = 0


ACC = {"total_cost": 0, "server_cost": 1, "device_cost": 2,
       "server_prefill_tok": 3, "device_prefill_tok": 4}

_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_u23.restype = C.c_float
        _lib.orc_u23.argtypes = [C.c_uint32]
        for name in ("orc_ln", "orc_exp", "orc_cos2pi"):
            fn = getattr(_lib, name)
            fn.restype = C.c_float
            fn.argtypes = [C.c_float]
        _lib.orc_normal.restype = C.c_float
        _lib.orc_normal.argtypes = [C.c_uint32, C.c_uint32]
        _lib.orc_lognormal.restype = C.c_float
        _lib.orc_lognormal.argtypes = [C.c_uint32, C.c_uint32, C.c_float, C.c_float]
        _lib.orc_gen_gap.restype = C.c_float
        _lib.orc_device_ttft.restype = C.c_float
        _lib.orc_device_ttft.argtypes = [C.c_int32, C.c_float, C.c_float]
        _lib.orc_wait.restype = C.c_float
        _lib.orc_quantile.restype = C.c_int64
        _lib.orc_search_wait.restype = C.c_float
        _lib.orc_search_slope.restype = C.c_float
        _lib.orc_search_lth.restype = C.c_int32
        for name in ("orc_server_cost", "orc_device_energy", "orc_total_cost"):
            getattr(_lib, name).restype = C.c_double
        _lib.orc_server_cost.argtypes = [C.c_double, C.c_double, C.c_int64, C.c_int64]
        _lib.orc_device_energy.argtypes = [C.c_double, C.c_double, C.c_int64, C.c_int64]
        _lib.orc_total_cost.argtypes = [C.c_double] * 5 + [C.c_int64] * 4
    return _lib


def _ptr(a, ctype):
    if a is None:
        return None
    return a.ctypes.data_as(C.POINTER(ctype))


def _cfg(gen: dict) -> _GenCfg:
    g = _GenCfg()
    for name, _ in _GenCfg._fields_:
        setattr(g, name, gen[name])
    return g


def _pols(policies) -> C.Array:
    arr = (_Policy * len(policies))()
    for j, p in enumerate(policies):
        arr[j] = _Policy(p.mode, p.l_th, p.l_mid, p.w_mid, p.beta, p.w_tail, p.mig_mode)
    return arr


# ---------------------------------------------------------------- generator

def philox_raw(ctr, key) -> np.ndarray:
    c = (C.c_uint32 * 4)(*ctr)
    k = (C.c_uint32 * 2)(*key)
    out = (C.c_uint32 * 4)()
    lib().orc_philox_raw(c, k, out)
    return np.array(list(out), dtype=np.uint32)


def philox(seed: int, index: int, field: int) -> np.ndarray:
    out = (C.c_uint32 * 4)()
    lib().orc_philox(C.c_uint64(seed), C.c_uint64(index), C.c_uint32(field), out)
    return np.array(list(out), dtype=np.uint32)


def gen_requests(gen: dict) -> dict:
    """Per-request fields and CSR offsets of a synthetic trace."""
    n = int(gen["n_req"])
    tr = {
        "n_req": n,
        "prompt_len": np.empty(n, np.int32), "output_len": np.empty(n, np.int32),
        "srv_ttft": np.empty(n, np.float32), "srv_tbt": np.empty(n, np.float32),
        "dev_pre_spt": np.empty(n, np.float32), "dev_dec_spt": np.empty(n, np.float32),
        "tok_off": np.empty(n + 1, np.int64), "tok_arr": None,
        "dev_pre_spt_s": 0.0, "dev_dec_spt_s": 0.0, "dev_ttft_c": float(gen.get("dev_ttft_c", 0.0)),
    }
    g = _cfg(gen)
    lib().orc_gen_requests(C.byref(g), _ptr(tr["prompt_len"], C.c_int32),
                           _ptr(tr["output_len"], C.c_int32), _ptr(tr["srv_ttft"], C.c_float),
                           _ptr(tr["srv_tbt"], C.c_float), _ptr(tr["dev_pre_spt"], C.c_float),
                           _ptr(tr["dev_dec_spt"], C.c_float), _ptr(tr["tok_off"], C.c_int64))
    tr["n_tok"] = int(tr["tok_off"][-1])
    return tr


def gen_tokens(gen: dict, tok_off: np.ndarray, req_lo: int = 0, req_hi: int | None = None) -> np.ndarray:
    """Server arrival offsets of requests [req_lo, req_hi), first element =
    global token index tok_off[req_lo]."""
    if req_hi is None:
        req_hi = len(tok_off) - 1
    base = int(tok_off[req_lo])
    out = np.empty(int(tok_off[req_hi]) - base, np.float32)
    g = _cfg(gen)
    lib().orc_gen_tokens(C.byref(g), _ptr(tok_off, C.c_int64), C.c_int64(req_lo),
                         C.c_int64(req_hi), C.c_int64(base), _ptr(out, C.c_float))
    return out


def gen_trace(gen: dict, tokens: bool | None = None) -> dict:
    tr = gen_requests(gen)
    if tokens is None:
        tokens = bool(gen.get("tokens", False))
    if tokens:
        tr["tok_arr"] = gen_tokens(gen, tr["tok_off"])
    return tr


# ----------------------------------------------------------------- dispatch

def device_ttft(l: int, k: float, c: float) -> float:
    return float(lib().orc_device_ttft(int(l), C.c_float(k), C.c_float(c)))


def _trace_args(tr):
    return dict(
        N=C.c_int64(tr["n_req"]),
        l=_ptr(tr["prompt_len"], C.c_int32), s=_ptr(tr["srv_ttft"], C.c_float),
        n=_ptr(tr["output_len"], C.c_int32),
        k=_ptr(tr.get("dev_pre_spt"), C.c_float), ks=C.c_float(tr.get("dev_pre_spt_s", 0.0)),
        c=C.c_float(tr.get("dev_ttft_c", 0.0)),
    )


def dispatch(tr: dict, policies, materialise: bool = True) -> dict:
    a = _trace_args(tr)
    N, P = tr["n_req"], len(policies)
    decision = np.empty((P, N), np.uint8) if materialise else None
    ttft = np.empty((P, N), np.float32) if materialise else None
    tok = np.zeros((P, 4), np.int64)
    cnt = np.zeros((P, 2), np.int64)
    ttft_sum = np.zeros(P, np.float64)
    lib().orc_dispatch(a["N"], C.c_int32(P), a["l"], a["s"], a["n"], a["k"], a["ks"], a["c"],
                       _pols(policies), _ptr(decision, C.c_uint8), _ptr(ttft, C.c_float),
                       _ptr(tok, C.c_int64), _ptr(ttft_sum, C.c_double), _ptr(cnt, C.c_int64))
    return {"decision": decision, "ttft": ttft, "s_pre": tok[:, 0].copy(), "s_dec": tok[:, 1].copy(),
            "d_pre": tok[:, 2].copy(), "d_dec": tok[:, 3].copy(), "ttft_sum": ttft_sum,
            "n_dev_started": cnt[:, 0].copy(), "n_dev_win": cnt[:, 1].copy()}


# ---------------------------------------------------------------- timelines

def timeline(n, r_srv, gap_const, src_is_device, lag_mode, tau, kappa, l, k, c, g_dev):
    """One request: (mig_idx, t_last, delivered[n], tbt[n-1])."""
    r = None if r_srv is None else np.ascontiguousarray(r_srv, np.float32)
    delivered = np.empty(n, np.float32)
    tbt = np.empty(max(n - 1, 0), np.float32)
    m = C.c_int32()
    tl = C.c_float()
    lib().orc_timeline(C.c_int32(n), _ptr(r, C.c_float), C.c_float(gap_const),
                       C.c_int32(int(src_is_device)), C.c_int32(int(lag_mode)), C.c_float(tau),
                       C.c_float(kappa), C.c_int32(l), C.c_float(k), C.c_float(c), C.c_float(g_dev),
                       C.byref(m), C.byref(tl), _ptr(delivered, C.c_float), _ptr(tbt, C.c_float))
    return m.value, tl.value, delivered, tbt


def timeline_buffer(n, r_srv, gap_srv, src_is_device, dc, cp, srv_ttft, tau, l, k, c, g_dev):
    """One request with the buffer hand-off: (mig_last, delay_num, t_last, delivered[n], tbt[n-1])."""
    r = None if r_srv is None else np.ascontiguousarray(r_srv, np.float32)
    delivered = np.empty(n, np.float32)
    tbt = np.empty(max(n - 1, 0), np.float32)
    m = C.c_int32()
    dn = C.c_int32()
    tl = C.c_float()
    lib().orc_timeline_buffer(C.c_int32(n), _ptr(r, C.c_float), C.c_float(gap_srv), C.c_int32(int(src_is_device)),
                              C.c_double(dc), C.c_double(cp), C.c_float(srv_ttft), C.c_float(tau), C.c_int32(l),
                              C.c_float(k), C.c_float(c), C.c_float(g_dev), C.byref(m), C.byref(dn), C.byref(tl),
                              _ptr(delivered, C.c_float), _ptr(tbt, C.c_float))
    return m.value, dn.value, tl.value, delivered, tbt


def migration(tr: dict, policies, tau: float, kappa: float, materialise: bool = True,
              tbt_col: int = -1, want_delivered: bool = False, cost: dict | None = None) -> dict:
    """``cost`` (rates) is needed by columns with the buffer hand-off (mig_mode 2)."""
    a = _trace_args(tr)
    N, P = tr["n_req"], len(policies)
    mig_idx = np.empty((P, N), np.int32) if materialise else None
    n_src = np.empty((P, N), np.int32) if materialise else None
    t_last = np.empty((P, N), np.float32) if materialise else None
    delay_num = np.empty((P, N), np.int32) if materialise else None
    mtok = np.zeros((P, 4), np.int64)
    cnt = np.zeros((P, 3), np.int64)
    tlast_sum = np.zeros(P, np.float64)
    n_total = int(np.sum(tr["output_len"], dtype=np.int64))
    tbt_out = np.empty(max(n_total - N, 0), np.float32) if tbt_col >= 0 else None
    delivered = np.empty(n_total, np.float32) if (tbt_col >= 0 and want_delivered) else None
    rates = _rates(cost) if cost is not None else None
    lib().orc_migration(a["N"], C.c_int32(P), a["l"], a["s"], a["n"], _ptr(tr.get("srv_tbt"), C.c_float),
                        a["k"], a["ks"], _ptr(tr.get("dev_dec_spt"), C.c_float),
                        C.c_float(tr.get("dev_dec_spt_s", 0.0)), a["c"],
                        _ptr(tr.get("tok_off"), C.c_int64) if tr.get("tok_arr") is not None else None,
                        _ptr(tr.get("tok_arr"), C.c_float), _pols(policies), C.c_float(tau),
                        C.c_float(kappa), rates, _ptr(mig_idx, C.c_int32), _ptr(n_src, C.c_int32),
                        _ptr(t_last, C.c_float), _ptr(delay_num, C.c_int32), _ptr(mtok, C.c_int64),
                        _ptr(cnt, C.c_int64), _ptr(tlast_sum, C.c_double), C.c_int32(tbt_col),
                        _ptr(tbt_out, C.c_float), _ptr(delivered, C.c_float))
    return {"mig_idx": mig_idx, "n_src_tok": n_src, "t_last": t_last, "delay_num": delay_num,
            "m_s_dec": mtok[:, 0].copy(), "m_d_dec": mtok[:, 1].copy(), "m_d_repre": mtok[:, 2].copy(),
            "m_s_repre": mtok[:, 3].copy(),
            "n_migrated": cnt[:, 0].copy(), "tbt_count": cnt[:, 1].copy(), "delay_sum": cnt[:, 2].copy(),
            "tlast_sum": tlast_sum, "tbt": tbt_out, "delivered": delivered}


# --------------------------------------------------------------- statistics

def quantile(values: np.ndarray, num: int, den: int):
    """Nearest-rank order statistic: (rank, value)."""
    v = np.ascontiguousarray(values, np.float32)
    out = C.c_float()
    k = lib().orc_quantile(_ptr(v, C.c_float), C.c_int64(v.size), C.c_int64(num), C.c_int64(den),
                           C.byref(out))
    return int(k), np.float32(out.value)


def total_cost(cost: dict, s_pre, s_dec, d_pre, d_dec) -> float:
    return float(lib().orc_total_cost(cost["cs_pre"], cost["cs_dec"], cost["e_pre"], cost["e_dec"],
                                      cost["lam"], int(s_pre), int(s_dec), int(d_pre), int(d_dec)))


def policy_type(cost: dict) -> int:
    """Alg. 1: device-constrained (1) if both device token costs exceed both server token costs, else
    server-constrained (0).  Device costs in money: lambda times the energy per token (Sec. 4.1)."""
    cd_p, cd_d = cost["lam"] * cost["e_pre"], cost["lam"] * cost["e_dec"]
    if min(cd_p, cd_d) > max(cost["cs_pre"], cost["cs_dec"]):
        return 1
    return 0


def server_cost(cost: dict, s_pre, s_dec) -> float:
    return float(lib().orc_server_cost(cost["cs_pre"], cost["cs_dec"], int(s_pre), int(s_dec)))


def device_energy(cost: dict, d_pre, d_dec) -> float:
    return float(lib().orc_device_energy(cost["e_pre"], cost["e_dec"], int(d_pre), int(d_dec)))


def stats(tr: dict, policies, cost: dict, quantiles=((50, 100), (99, 100)),
          tau: float | None = None, kappa: float = 3.0) -> list:
    """Per-column statistics.  With ``tau`` given, token timelines are
    evaluated too (TBT statistics, migration-aware decode accounting)."""
    dp = dispatch(tr, policies, materialise=True)
    N = tr["n_req"]
    out = []
    for j, _ in enumerate(policies):
        st = {"n_req": N, "s_pre": int(dp["s_pre"][j]), "d_pre": int(dp["d_pre"][j]),
              "s_dec": int(dp["s_dec"][j]), "d_dec": int(dp["d_dec"][j]),
              "n_dev_started": int(dp["n_dev_started"][j]), "n_dev_win": int(dp["n_dev_win"][j]),
              "mean_ttft": float(dp["ttft_sum"][j]) / N if N else math.nan,
              "ttft_rank": [], "ttft_q": [], "tbt_rank": [], "tbt_q": [],
              "n_migrated": 0, "tbt_count": 0, "mean_tbt": math.nan}
        for num, den in quantiles:
            k, v = quantile(dp["ttft"][j], num, den)
            st["ttft_rank"].append(k)
            st["ttft_q"].append(v)
        if tau is not None:
            mg = migration(tr, [policies[j]], tau, kappa, materialise=True, tbt_col=0, cost=cost)
            st["s_dec"] = int(mg["m_s_dec"][0])
            st["d_dec"] = int(mg["m_d_dec"][0])
            st["d_pre"] += int(mg["m_d_repre"][0])
            st["s_pre"] += int(mg["m_s_repre"][0])
            st["delay_sum"] = int(mg["delay_sum"][0])
            st["n_migrated"] = int(mg["n_migrated"][0])
            st["tbt_count"] = int(mg["tbt_count"][0])
            st["mean_tbt"] = (float(mg["tlast_sum"][0]) / st["tbt_count"]
                              if st["tbt_count"] else math.nan)
            for num, den in quantiles:
                k, v = quantile(mg["tbt"], num, den)
                st["tbt_rank"].append(k)
                st["tbt_q"].append(v)
            # delayed tokens per migrated request (TBT table of Sec. 5.2: mean and P99 delay_num over the requests
            # that migrated); nearest-rank order statistic like the others
            delays = mg["delay_num"][0][mg["mig_idx"][0] >= 0].astype(np.float32)
            st["delay_q"] = [quantile(delays, num, den)[1] for num, den in quantiles]
        st["server_cost"] = server_cost(cost, st["s_pre"], st["s_dec"])
        st["device_energy"] = device_energy(cost, st["d_pre"], st["d_dec"])
        st["device_cost"] = cost["lam"] * st["device_energy"]
        st["total_cost"] = total_cost(cost, st["s_pre"], st["s_dec"], st["d_pre"], st["d_dec"])
        out.append(st)
    return out


def average_runs(stats_list: list, runs: int) -> list:
    """Mean over runs (Sec. 5.1: results are reported as the mean over 10 runs): consecutive groups of ``runs``
    records of ``stats``; floating-point fields averaged in fp64 in run order (order statistics rounded back to
    fp32), integer totals summed, ranks of the first run."""
    assert runs >= 1 and len(stats_list) % runs == 0
    out = []
    for g in range(len(stats_list) // runs):
        grp = stats_list[g * runs:(g + 1) * runs]
        o = {}
        for f in ("mean_ttft", "mean_tbt", "server_cost", "device_energy", "device_cost", "total_cost"):
            acc = 0.0
            for st in grp:
                acc += float(st[f])
            o[f] = acc / runs
        acc = 0.0
        for st in grp:                                          # delayed tokens per migrated request (NaN without hand-offs)
            acc += st.get("delay_sum", 0) / st["n_migrated"] if st["n_migrated"] else math.nan
        o["mean_delay_num"] = acc / runs
        for f in ("s_pre", "s_dec", "d_pre", "d_dec", "n_req", "tbt_count", "n_migrated", "n_dev_started", "n_dev_win"):
            o[f] = sum(int(st[f]) for st in grp)
        for f in ("ttft_rank", "tbt_rank"):
            o[f] = list(grp[0][f])
        for f in ("ttft_q", "tbt_q"):
            o[f] = []
            for qi in range(len(grp[0][f])):
                acc = 0.0
                for st in grp:
                    acc += float(np.float32(st[f][qi]))
                o[f].append(np.float32(acc / runs))
        out.append(o)
    return out


# ------------------------------------------------------------ budget search

def _rates(cost: dict):
    return (C.c_double * 5)(cost["cs_pre"], cost["cs_dec"], cost["e_pre"], cost["e_dec"], cost["lam"])


def search_wait(tr: dict, templ: Policy, lo: float, hi: float, n_steps: int, which: str,
                cost: dict, target: float):
    a = _trace_args(tr)
    hp = np.zeros(n_steps, np.float32)
    ha = np.zeros(n_steps, np.float64)
    w = lib().orc_search_wait(a["N"], a["l"], a["s"], a["n"], a["k"], a["ks"], a["c"],
                              _pols([templ]), C.c_float(lo), C.c_float(hi), C.c_int32(n_steps),
                              C.c_int32(ACC[which]), _rates(cost), C.c_double(target),
                              _ptr(hp, C.c_float), _ptr(ha, C.c_double))
    return np.float32(w), hp, ha


def search_slope(tr: dict, templ: Policy, lo: float, hi: float, n_steps: int, which: str,
                 cost: dict, target: float):
    """Bisection on the ramp slope beta of Eq. 1 (the root of Eq. 2 on the trace)."""
    a = _trace_args(tr)
    hp = np.zeros(n_steps, np.float32)
    ha = np.zeros(n_steps, np.float64)
    b = lib().orc_search_slope(a["N"], a["l"], a["s"], a["n"], a["k"], a["ks"], a["c"],
                               _pols([templ]), C.c_float(lo), C.c_float(hi), C.c_int32(n_steps),
                               C.c_int32(ACC[which]), _rates(cost), C.c_double(target),
                               _ptr(hp, C.c_float), _ptr(ha, C.c_double))
    return np.float32(b), hp, ha


def search_lth(tr: dict, templ: Policy, lo: int, hi: int, n_steps: int, which: str,
               cost: dict, target: float):
    a = _trace_args(tr)
    hp = np.zeros(n_steps, np.int32)
    ha = np.zeros(n_steps, np.float64)
    l_th = lib().orc_search_lth(a["N"], a["l"], a["s"], a["n"], a["k"], a["ks"], a["c"],
                                _pols([templ]), C.c_int32(lo), C.c_int32(hi), C.c_int32(n_steps),
                                C.c_int32(ACC[which]), _rates(cost), C.c_double(target),
                                _ptr(hp, C.c_int32), _ptr(ha, C.c_double))
    return int(l_th), hp, ha
