"""Thin ctypes binding of libdisco's C ABI (``include/disco.h``).

Argument marshalling only: every step of the evaluation runs in the library's
HIP kernels.  PyTorch is used for device memory and streams, nothing else.
The functions carry the names of the entry points they call.  There is no
CPU fallback: if the shared library is missing, importing fails.
"""
from __future__ import annotations

import ctypes as C
import math
import os
from dataclasses import dataclass, field

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdisco.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
        "or python paper_2502_11417_amd/build.py); there is no fallback path")

_lib = C.CDLL(LIB_PATH)

MAX_COLS, MAX_Q, MAX_STEPS = 64, 4, 64
GEN_REQUESTS, GEN_TOKENS = 1, 2
MODE_S, MODE_D, MODE_STOCH_S, MODE_STOCH_D = 0, 1, 2, 3
MIG_NONE, MIG_LAG, MIG_BUFFER = 0, 1, 2
PARAM_L_TH, PARAM_W_TAIL, PARAM_BETA = 0, 1, 2
ACC = {"total_cost": 0, "server_cost": 1, "device_cost": 2, "server_prefill_tok": 3, "device_prefill_tok": 4}
ERR = {"null": -1, "shape": -2, "range": -3, "csr": -4, "workspace": -5, "hip": -6}


class DiscoError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = _lib.disco_strerror(code).decode()
        if code == ERR["hip"]:
            msg += ": " + _lib.disco_last_hip_error().decode()
        super().__init__(f"{where}: {msg} ({code})")


# ------------------------------------------------------------- C structures

class CTrace(C.Structure):
    _fields_ = [("n_req", C.c_int64), ("n_tok", C.c_int64),
                ("prompt_len", C.c_void_p), ("output_len", C.c_void_p), ("srv_ttft", C.c_void_p),
                ("srv_tbt", C.c_void_p), ("dev_pre_spt", C.c_void_p), ("dev_dec_spt", C.c_void_p),
                ("tok_off", C.c_void_p), ("tok_arr", C.c_void_p),
                ("dev_pre_spt_s", C.c_float), ("dev_dec_spt_s", C.c_float), ("dev_ttft_c", C.c_float),
                ("reserved", C.c_float)]


class CGenParams(C.Structure):
    _fields_ = [("seed", C.c_uint64), ("n_req", C.c_int64),
                ("prompt_mu", C.c_float), ("prompt_sigma", C.c_float), ("prompt_lo", C.c_int32), ("prompt_hi", C.c_int32),
                ("out_mu", C.c_float), ("out_sigma", C.c_float), ("out_lo", C.c_int32), ("out_hi", C.c_int32),
                ("ttft_mu", C.c_float), ("ttft_sigma", C.c_float),
                ("ttft_pareto_p", C.c_float), ("ttft_pareto_xm", C.c_float), ("ttft_pareto_alpha", C.c_float),
                ("tbt_mu", C.c_float), ("tbt_sigma", C.c_float),
                ("dev_mode", C.c_int32), ("dev_a", C.c_float), ("dev_b", C.c_float), ("dev_p", C.c_float),
                ("dev_pre_ratio", C.c_float),
                ("gap_mu", C.c_float), ("gap_sigma", C.c_float),
                ("gap_stall_p", C.c_float), ("gap_stall_lo", C.c_float), ("gap_stall_hi", C.c_float)]


class CPolicy(C.Structure):
    _fields_ = [("mode", C.c_int32), ("l_th", C.c_int32), ("l_mid", C.c_int32), ("w_mid", C.c_float),
                ("beta", C.c_float), ("w_tail", C.c_float), ("mig_mode", C.c_int32), ("reserved", C.c_int32)]


class CCost(C.Structure):
    _fields_ = [("cs_pre", C.c_double), ("cs_dec", C.c_double), ("e_pre", C.c_double), ("e_dec", C.c_double),
                ("lam", C.c_double)]


class CTimeline(C.Structure):
    _fields_ = [("tau", C.c_float), ("kappa_lag", C.c_float), ("cost", C.POINTER(CCost)),
                ("reuse_walk", C.c_int32), ("reserved", C.c_int32)]


class CPairOut(C.Structure):
    _fields_ = [("decision", C.c_void_p), ("ttft", C.c_void_p)]


class CMigOut(C.Structure):
    _fields_ = [("mig_idx", C.c_void_p), ("n_src_tok", C.c_void_p), ("t_last", C.c_void_p),
                ("delivered", C.c_void_p), ("delivered_col", C.c_int32), ("reserved", C.c_int32),
                ("delay_num", C.c_void_p)]


class CQuantile(C.Structure):
    _fields_ = [("num", C.c_int32), ("den", C.c_int32)]


class CSearchSpec(C.Structure):
    _fields_ = [("which_param", C.c_int32), ("which_acc", C.c_int32), ("n_steps", C.c_int32),
                ("reserved", C.c_int32), ("lo", C.c_double), ("hi", C.c_double), ("target", C.c_double)]


class CSolveSpec(C.Structure):
    _fields_ = [("mode", C.c_int32), ("b_num", C.c_int32), ("b_den", C.c_int32), ("a_num", C.c_int32),
                ("a_den", C.c_int32), ("mig_mode", C.c_int32), ("reserved", C.c_int32 * 2)]


SOLVE_DTYPE = np.dtype([("rank_tail", "<i8"), ("rank_mid", "<i8"), ("zero_wait_tokens", "<i8"), ("total_tokens", "<i8"),
                        ("status", "<i4"), ("reserved", "<i4", (3,))])
ACCUM_DTYPE = np.dtype([
    ("s_pre", "<i8"), ("s_dec", "<i8"), ("d_pre", "<i8"), ("d_dec", "<i8"),
    ("n_dev_started", "<i8"), ("n_dev_win", "<i8"), ("ttft_sum", "<f8"),
    ("m_s_dec", "<i8"), ("m_d_dec", "<i8"), ("m_d_repre", "<i8"), ("n_migrated", "<i8"), ("tbt_count", "<i8"),
    ("tlast_sum", "<f8"),
    ("ttft_min_bits", "<u4"), ("ttft_max_bits", "<u4"), ("m_s_repre", "<i8"), ("delay_sum", "<i8")])
STATS_DTYPE = np.dtype([
    ("mean_ttft", "<f8"), ("mean_tbt", "<f8"),
    ("server_cost", "<f8"), ("device_energy", "<f8"), ("device_cost", "<f8"), ("total_cost", "<f8"),
    ("s_pre", "<i8"), ("s_dec", "<i8"), ("d_pre", "<i8"), ("d_dec", "<i8"),
    ("n_req", "<i8"), ("tbt_count", "<i8"), ("n_migrated", "<i8"), ("n_dev_started", "<i8"), ("n_dev_win", "<i8"),
    ("ttft_rank", "<i8", (MAX_Q,)), ("tbt_rank", "<i8", (MAX_Q,)),
    ("ttft_q", "<f4", (MAX_Q,)), ("tbt_q", "<f4", (MAX_Q,)), ("mean_delay_num", "<f8"),
    ("delay_q", "<f4", (MAX_Q,)), ("reserved", "<i8", (2,))])
SEARCH_DTYPE = np.dtype([
    ("param", "<f8"), ("acc_at_param", "<f8"), ("lo", "<f8"), ("hi", "<f8"),
    ("hist_param", "<f8", (MAX_STEPS,)), ("hist_acc", "<f8", (MAX_STEPS,)), ("at_param", ACCUM_DTYPE)])
POLICY_DTYPE = np.dtype([("mode", "<i4"), ("l_th", "<i4"), ("l_mid", "<i4"), ("w_mid", "<f4"), ("beta", "<f4"),
                         ("w_tail", "<f4"), ("mig_mode", "<i4"), ("reserved", "<i4")])
assert ACCUM_DTYPE.itemsize == 128 and STATS_DTYPE.itemsize == 256 and POLICY_DTYPE.itemsize == 32
assert C.sizeof(CPolicy) == 32 and C.sizeof(CSearchSpec) == 40

EXPORTS = ["disco_gen_trace", "disco_eval_dispatch", "disco_eval_dispatch_static", "disco_eval_migration", "disco_reduce_stats",
           "disco_average_runs", "disco_solve_policy", "disco_ingest_trace", "disco_fit_lognormal",
           "disco_device_profile", "disco_budget_search", "disco_read_probe", "disco_time_token_walk", "disco_validate_trace", "disco_set_grid_divisor", "disco_policy_type", "disco_workspace_bytes", "disco_strerror", "disco_last_hip_error",
           "disco_version"]

_lib.disco_strerror.restype = C.c_char_p
_lib.disco_strerror.argtypes = [C.c_int32]
_lib.disco_last_hip_error.restype = C.c_char_p
_lib.disco_version.restype = C.c_int32
_lib.disco_workspace_bytes.restype = C.c_size_t
_lib.disco_workspace_bytes.argtypes = [C.c_int64, C.c_int32]
_lib.disco_gen_trace.restype = C.c_int32
_lib.disco_gen_trace.argtypes = [C.POINTER(CGenParams), C.POINTER(CTrace), C.c_int32, C.c_void_p]
_lib.disco_eval_dispatch.restype = C.c_int32
_lib.disco_eval_dispatch.argtypes = [C.POINTER(CTrace), C.POINTER(CPolicy), C.c_int32, C.POINTER(CPairOut),
                                     C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
_lib.disco_eval_dispatch_static.restype = C.c_int32
_lib.disco_eval_dispatch_static.argtypes = [C.POINTER(CTrace), C.POINTER(CPolicy), C.c_int32, C.POINTER(CPairOut),
                                            C.c_void_p, C.c_void_p]
_lib.disco_eval_migration.restype = C.c_int32
_lib.disco_eval_migration.argtypes = [C.POINTER(CTrace), C.POINTER(CTimeline), C.POINTER(CPolicy), C.c_int32,
                                      C.POINTER(CMigOut), C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
_lib.disco_reduce_stats.restype = C.c_int32
_lib.disco_reduce_stats.argtypes = [C.POINTER(CTrace), C.POINTER(CCost), C.POINTER(CTimeline), C.POINTER(CPolicy),
                                    C.c_int32, C.c_void_p, C.POINTER(CQuantile), C.c_int32, C.c_void_p,
                                    C.c_void_p, C.c_size_t, C.c_void_p]
_lib.disco_average_runs.restype = C.c_int32
_lib.disco_average_runs.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
class CRawTrace(C.Structure):
    _fields_ = [("n_req", C.c_int64), ("n_tok", C.c_int64), ("t_send", C.c_void_p), ("t_token", C.c_void_p),
                ("tok_off", C.c_void_p)]


class CDevicePreset(C.Structure):
    _fields_ = [("prefill_tok_per_s", C.c_double), ("decode_tok_per_s", C.c_double), ("dev_pre_spt_s", C.c_float),
                ("dev_dec_spt_s", C.c_float), ("dev_ttft_c", C.c_float), ("name", C.c_char * 44)]


FIT_DTYPE = np.dtype([("mu", "<f8"), ("sigma", "<f8"), ("n_used", "<i8"), ("n_skipped", "<i8")])
_lib.disco_ingest_trace.restype = C.c_int32
_lib.disco_ingest_trace.argtypes = [C.POINTER(CRawTrace), C.POINTER(CTrace), C.c_void_p]
_lib.disco_fit_lognormal.restype = C.c_int32
_lib.disco_fit_lognormal.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
_lib.disco_device_profile.restype = C.c_int32
_lib.disco_device_profile.argtypes = [C.c_int32, C.POINTER(CDevicePreset)]
_lib.disco_solve_policy.restype = C.c_int32
_lib.disco_solve_policy.argtypes = [C.POINTER(CTrace), C.POINTER(CSolveSpec), C.c_int32, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_size_t, C.c_void_p]
_lib.disco_read_probe.restype = C.c_int32
_lib.disco_read_probe.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
_lib.disco_time_token_walk.restype = C.c_int32
_lib.disco_time_token_walk.argtypes = [C.POINTER(CTrace), C.POINTER(CTimeline), C.POINTER(CPolicy), C.c_int32, C.c_void_p,
                                       C.c_size_t, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_void_p]
_lib.disco_validate_trace.restype = C.c_int32
_lib.disco_validate_trace.argtypes = [C.POINTER(CTrace), C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
_lib.disco_set_grid_divisor.restype = C.c_int32
_lib.disco_set_grid_divisor.argtypes = [C.c_int32]
_lib.disco_policy_type.restype = C.c_int32
_lib.disco_policy_type.argtypes = [C.POINTER(CCost), C.POINTER(C.c_int32)]
_lib.disco_budget_search.restype = C.c_int32
_lib.disco_budget_search.argtypes = [C.POINTER(CTrace), C.POINTER(CCost), C.POINTER(CPolicy),
                                     C.POINTER(CSearchSpec), C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_size_t, C.c_void_p]


# ----------------------------------------------------------------- helpers

@dataclass
class Policy:
    mode: int = MODE_S
    l_th: int = 0
    l_mid: int = -1
    w_mid: float = 0.0
    beta: float = math.inf
    w_tail: float = math.inf
    mig_mode: int = MIG_NONE


@dataclass
class Trace:
    """Device-resident trace: torch tensors plus the scalars of ``disco_trace``."""
    n_req: int
    n_tok: int = 0
    prompt_len: torch.Tensor | None = None
    output_len: torch.Tensor | None = None
    srv_ttft: torch.Tensor | None = None
    srv_tbt: torch.Tensor | None = None
    dev_pre_spt: torch.Tensor | None = None
    dev_dec_spt: torch.Tensor | None = None
    tok_off: torch.Tensor | None = None
    tok_arr: torch.Tensor | None = None
    dev_pre_spt_s: float = 0.0
    dev_dec_spt_s: float = 0.0
    dev_ttft_c: float = 0.0
    _ws: dict = field(default_factory=dict, repr=False)

    def c_struct(self) -> CTrace:
        def p(t):
            return None if t is None else t.data_ptr()
        return CTrace(self.n_req, self.n_tok, p(self.prompt_len), p(self.output_len), p(self.srv_ttft),
                      p(self.srv_tbt), p(self.dev_pre_spt), p(self.dev_dec_spt), p(self.tok_off), p(self.tok_arr),
                      self.dev_pre_spt_s, self.dev_dec_spt_s, self.dev_ttft_c, 0.0)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(rc: int, where: str):
    if rc != 0:
        raise DiscoError(rc, where)


class DevicePolicies:
    """A policy table that already lives on the device (P records of 32 bytes)."""

    def __init__(self, buf: torch.Tensor, P: int):
        self.buf, self.P = buf, P

    def __len__(self):
        return self.P


def _policies(policies):
    if isinstance(policies, DevicePolicies):
        return C.cast(C.c_void_p(policies.buf.data_ptr()), C.POINTER(CPolicy))
    if isinstance(policies, C.Array):              # marshalled before (prepare_policies)
        return policies
    arr = (CPolicy * max(len(policies), 1))()
    for j, p in enumerate(policies):
        arr[j] = CPolicy(p.mode, p.l_th, p.l_mid, p.w_mid, p.beta, p.w_tail, p.mig_mode, 0)
    return arr


def prepare_policies(policies) -> C.Array:
    """The host policy table as the C array the entry points take; pass it instead of the list to skip the
    marshalling in a loop that calls with the same table."""
    return _policies(list(policies))


def prepare_specs(specs) -> C.Array:
    """Search specs (see ``disco_budget_search``) as a C array, for repeated calls."""
    sp = (CSearchSpec * max(len(specs), 1))()
    for j, s in enumerate(specs):
        wa = s["which_acc"]
        sp[j] = CSearchSpec(int(s["which_param"]), ACC[wa] if isinstance(wa, str) else int(wa), int(s["n_steps"]), 0,
                            float(s["lo"]), float(s["hi"]), float(s["target"]))
    return sp


def _cost(cost: dict) -> CCost:
    return CCost(cost["cs_pre"], cost["cs_dec"], cost["e_pre"], cost["e_dec"], cost["lam"])


def disco_workspace_bytes(n_req: int, P: int) -> int:
    return int(_lib.disco_workspace_bytes(n_req, P))


def workspace(n_req: int, P: int, device="cuda") -> torch.Tensor:
    return torch.empty(disco_workspace_bytes(n_req, P), dtype=torch.uint8, device=device)


def upload_trace(tr: dict, device="cuda") -> Trace:
    """Host arrays (numpy) of a trace -> device tensors."""
    def up(a, dt):
        return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dt)).to(device)
    has_tok = tr.get("tok_arr") is not None
    return Trace(
        n_req=int(tr["n_req"]), n_tok=int(tr.get("n_tok", 0)) if has_tok else 0,
        prompt_len=up(tr["prompt_len"], np.int32), output_len=up(tr["output_len"], np.int32),
        srv_ttft=up(tr["srv_ttft"], np.float32), srv_tbt=up(tr.get("srv_tbt"), np.float32),
        dev_pre_spt=up(tr.get("dev_pre_spt"), np.float32), dev_dec_spt=up(tr.get("dev_dec_spt"), np.float32),
        tok_off=up(tr.get("tok_off"), np.int64) if (has_tok or tr.get("tok_off") is not None) else None,
        tok_arr=up(tr.get("tok_arr"), np.float32),
        dev_pre_spt_s=float(tr.get("dev_pre_spt_s", 0.0)), dev_dec_spt_s=float(tr.get("dev_dec_spt_s", 0.0)),
        dev_ttft_c=float(tr.get("dev_ttft_c", 0.0)))


# ------------------------------------------------------------- entry points

def disco_gen_trace(gen: dict, tokens: bool | None = None, device="cuda") -> Trace:
    """Allocate the arrays of a synthetic trace and fill them on the device."""
    n = int(gen["n_req"])
    g = CGenParams()
    for name, _ in CGenParams._fields_:
        setattr(g, name, gen[name])
    t = Trace(n_req=n, dev_ttft_c=float(gen.get("dev_ttft_c", 0.0)))
    t.prompt_len = torch.empty(n, dtype=torch.int32, device=device)
    t.output_len = torch.empty(n, dtype=torch.int32, device=device)
    t.srv_ttft = torch.empty(n, dtype=torch.float32, device=device)
    t.srv_tbt = torch.empty(n, dtype=torch.float32, device=device)
    t.dev_pre_spt = torch.empty(n, dtype=torch.float32, device=device)
    t.dev_dec_spt = torch.empty(n, dtype=torch.float32, device=device)
    t.tok_off = torch.empty(n + 1, dtype=torch.int64, device=device)
    cs = t.c_struct()
    _check(_lib.disco_gen_trace(C.byref(g), C.byref(cs), GEN_REQUESTS, _stream()), "disco_gen_trace(requests)")
    total = int(cs.n_tok)
    if tokens is None:
        tokens = bool(gen.get("tokens", False))
    if tokens:
        t.n_tok = total
        t.tok_arr = torch.empty(total, dtype=torch.float32, device=device)
        cs = t.c_struct()
        _check(_lib.disco_gen_trace(C.byref(g), C.byref(cs), GEN_TOKENS, _stream()), "disco_gen_trace(tokens)")
    t._ws["n_tok_total"] = total
    return t


def disco_eval_dispatch(trace: Trace, policies, materialise: bool = False, ws: torch.Tensor | None = None,
                        acc: torch.Tensor | None = None) -> dict:
    P = len(policies)
    dev = trace.prompt_len.device if trace.prompt_len is not None else "cuda"
    if ws is None:
        ws = workspace(trace.n_req, P, dev)
    if acc is None:
        acc = torch.zeros(max(P, 1) * 128, dtype=torch.uint8, device=dev)
    out = None
    res = {"acc": acc}
    if materialise:
        res["decision"] = torch.empty((P, trace.n_req), dtype=torch.uint8, device=dev)
        res["ttft"] = torch.empty((P, trace.n_req), dtype=torch.float32, device=dev)
        out = CPairOut(res["decision"].data_ptr(), res["ttft"].data_ptr())
    cs = trace.c_struct()
    rc = _lib.disco_eval_dispatch(C.byref(cs), _policies(policies), P, C.byref(out) if out else None,
                                  acc.data_ptr(), ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "disco_eval_dispatch")
    return res


def disco_eval_dispatch_static(trace: Trace, policies, acc: torch.Tensor, decision: torch.Tensor | None = None,
                               ttft: torch.Tensor | None = None) -> None:
    """The dispatch pass on the library's fixed scratch area: no workspace, nothing allocated (the caller brings
    ``acc`` and, optionally, the [P][n_req] per-pair arrays)."""
    out = CPairOut(decision.data_ptr() if decision is not None else None, ttft.data_ptr() if ttft is not None else None)
    cs = trace.c_struct()
    rc = _lib.disco_eval_dispatch_static(C.byref(cs), _policies(policies), len(policies), C.byref(out), acc.data_ptr(),
                                         _stream())
    _check(rc, "disco_eval_dispatch_static")


def disco_eval_migration(trace: Trace, tau: float, kappa: float, policies, materialise: bool = False,
                         delivered_col: int | None = None, ws: torch.Tensor | None = None,
                         acc: torch.Tensor | None = None, cost: dict | None = None) -> dict:
    """``cost``: the rates behind the buffer hand-off's cost test (columns with ``MIG_BUFFER``); without
    them such columns never hand off."""
    P = len(policies)
    dev = trace.prompt_len.device if trace.prompt_len is not None else "cuda"
    if ws is None:
        ws = workspace(trace.n_req, P, dev)
    if acc is None:
        acc = torch.zeros(max(P, 1) * 128, dtype=torch.uint8, device=dev)
    res = {"acc": acc}
    out = CMigOut(None, None, None, None, 0, 0, None)
    if materialise:
        res["mig_idx"] = torch.empty((P, trace.n_req), dtype=torch.int32, device=dev)
        res["n_src_tok"] = torch.empty((P, trace.n_req), dtype=torch.int32, device=dev)
        res["t_last"] = torch.empty((P, trace.n_req), dtype=torch.float32, device=dev)
        res["delay_num"] = torch.empty((P, trace.n_req), dtype=torch.int32, device=dev)
        out.mig_idx, out.n_src_tok, out.t_last = (res["mig_idx"].data_ptr(), res["n_src_tok"].data_ptr(),
                                                  res["t_last"].data_ptr())
        out.delay_num = res["delay_num"].data_ptr()
    if delivered_col is not None:
        total = int(trace.tok_off[-1].item()) if trace.tok_off is not None else 0
        res["delivered"] = torch.empty(total, dtype=torch.float32, device=dev)
        out.delivered = res["delivered"].data_ptr()
        out.delivered_col = delivered_col
    cc = _cost(cost) if cost is not None else None
    tl = CTimeline(tau, kappa, C.pointer(cc) if cc is not None else None, 0, 0)
    cs = trace.c_struct()
    rc = _lib.disco_eval_migration(C.byref(cs), C.byref(tl), _policies(policies), P, C.byref(out),
                                   acc.data_ptr(), ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "disco_eval_migration")
    return res


def disco_reduce_stats(trace: Trace, cost: dict, policies, acc: torch.Tensor, quantiles=((50, 100), (99, 100)),
                       tau: float | None = None, kappa: float = 3.0, ws: torch.Tensor | None = None,
                       out: torch.Tensor | None = None, mig_cost: dict | None = None,
                       reuse_walk: bool = False) -> torch.Tensor:
    """Returns the device buffer of P ``disco_stats`` records (see ``stats_to_host``).  ``tau``, ``kappa`` and
    ``mig_cost`` must be the timeline parameters ``acc`` was accumulated with.  ``reuse_walk``: ``ws`` is the
    workspace ``disco_eval_migration`` just ran in, for the same trace, table and parameters."""
    P = len(policies)
    dev = acc.device
    if ws is None:
        ws = workspace(trace.n_req, P, dev)
    if out is None:
        out = torch.zeros(max(P, 1) * 256, dtype=torch.uint8, device=dev)
    q = (CQuantile * max(len(quantiles), 1))()
    for i, (num, den) in enumerate(quantiles):
        q[i] = CQuantile(num, den)
    mc = _cost(mig_cost) if mig_cost is not None else None
    tl = CTimeline(tau, kappa, C.pointer(mc) if mc is not None else None, 1 if reuse_walk else 0, 0) if tau is not None else None
    cs = trace.c_struct()
    cc = _cost(cost)
    rc = _lib.disco_reduce_stats(C.byref(cs), C.byref(cc), C.byref(tl) if tl else None, _policies(policies), P,
                                 acc.data_ptr(), q, len(quantiles), out.data_ptr(), ws.data_ptr(), ws.numel(),
                                 _stream())
    _check(rc, "disco_reduce_stats")
    return out


def disco_average_runs(stats: torch.Tensor, groups: int, runs: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """Mean over the ``runs`` consecutive columns of each of ``groups`` groups of ``disco_stats`` records."""
    if out is None:
        out = torch.zeros(max(groups, 1) * 256, dtype=torch.uint8, device=stats.device)
    _check(_lib.disco_average_runs(stats.data_ptr(), groups, runs, out.data_ptr(), _stream()), "disco_average_runs")
    return out


def disco_device_profile(index: int) -> dict:
    p = CDevicePreset()
    _check(_lib.disco_device_profile(index, C.byref(p)), "disco_device_profile")
    return {"name": p.name.decode(), "prefill_tok_per_s": p.prefill_tok_per_s, "decode_tok_per_s": p.decode_tok_per_s,
            "dev_pre_spt_s": p.dev_pre_spt_s, "dev_dec_spt_s": p.dev_dec_spt_s, "dev_ttft_c": p.dev_ttft_c}


def disco_ingest_trace(t_send: torch.Tensor, t_token: torch.Tensor, tok_off: torch.Tensor, prompt_len: torch.Tensor,
                       profile: dict | None = None) -> Trace:
    """Recorded timestamps (fp64 device tensors) -> a device-resident ``Trace``; prompt lengths and the device
    speeds (``disco_device_profile``) are supplied by the caller."""
    n, T = int(t_send.numel()), int(t_token.numel())
    dev = t_send.device
    t = Trace(n_req=n, n_tok=T, prompt_len=prompt_len, tok_off=tok_off)
    t.output_len = torch.empty(n, dtype=torch.int32, device=dev)
    t.srv_ttft = torch.empty(n, dtype=torch.float32, device=dev)
    t.tok_arr = torch.empty(T, dtype=torch.float32, device=dev)
    if profile:
        t.dev_pre_spt_s, t.dev_dec_spt_s, t.dev_ttft_c = profile["dev_pre_spt_s"], profile["dev_dec_spt_s"], profile["dev_ttft_c"]
    raw = CRawTrace(n, T, t_send.data_ptr(), t_token.data_ptr(), tok_off.data_ptr())
    cs = t.c_struct()
    _check(_lib.disco_ingest_trace(C.byref(raw), C.byref(cs), _stream()), "disco_ingest_trace")
    return t


def disco_fit_lognormal(x: torch.Tensor, ws: torch.Tensor | None = None, out: torch.Tensor | None = None) -> torch.Tensor:
    """mu, sigma of ln x for an int32 or float32 device tensor; returns the device record (see ``fit_to_host``)."""
    kind = {torch.int32: 0, torch.float32: 1}[x.dtype]
    if ws is None:
        ws = workspace(0, 1, x.device)
    if out is None:
        out = torch.zeros(FIT_DTYPE.itemsize, dtype=torch.uint8, device=x.device)
    _check(_lib.disco_fit_lognormal(x.data_ptr(), kind, x.numel(), out.data_ptr(), ws.data_ptr(), ws.numel(), _stream()),
           "disco_fit_lognormal")
    return out


def fit_to_host(out: torch.Tensor) -> np.ndarray:
    return np.frombuffer(out.cpu().numpy().tobytes(), dtype=FIT_DTYPE, count=1)[0]


def disco_solve_policy(trace: Trace, specs, ws: torch.Tensor | None = None, pol_out: torch.Tensor | None = None,
                       out: torch.Tensor | None = None) -> dict:
    """specs: dicts with mode, b = (num, den), alpha = (num, den) (Alg. 2 only), optional mig_mode."""
    n = len(specs)
    dev = trace.prompt_len.device if trace.prompt_len is not None else "cuda"
    if ws is None:
        ws = workspace(trace.n_req, max(n, 1), dev)
    sp = (CSolveSpec * max(n, 1))()
    for j, s in enumerate(specs):
        a = s.get("alpha", (0, 1))
        sp[j] = CSolveSpec(int(s["mode"]), int(s["b"][0]), int(s["b"][1]), int(a[0]), int(a[1]), int(s.get("mig_mode", 0)))
    if pol_out is None:
        pol_out = torch.zeros(max(n, 1) * 32, dtype=torch.uint8, device=dev)
    if out is None:
        out = torch.zeros(max(n, 1) * SOLVE_DTYPE.itemsize, dtype=torch.uint8, device=dev)
    cs = trace.c_struct()
    rc = _lib.disco_solve_policy(C.byref(cs), sp, n, pol_out.data_ptr(), out.data_ptr(), ws.data_ptr(), ws.numel(),
                                 _stream())
    _check(rc, "disco_solve_policy")
    return {"pol_out": pol_out, "policies": DevicePolicies(pol_out, n), "out": out}


def solve_to_host(out: torch.Tensor, n: int) -> np.ndarray:
    return np.frombuffer(out.cpu().numpy().tobytes(), dtype=SOLVE_DTYPE, count=n)


def disco_budget_search(trace: Trace, cost: dict, templates, specs, ws: torch.Tensor | None = None,
                        out: torch.Tensor | None = None, pol_out: torch.Tensor | None = None,
                        acc: torch.Tensor | None = None) -> dict:
    """specs: dicts with which_param, which_acc (names or ints), n_steps, lo, hi, target.  ``acc``: receives the
    accumulators at the found parameters (what ``disco_eval_dispatch`` would compute for them)."""
    n = len(templates)
    dev = trace.prompt_len.device if trace.prompt_len is not None else "cuda"
    if ws is None:
        ws = workspace(trace.n_req, n, dev)
    sp = specs if isinstance(specs, C.Array) else prepare_specs(specs)
    if out is None:
        out = torch.zeros(max(n, 1) * SEARCH_DTYPE.itemsize, dtype=torch.uint8, device=dev)
    if pol_out is None:
        pol_out = torch.zeros(max(n, 1) * 32, dtype=torch.uint8, device=dev)
    cs = trace.c_struct()
    cc = _cost(cost)
    rc = _lib.disco_budget_search(C.byref(cs), C.byref(cc), _policies(templates), sp, n, out.data_ptr(),
                                  pol_out.data_ptr(), acc.data_ptr() if acc is not None else None, ws.data_ptr(),
                                  ws.numel(), _stream())
    _check(rc, "disco_budget_search")
    return {"out": out, "pol_out": pol_out, "policies": DevicePolicies(pol_out, n)}


def disco_policy_type(cost: dict) -> int:
    """MODE_D or MODE_S from the unified cost rates (Alg. 1)."""
    cc, mode = _cost(cost), C.c_int32(-1)
    _check(_lib.disco_policy_type(C.byref(cc), C.byref(mode)), "disco_policy_type")
    return mode.value


def disco_validate_trace(trace: Trace, check_tokens: bool = True, ws: torch.Tensor | None = None) -> int:
    """0 if the trace's data are sound, else the (negative) code: ERR['csr'] or ERR['range'].  Other failures raise."""
    if ws is None:
        ws = torch.empty(256, dtype=torch.uint8, device=trace.prompt_len.device if trace.prompt_len is not None else "cuda")
    cs = trace.c_struct()
    rc = _lib.disco_validate_trace(C.byref(cs), 1 if check_tokens else 0, ws.data_ptr(), ws.numel(), _stream())
    if rc not in (0, ERR["csr"], ERR["range"]):
        _check(rc, "disco_validate_trace")
    return rc


def disco_time_token_walk(trace: Trace, tau: float, kappa: float, policies, ws: torch.Tensor, reps: int = 10) -> tuple:
    """(mean, minimum) duration in ms of the streaming token-walk kernel alone (HIP events; synchronises)."""
    tl = CTimeline(tau, kappa, None, 0, 0)
    cs = trace.c_struct()
    mean, best = C.c_double(0.0), C.c_double(0.0)
    rc = _lib.disco_time_token_walk(C.byref(cs), C.byref(tl), _policies(policies), len(policies), ws.data_ptr(), ws.numel(),
                                    reps, C.byref(mean), C.byref(best), _stream())
    _check(rc, "disco_time_token_walk")
    return mean.value, best.value


def disco_read_probe(buf: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """One streaming read-and-reduce pass over ``buf`` (measurement aid)."""
    if out is None:
        out = torch.zeros(64, dtype=torch.int32, device=buf.device)
    _check(_lib.disco_read_probe(buf.data_ptr(), buf.numel() * buf.element_size(), out.data_ptr(), _stream()), "disco_read_probe")
    return out


# ------------------------------------------------------- host-side parsing

def accum_to_host(acc: torch.Tensor, P: int) -> np.ndarray:
    return np.frombuffer(acc.cpu().numpy().tobytes(), dtype=ACCUM_DTYPE, count=P)


def stats_to_host(stats: torch.Tensor, P: int) -> np.ndarray:
    return np.frombuffer(stats.cpu().numpy().tobytes(), dtype=STATS_DTYPE, count=P)


def search_to_host(out: torch.Tensor, n: int) -> np.ndarray:
    return np.frombuffer(out.cpu().numpy().tobytes(), dtype=SEARCH_DTYPE, count=n)


def policies_to_host(pol_out: torch.Tensor, n: int):
    rec = np.frombuffer(pol_out.cpu().numpy().tobytes(), dtype=POLICY_DTYPE, count=n)
    return [Policy(int(r["mode"]), int(r["l_th"]), int(r["l_mid"]), float(r["w_mid"]), float(r["beta"]),
                   float(r["w_tail"]), int(r["mig_mode"])) for r in rec]
