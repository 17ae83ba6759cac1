"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function the public header declares, keeps the documented struct sizes,
and rejects bad arguments before anything is launched."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "disco.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(disco_[a-z_]+)\s*\(", text)))


def test_every_declared_function_is_exported(B):
    names = declared_functions()
    assert {"disco_gen_trace", "disco_eval_dispatch", "disco_eval_migration", "disco_reduce_stats",
            "disco_budget_search"} <= set(names)
    lib = C.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names


def test_struct_sizes_match_the_header(B):
    assert C.sizeof(B.CPolicy) == 32
    assert B.ACCUM_DTYPE.itemsize == 128 and B.STATS_DTYPE.itemsize == 256
    assert C.sizeof(B.CTrace) == 96
    assert B.disco_workspace_bytes(1000, 64) >= 1 << 20
    assert B._lib.disco_version() >= 100


def test_struct_layouts_match_a_c_compiler(B, tmp_path):
    """sizeof / offsetof as gcc sees the public header against the binding's ctypes and numpy records."""
    import subprocess
    probes = [("disco_timeline_params", ["tau", "kappa_lag", "cost", "reuse_walk"], B.CTimeline),
              ("disco_mig_out", ["mig_idx", "n_src_tok", "t_last", "delivered", "delivered_col", "delay_num"], B.CMigOut),
              ("disco_accum", ["m_s_dec", "tlast_sum", "ttft_min_bits", "m_s_repre", "delay_sum"], B.ACCUM_DTYPE),
              ("disco_stats", ["mean_tbt", "ttft_rank", "tbt_q", "mean_delay_num"], B.STATS_DTYPE),
              ("disco_policy", ["mode", "w_tail", "mig_mode"], B.CPolicy)]
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "disco.h"', 'int main(void) {']
    for name, fields, _ in probes:
        lines.append(f'printf("%zu", sizeof({name}));')
        for f in fields:
            lines.append(f'printf(" %zu", offsetof({name}, {f}));')
        lines.append('printf("\\n");')
    lines += ['return 0; }']
    src = tmp_path / "probe.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "probe"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.strip().splitlines()
    for (name, fields, rec), line in zip(probes, out):
        want = [int(x) for x in line.split()]
        if isinstance(rec, type) and issubclass(rec, C.Structure):
            got = [C.sizeof(rec)] + [getattr(rec, f).offset for f in fields]
        else:
            got = [rec.itemsize] + [rec.fields[f][1] for f in fields]
        assert got == want, (name, got, want)


def test_error_strings(B):
    for code in (0, -1, -2, -3, -4, -5, -6, -99):
        assert len(B._lib.disco_strerror(code)) > 0


def test_bad_arguments_are_rejected_on_the_host(B):
    lib = B._lib
    tr = B.CTrace()
    tr.n_req = 0
    pol = (B.CPolicy * 1)(B.CPolicy(0, 0, -1, 0.0, float("inf"), float("inf"), 0, 0))
    # null trace / null accumulators / bad column count / missing workspace
    assert lib.disco_eval_dispatch(None, pol, 1, None, None, None, 0, None) == B.ERR["null"]
    assert lib.disco_eval_dispatch(C.byref(tr), pol, 1, None, None, None, 0, None) == B.ERR["null"]
    assert lib.disco_eval_dispatch(C.byref(tr), pol, 0, None, 8, None, 0, None) == B.ERR["shape"]
    assert lib.disco_eval_dispatch(C.byref(tr), pol, 65, None, 8, None, 0, None) == B.ERR["shape"]
    assert lib.disco_eval_dispatch(C.byref(tr), pol, 1, None, 256, None, 0, None) == B.ERR["workspace"]
    assert lib.disco_eval_dispatch(C.byref(tr), pol, 1, None, 256, 256, 16, None) == B.ERR["workspace"]
    bad = (B.CPolicy * 1)(B.CPolicy(7, 0, -1, 0.0, 1.0, 1.0, 0, 0))
    assert lib.disco_eval_dispatch(C.byref(tr), bad, 1, None, 256, 256, 1 << 30, None) == B.ERR["range"]
    for b in (1.5, -0.1, float("inf")):                                      # routing probability of a stochastic baseline
        bad = (B.CPolicy * 1)(B.CPolicy(2, 0, 0, 0.0, b, 0.0, 0, 0))
        assert lib.disco_eval_dispatch(C.byref(tr), bad, 1, None, 256, 256, 1 << 30, None) == B.ERR["range"]
    bad = (B.CPolicy * 1)(B.CPolicy(4, 0, -1, 0.0, 1.0, 1.0, 0, 0))          # unknown mode
    assert lib.disco_eval_dispatch(C.byref(tr), bad, 1, None, 256, 256, 1 << 30, None) == B.ERR["range"]
    bad = (B.CPolicy * 1)(B.CPolicy(0, 0, -1, 0.0, 1.0, 1.0, 3, 0))          # unknown migration mode
    assert lib.disco_eval_dispatch(C.byref(tr), bad, 1, None, 256, 256, 1 << 30, None) == B.ERR["range"]
    tr.n_req = -1
    assert lib.disco_eval_dispatch(C.byref(tr), pol, 1, None, 256, 256, 1 << 30, None) == B.ERR["shape"]
    tr.n_req = 5          # arrays missing
    assert lib.disco_eval_dispatch(C.byref(tr), pol, 1, None, 256, 256, 1 << 30, None) == B.ERR["null"]
    tr.n_req = 0
    tl = B.CTimeline(0.0, 3.0, None, 0, 0)
    assert lib.disco_eval_migration(C.byref(tr), C.byref(tl), pol, 1, None, 256, 256, 1 << 30, None) == B.ERR["range"]
    q = (B.CQuantile * 1)(B.CQuantile(3, 2))
    cost = B.CCost(1, 1, 1, 1, 1)
    assert lib.disco_reduce_stats(C.byref(tr), C.byref(cost), None, pol, 1, 256, q, 1, 256, 256, 1 << 30, None) == B.ERR["range"]
    assert lib.disco_reduce_stats(C.byref(tr), C.byref(cost), None, pol, 1, 256, q, 9, 256, 256, 1 << 30, None) == B.ERR["shape"]
    spec = (B.CSearchSpec * 1)(B.CSearchSpec(1, 2, 0, 0, 0.0, 5.0, 1.0))
    assert lib.disco_budget_search(C.byref(tr), C.byref(cost), pol, spec, 1, 256, None, None, 256, 1 << 30, None) == B.ERR["shape"]
    spec[0].n_steps = 4
    stoch = (B.CPolicy * 1)(B.CPolicy(2, 0, 0, 0.0, 0.5, 0.0, 0, 0))         # a stochastic baseline has nothing to search
    assert lib.disco_budget_search(C.byref(tr), C.byref(cost), stoch, spec, 1, 256, None, None, 256, 1 << 30, None) == B.ERR["range"]
    assert lib.disco_average_runs(None, 1, 1, 256, None) == B.ERR["null"]
    assert lib.disco_average_runs(256, 1, 0, 256, None) == B.ERR["shape"]
    spec[0].lo = 6.0
    assert lib.disco_budget_search(C.byref(tr), C.byref(cost), pol, spec, 1, 256, None, None, 256, 1 << 30, None) == B.ERR["range"]
    g = B.CGenParams()
    assert lib.disco_gen_trace(None, None, 1, None) == B.ERR["null"]
    g.n_req = -3
    tr.n_req = -3
    assert lib.disco_gen_trace(C.byref(g), C.byref(tr), 1, None) == B.ERR["shape"]


def test_device_profiles_match_the_printed_speeds(B):
    """Host-only entry point: the three on-device configurations of Sec. 5.1 (golden file) as seconds per token."""
    import numpy as np
    rows = [ln.split("|") for ln in open(os.path.join(ROOT, "tests", "golden", "device_profiles.txt"))
            if ln.strip() and not ln.startswith("#")]
    for idx, (dev, model, pre, dec) in enumerate(rows):
        p = B.disco_device_profile(idx)
        assert dev.strip() in p["name"] and model.strip() in p["name"]
        assert p["prefill_tok_per_s"] == float(pre) and p["decode_tok_per_s"] == float(dec)
        assert np.float32(p["dev_pre_spt_s"]) == np.float32(1.0 / float(pre))
        assert np.float32(p["dev_dec_spt_s"]) == np.float32(1.0 / float(dec)) and p["dev_ttft_c"] == 0.0
    p = B.CDevicePreset()
    assert B._lib.disco_device_profile(3, C.byref(p)) == B.ERR["range"]
    assert B._lib.disco_device_profile(0, None) == B.ERR["null"]
    assert B._lib.disco_fit_lognormal(None, 0, 5, 256, 256, 1 << 30, None) == B.ERR["null"]
    assert B._lib.disco_fit_lognormal(256, 7, 5, 256, 256, 1 << 30, None) == B.ERR["range"]
    assert B._lib.disco_ingest_trace(None, None, None) == B.ERR["null"]


def test_new_entry_points_reject_bad_arguments_on_the_host(B):
    """disco_validate_trace, disco_time_token_walk, disco_read_probe, disco_policy_type, disco_set_grid_divisor:
    everything that can be refused without touching a GPU is refused before anything is launched."""
    import disco_inputs as DI
    lib = B._lib
    tr = B.CTrace()
    # validation
    assert lib.disco_validate_trace(None, 1, 256, 256, None) == B.ERR["null"]
    tr.n_req = -1
    assert lib.disco_validate_trace(C.byref(tr), 1, 256, 256, None) == B.ERR["shape"]
    tr.n_req = 4
    assert lib.disco_validate_trace(C.byref(tr), 1, 256, 256, None) == B.ERR["null"]            # arrays missing
    tr.n_req = 0
    assert lib.disco_validate_trace(C.byref(tr), 1, None, 256, None) == B.ERR["workspace"]
    assert lib.disco_validate_trace(C.byref(tr), 1, 256, 16, None) == B.ERR["workspace"]
    assert lib.disco_validate_trace(C.byref(tr), 1, 260, 1024, None) == B.ERR["workspace"]      # misaligned
    tr.dev_ttft_c = float("nan")
    assert lib.disco_validate_trace(C.byref(tr), 1, 256, 256, None) == B.ERR["range"]
    tr.dev_ttft_c = 0.0
    tr.dev_pre_spt_s = -1.0
    assert lib.disco_validate_trace(C.byref(tr), 1, 256, 256, None) == B.ERR["range"]
    tr.dev_pre_spt_s = 0.0
    tr.tok_arr = 512                                                                            # token array without offsets
    assert lib.disco_validate_trace(C.byref(tr), 1, 256, 256, None) == B.ERR["csr"]
    tr.tok_arr = None
    assert lib.disco_validate_trace(C.byref(tr), 1, 256, 256, None) == 0                        # an empty trace is sound
    # timing aid
    pol = (B.CPolicy * 1)(B.CPolicy(0, 0, -1, 0.0, float("inf"), float("inf"), 1, 0))
    tl = B.CTimeline(0.2, 3.0, None, 0, 0)
    a, b = C.c_double(0), C.c_double(0)
    assert lib.disco_time_token_walk(C.byref(tr), C.byref(tl), pol, 1, 256, 1 << 30, 5, None, None, None) == B.ERR["null"]
    assert lib.disco_time_token_walk(C.byref(tr), C.byref(tl), pol, 1, 256, 1 << 30, 0, C.byref(a), C.byref(b), None) == B.ERR["shape"]
    assert lib.disco_time_token_walk(C.byref(tr), C.byref(tl), pol, 1, 256, 1 << 30, 5, C.byref(a), C.byref(b), None) == B.ERR["csr"]
    # read probe
    assert lib.disco_read_probe(None, 1024, 256, None) == B.ERR["null"]
    assert lib.disco_read_probe(256, 1000, 256, None) == B.ERR["shape"]                         # not a multiple of 16
    assert lib.disco_read_probe(264, 1024, 256, None) == B.ERR["shape"]                         # misaligned
    assert lib.disco_read_probe(256, 0, 256, None) == 0
    # policy type (Alg. 1)
    assert B.disco_policy_type(DI.COST_S) == B.MODE_S and B.disco_policy_type(DI.COST_D) == B.MODE_D
    assert B.disco_policy_type(dict(DI.COST_S, lam=DI.COST_S["cs_pre"] / DI.COST_S["e_pre"])) == B.MODE_S     # equality
    assert lib.disco_policy_type(None, None) == B.ERR["null"]
    nan = B.CCost(float("nan"), 1, 1, 1, 1)
    m = C.c_int32(0)
    assert lib.disco_policy_type(C.byref(nan), C.byref(m)) == B.ERR["range"]
    # grid divisor
    assert lib.disco_set_grid_divisor(0) == B.ERR["range"] and lib.disco_set_grid_divisor(2000) == B.ERR["range"]
    assert lib.disco_set_grid_divisor(1) == 0


def test_policy_type_agrees_with_the_oracle(B, oracle):
    import itertools
    vals = (0.5, 1.0, 2.0, 3.0)
    for cs_pre, cs_dec, e_pre, e_dec, lam in itertools.product(vals, vals, vals, vals, (0.5, 1.0, 1.5)):
        cost = {"cs_pre": cs_pre, "cs_dec": cs_dec, "e_pre": e_pre, "e_dec": e_dec, "lam": lam}
        assert B.disco_policy_type(cost) == oracle.policy_type(cost), cost
