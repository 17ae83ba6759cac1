"""Opt-in trace validation (disco_validate_trace), guard words around every per-pair output buffer, and the same
input under two launch geometries: host-forced conditions only, every kernel exits normally."""
import ctypes as C

import numpy as np
import pytest
import torch

import disco_inputs as DI

pytestmark = pytest.mark.gpu


def small_trace(B, n_req=700, seed=3):
    cfg = DI.config(2, n_req=n_req, seed=seed)
    return cfg, B.disco_gen_trace(cfg["gen"])


def test_a_generated_trace_is_sound(B):
    cfg, tr = small_trace(B)
    assert B.disco_validate_trace(tr) == 0
    cfg0 = DI.config(0, n_req=500, seed=2)
    t0 = B.disco_gen_trace(cfg0["gen"])                     # no token array
    assert B.disco_validate_trace(t0) == 0


@pytest.mark.parametrize("what", ["decreasing_offset", "length_mismatch", "first_offset", "last_offset", "offset_beyond"])
def test_inconsistent_offsets_are_reported_as_csr(B, what):
    print(f"validate: {what}", flush=True)
    cfg, tr = small_trace(B)
    off = tr.tok_off.clone()
    n = tr.output_len.clone()
    if what == "decreasing_offset":
        off[200] = off[199] - 1
    elif what == "length_mismatch":
        n[300] += 1
    elif what == "first_offset":
        off[0] = 1
    elif what == "last_offset":
        off[-1] -= 1
    else:
        off[400] = tr.n_tok + 5
    tr.tok_off, tr.output_len = off, n
    assert B.disco_validate_trace(tr) == B.ERR["csr"]       # (the token pass is not run on unsound offsets)


@pytest.mark.parametrize("what", ["nan_ttft", "negative_ttft", "zero_length", "negative_prompt", "nan_rate",
                                  "negative_token", "decreasing_token", "nan_token", "first_token_not_zero"])
def test_values_out_of_range_are_reported_as_range(B, what):
    print(f"validate: {what}", flush=True)
    cfg, tr = small_trace(B)
    arr = tr.tok_arr.clone()
    lo = int(tr.tok_off[100].item())
    assert int(tr.output_len[100].item()) >= 1
    if what == "nan_ttft":
        tr.srv_ttft = tr.srv_ttft.clone(); tr.srv_ttft[5] = float("nan")
    elif what == "negative_ttft":
        tr.srv_ttft = tr.srv_ttft.clone(); tr.srv_ttft[6] = -0.25
    elif what == "zero_length":
        # (kept consistent with the offsets: an empty request, as the ingest marks one without tokens)
        n = tr.output_len.clone(); off = tr.tok_off.clone()
        k = int(n[7].item()); n[7] = 0; off[8:] -= k
        tr.output_len, tr.tok_off, tr.n_tok = n, off, tr.n_tok - k
    elif what == "negative_prompt":
        tr.prompt_len = tr.prompt_len.clone(); tr.prompt_len[9] = -4
    elif what == "nan_rate":
        tr.dev_dec_spt = tr.dev_dec_spt.clone(); tr.dev_dec_spt[10] = float("nan")
    elif what == "negative_token":
        arr[lo + 1] = -1.0
    elif what == "decreasing_token":
        n100 = int(tr.output_len[100].item())
        i = next(j for j in range(100, 700) if int(tr.output_len[j].item()) >= 3)
        a = int(tr.tok_off[i].item())
        arr[a + 2] = arr[a + 1] * 0.5 if float(arr[a + 1]) > 0 else -1.0
    elif what == "nan_token":
        arr[lo] = float("nan")
    else:
        arr[lo] = 0.125
    tr.tok_arr = arr
    assert B.disco_validate_trace(tr) == B.ERR["range"]
    if what.endswith("token") or what == "first_token_not_zero":
        assert B.disco_validate_trace(tr, check_tokens=False) == 0      # the token pass is optional


def test_an_ingested_trace_with_a_disordered_recording_is_caught(B):
    """Recorded timestamps enter through disco_ingest_trace: a token stamped before its predecessor, or before the
    request was sent, shows up as a value out of range."""
    rng = np.random.default_rng(8)
    n_req = 300
    n = rng.integers(1, 60, n_req)
    off = np.zeros(n_req + 1, np.int64); np.cumsum(n, out=off[1:])
    send = np.cumsum(rng.uniform(0.1, 1.0, n_req)) + 1.7e9
    tok = np.concatenate([send[i] + 0.3 + np.cumsum(rng.uniform(0.01, 0.05, n[i])) for i in range(n_req)])
    plen = torch.from_numpy(rng.integers(8, 500, n_req).astype(np.int32)).cuda()
    prof = B.disco_device_profile(0)
    def ingest(tok_, send_):
        return B.disco_ingest_trace(torch.from_numpy(send_).cuda(), torch.from_numpy(tok_).cuda(), torch.from_numpy(off).cuda(), plen, prof)
    assert B.disco_validate_trace(ingest(tok, send)) == 0
    bad = tok.copy(); bad[off[50] + 3] = bad[off[50] + 1]            # a token stamped before its predecessor
    if n[50] > 4:
        assert B.disco_validate_trace(ingest(bad, send)) == B.ERR["range"]
    late = send.copy(); late[70] = tok[off[70]] + 1.0                  # sent after its first token arrived
    assert B.disco_validate_trace(ingest(tok, late)) == B.ERR["range"]


GUARD = 64        # elements of guard on each side


def guarded(shape, dtype, fill):
    """A buffer with GUARD sentinel elements in front of and behind the part handed to the library."""
    n = int(np.prod(shape))
    whole = torch.full((n + 2 * GUARD,), fill, dtype=dtype, device="cuda")
    return whole, whole[GUARD:GUARD + n]


def test_guard_words_around_every_output_buffer_stay_intact(B):
    """Every optional per-pair and per-token output, the accumulators and the statistics records are handed over as
    the middle of a larger buffer filled with a sentinel: nothing may be written outside the part that was passed."""
    cfg = DI.config(2, n_req=1_237, seed=21)
    tr = B.disco_gen_trace(cfg["gen"])
    N, T = tr.n_req, tr.n_tok
    pols = [B.Policy(mode=0, l_th=0, mig_mode=1), B.Policy(mode=0, l_th=200, mig_mode=0), B.Policy(mode=0, l_th=250, mig_mode=2),
            B.Policy(mode=1, l_th=-1, w_tail=DI.f32(0.3), mig_mode=1), B.Policy(mode=1, l_th=-1, w_tail=0.0, mig_mode=2)]
    P = len(pols)
    ws = B.workspace(N, P)
    bufs = {}
    def g(name, shape, dtype, fill):
        bufs[name] = guarded(shape, dtype, fill) + (fill,)
        return bufs[name][1]
    dec = g("decision", (P, N), torch.uint8, 0xA5)
    ttft = g("ttft", (P, N), torch.float32, -7.0)
    acc = g("acc", (P * 128,), torch.uint8, 0x5A)
    mig = g("mig_idx", (P, N), torch.int32, -77)
    nsrc = g("n_src_tok", (P, N), torch.int32, -77)
    tlast = g("t_last", (P, N), torch.float32, -7.0)
    dnum = g("delay_num", (P, N), torch.int32, -77)
    deliv = g("delivered", (T,), torch.float32, -7.0)
    stats = g("stats", (P * 256,), torch.uint8, 0x5A)
    cs = tr.c_struct()
    arr = B._policies(pols)
    out = B.CPairOut(dec.data_ptr(), ttft.data_ptr())
    st = torch.cuda.current_stream().cuda_stream
    assert B._lib.disco_eval_dispatch(C.byref(cs), arr, P, C.byref(out), acc.data_ptr(), ws.data_ptr(), ws.numel(), st) == 0
    cost = B._cost(DI.COST_S)
    tl = B.CTimeline(cfg["tau"], cfg["kappa"], C.pointer(cost), 0, 0)
    for with_delivered in (False, True):                   # the streaming kernels, then the general one
        mo = B.CMigOut(mig.data_ptr(), nsrc.data_ptr(), tlast.data_ptr(), deliv.data_ptr() if with_delivered else None, 0, 0,
                       dnum.data_ptr())
        assert B._lib.disco_eval_migration(C.byref(cs), C.byref(tl), arr, P, C.byref(mo), acc.data_ptr(), ws.data_ptr(),
                                           ws.numel(), st) == 0
    q = (B.CQuantile * 2)(B.CQuantile(50, 100), B.CQuantile(99, 100))
    assert B._lib.disco_reduce_stats(C.byref(cs), C.byref(cost), C.byref(tl), arr, P, acc.data_ptr(), q, 2, stats.data_ptr(),
                                     ws.data_ptr(), ws.numel(), st) == 0
    torch.cuda.synchronize()
    for name, (whole, inner, fill) in bufs.items():
        front, back = whole[:GUARD], whole[GUARD + inner.numel():]
        assert bool((front == fill).all().item()) and bool((back == fill).all().item()), name
    # ... and the buffers themselves were filled
    assert not bool((dec == 0xA5).all().item()) and bool((mig >= -1).all().item()) and bool((deliv >= 0).all().item())


def test_two_launch_geometries_give_the_same_bits(B):
    """The dispatch pass and the token walk under the normal grids and under grids a third (and a 64th) as large:
    every integer total, per-pair output and order statistic identical, the fp64 sums to 1e-12 relative."""
    cfg = DI.config(4, n_req=30_011, seed=6)
    tr = B.disco_gen_trace(cfg["gen"])
    P = 8
    lths = [40_000, 2_000, 900, 500, 300, 150, 60, 0]
    pols = [B.Policy(mode=0, l_th=l, mig_mode=1 if j % 3 else 0) for j, l in enumerate(lths)]
    ws = B.workspace(tr.n_req, P)
    def run():
        r = B.disco_eval_dispatch(tr, pols, materialise=True, ws=ws)
        mg = B.disco_eval_migration(tr, cfg["tau"], cfg["kappa"], pols, materialise=True, ws=ws, acc=r["acc"])
        st = B.disco_reduce_stats(tr, cfg["cost"], pols, r["acc"], tau=cfg["tau"], kappa=cfg["kappa"], ws=ws, reuse_walk=True)
        torch.cuda.synchronize()
        return (B.accum_to_host(r["acc"], P).copy(), r["decision"].clone(), r["ttft"].clone(), mg["mig_idx"].clone(),
                mg["n_src_tok"].clone(), mg["t_last"].clone(), B.stats_to_host(st, P).copy())
    try:
        base = run()
        for d in (3, 64):
            assert B._lib.disco_set_grid_divisor(d) == 0
            other = run()
            for f in ("s_pre", "s_dec", "d_pre", "d_dec", "n_dev_started", "n_dev_win", "m_s_dec", "m_d_dec", "m_d_repre",
                      "n_migrated", "tbt_count", "ttft_min_bits", "ttft_max_bits"):
                assert (base[0][f] == other[0][f]).all(), (d, f)
            for f in ("ttft_sum", "tlast_sum"):
                assert np.allclose(base[0][f], other[0][f], rtol=1e-12, atol=0), (d, f)
            for a, b in zip(base[1:6], other[1:6]):
                assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), d
            for f in ("ttft_rank", "tbt_rank", "s_dec", "d_dec", "n_migrated"):
                assert (base[6][f] == other[6][f]).all(), (d, f)
            for f in ("ttft_q", "tbt_q"):
                assert (base[6][f].view(np.uint32) == other[6][f].view(np.uint32)).all(), (d, f)
    finally:
        assert B._lib.disco_set_grid_divisor(1) == 0
