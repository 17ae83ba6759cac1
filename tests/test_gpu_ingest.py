"""GPU parity of trace ingest and log-normal fitting (Sec. 5.1 traces, Sec. 5.3
fit) against the oracle: relative arrays bit for bit (one fp64 difference, one
rounding), fit parameters to 1e-12 (fp64 sums in a different order, logarithms
of two libraries), counts exactly; then an ingested trace is evaluated."""
import math

import numpy as np
import pytest
import torch

import disco_inputs as DI
from oracle import disco_ingest as I
from test_gpu_parity import assert_same_bits

pytestmark = pytest.mark.gpu


def raw_trace(seed, n, max_out=200):
    rng = np.random.default_rng(seed)
    out_len = rng.integers(1, max_out + 1, n)
    if n > 3:
        out_len[1] = 1
        out_len[2] = 5000
    off = np.zeros(n + 1, np.int64)
    np.cumsum(out_len, out=off[1:])
    send = 1.7e9 + np.cumsum(rng.exponential(0.3, n))                     # epoch seconds
    ttft = rng.lognormal(-1.2, 0.6, n)
    gaps = rng.lognormal(-3.5, 0.6, int(off[-1]))
    tok = np.empty(int(off[-1]))
    for i in range(n):
        a, b = off[i], off[i + 1]
        tok[a] = send[i] + ttft[i]
        tok[a + 1:b] = tok[a] + np.cumsum(gaps[a + 1:b])
    prompt = rng.integers(1, 3000, n).astype(np.int32)
    return send, tok, off, prompt


@pytest.mark.parametrize("n", [0, 1, 2, 777, 5000])
def test_ingest_matches_oracle(B, n):
    print(f"ingest parity n={n}", flush=True)
    send, tok, off, prompt = raw_trace(40 + n, n)
    want = I.ingest(send, tok, off)
    t = B.disco_ingest_trace(torch.from_numpy(send).cuda(), torch.from_numpy(tok).cuda(), torch.from_numpy(off).cuda(),
                             torch.from_numpy(prompt).cuda(), profile=B.disco_device_profile(1))
    assert t.n_req == n and t.n_tok == len(tok)
    assert_same_bits(t.srv_ttft.cpu().numpy(), want["srv_ttft"], "srv_ttft")
    assert_same_bits(t.tok_arr.cpu().numpy(), want["tok_arr"], "tok_arr")
    assert (t.output_len.cpu().numpy() == want["output_len"]).all()
    assert t.dev_dec_spt_s == I.device_profile(1)["dev_dec_spt_s"]


def test_ingest_request_without_tokens(B):
    send, tok, off, prompt = raw_trace(3, 10)
    off[4:] -= off[4] - off[3]                                            # request 3 loses its tokens
    tok = tok[:off[-1]]
    want = I.ingest(send, tok, off)
    t = B.disco_ingest_trace(torch.from_numpy(send).cuda(), torch.from_numpy(tok).cuda(), torch.from_numpy(off).cuda(),
                             torch.from_numpy(prompt).cuda())
    got = t.srv_ttft.cpu().numpy()
    assert math.isnan(got[3]) and math.isnan(want["srv_ttft"][3]) and int(t.output_len[3]) == 0
    keep = np.arange(10) != 3
    assert (got[keep] == want["srv_ttft"][keep]).all()


@pytest.mark.parametrize("n", [0, 1, 1000, 1_000_003])
def test_fit_matches_oracle(B, oracle, n):
    print(f"log-normal fit parity n={n}", flush=True)
    tr = oracle.gen_trace(DI.config(1, n_req=n, seed=8)["gen"])
    for x in (tr["prompt_len"], tr["srv_ttft"]):
        x = x.copy()
        if n >= 1000:                                                     # values without a logarithm
            x[5] = 0
            if x.dtype == np.float32:
                x[6] = -1.0
                x[7] = np.nan
        want = I.fit_lognormal(x)
        got = B.fit_to_host(B.disco_fit_lognormal(torch.from_numpy(x).cuda()))
        assert int(got["n_used"]) == want["n_used"] and int(got["n_skipped"]) == want["n_skipped"]
        if want["n_used"] == 0:
            assert math.isnan(got["mu"]) and math.isnan(got["sigma"])
        else:
            assert abs(got["mu"] - want["mu"]) <= 1e-12 * max(1.0, abs(want["mu"]))
            assert abs(got["sigma"] - want["sigma"]) <= 1e-12 * max(1.0, want["sigma"]) + (1e-7 if n == 1 else 0)
    if n > 1000:
        # the generator's laws come back: prompt lengths are floored and clipped, so only roughly
        fit = B.fit_to_host(B.disco_fit_lognormal(torch.from_numpy(tr["prompt_len"]).cuda()))
        assert abs(fit["mu"] - 5.5) < 0.05 and abs(fit["sigma"] - 1.0) < 0.1


def test_ingested_trace_evaluates_like_the_oracle(B, oracle):
    """Timestamps -> relative trace on the device -> token timelines with a phone profile, against the oracle on
    the oracle's ingest of the same timestamps."""
    print("ingest end to end", flush=True)
    n = 1200
    send, tok, off, prompt = raw_trace(77, n, max_out=300)
    prof = B.disco_device_profile(2)
    t = B.disco_ingest_trace(torch.from_numpy(send).cuda(), torch.from_numpy(tok).cuda(), torch.from_numpy(off).cuda(),
                             torch.from_numpy(prompt).cuda(), profile=prof)
    w = I.ingest(send, tok, off)
    op = I.device_profile(2)
    tr = {"n_req": n, "n_tok": int(off[-1]), "prompt_len": prompt, "output_len": w["output_len"], "srv_ttft": w["srv_ttft"],
          "srv_tbt": None, "dev_pre_spt": None, "dev_dec_spt": None, "tok_off": off, "tok_arr": w["tok_arr"],
          "dev_pre_spt_s": float(op["dev_pre_spt_s"]), "dev_dec_spt_s": float(op["dev_dec_spt_s"]), "dev_ttft_c": 0.0}
    specs = [dict(mode=0, l_th=0, mig_mode=1), dict(mode=0, l_th=500, mig_mode=1), dict(mode=1, l_th=-1, w_tail=0.3, mig_mode=1)]
    bp = [B.Policy(**s) for s in specs]
    opol = [oracle.Policy(**s) for s in specs]
    got = B.disco_eval_migration(t, DI.TAU, DI.KAPPA_LAG, bp, materialise=True)
    want = oracle.migration(tr, opol, DI.TAU, DI.KAPPA_LAG, materialise=True)
    assert_same_bits(got["mig_idx"].cpu().numpy(), want["mig_idx"], "mig_idx")
    assert_same_bits(got["t_last"].cpu().numpy(), want["t_last"], "t_last")
    d = B.disco_eval_dispatch(t, bp, materialise=True)
    wd = oracle.dispatch(tr, opol)
    assert_same_bits(d["ttft"].cpu().numpy(), wd["ttft"], "ttft")
