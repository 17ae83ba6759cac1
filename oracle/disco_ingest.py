"""Trace ingest, log-normal fitting and device profiles (Sec. 5.1 set-up,
Sec. 5.3 scalability study): a recorded trace with wall-clock timestamps
becomes the relative-time arrays the evaluation works on, and the log-normal
laws of the synthetic traces are fitted to it by the mean and standard
deviation of the logarithm.

TEST INFRASTRUCTURE ONLY (same rules as disco_oracle.c).  Plain numpy in fp64.

Readings: timestamps are fp64 seconds; a difference is taken in fp64 and
rounded once to fp32; the standard deviation is the population one (1/N);
values that are not positive have no logarithm and are left out of the fit
(counted).  Pins (tests/test_oracle_ingest.py): round trip of traces with
dyadic times, scipy's maximum-likelihood log-normal fit, samples with known
mean and deviation of the logarithm, the device speeds printed in Sec. 5.1.
"""
import numpy as np

# Device profiles of Sec. 5.1: (device, model, prefill tokens/s, decode tokens/s)
DEVICE_PROFILES = (
    ("Pixel 7 Pro", "Bloom 1.1B", 31.32, 13.93),
    ("Pixel 7 Pro", "Bloom 560M", 51.80, 20.14),
    ("Xiaomi 14", "Qwen 1.5 0.5B", 79.90, 21.47),
)


def device_profile(idx: int) -> dict:
    """Seconds per prompt token and per decoded token (fp32) of profile `idx`; the device TTFT is linear in the
    prompt length with this slope (Sec. 4.2) and no intercept."""
    dev, model, pre, dec = DEVICE_PROFILES[idx]
    return {"device": dev, "model": model,
            "dev_pre_spt_s": np.float32(np.float64(1.0) / np.float64(pre)),
            "dev_dec_spt_s": np.float32(np.float64(1.0) / np.float64(dec))}


def ingest(t_send: np.ndarray, t_token: np.ndarray, tok_off: np.ndarray) -> dict:
    """Server TTFT = first token's arrival - send time; token arrival offsets relative to the request's first
    token; output length = number of tokens."""
    t_send = np.asarray(t_send, np.float64)
    t_token = np.asarray(t_token, np.float64)
    tok_off = np.asarray(tok_off, np.int64)
    n = len(t_send)
    srv_ttft = np.empty(n, np.float32)
    output_len = np.empty(n, np.int32)
    tok_arr = np.empty(len(t_token), np.float32)
    for i in range(n):
        a, b = int(tok_off[i]), int(tok_off[i + 1])
        output_len[i] = max(b - a, 0)
        if b <= a:                                  # no token, no first token: the request cannot be evaluated
            output_len[i] = 0
            srv_ttft[i] = np.nan
            continue
        first = t_token[a]
        srv_ttft[i] = np.float32(first - t_send[i])
        for j in range(a, b):
            tok_arr[j] = np.float32(t_token[j] - first)
    return {"srv_ttft": srv_ttft, "output_len": output_len, "tok_arr": tok_arr}


def fit_lognormal(x: np.ndarray) -> dict:
    """mu, sigma = mean and (population) standard deviation of ln x over the positive values."""
    x = np.asarray(x).astype(np.float64)
    pos = x[x > 0]
    if len(pos) == 0:
        return {"mu": float("nan"), "sigma": float("nan"), "n_used": 0, "n_skipped": int(len(x))}
    lx = np.log(pos)
    mu = float(lx.sum() / len(pos))
    sigma = float(np.sqrt(((lx - mu) ** 2).sum() / len(pos)))
    return {"mu": mu, "sigma": sigma, "n_used": int(len(pos)), "n_skipped": int(len(x) - len(pos))}
