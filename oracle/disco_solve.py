"""Closed-form policy solves of the DiSCo dispatch controller on an empirical
trace: Alg. 3 (server-constrained length threshold, Eq. 3) and Alg. 2
(device-constrained wait times, Sec. 4.2 Phases 1 and 2).

TEST INFRASTRUCTURE ONLY (same rules as disco_oracle.c): plain, sequential,
exact.  The distributions of the algorithms are the trace's own: p(l) =
count(l) / N over the prompt lengths, F(t) = #{s_i <= t} / N over the server
TTFTs, independent of each other as the paper assumes (Sec. 3).  Budgets and
the tail ratio are rationals and every budget comparison is done in exact
integer / rational arithmetic, so the outcome has no rounding in it; the only
floating-point values are the selected server TTFTs themselves.

Readings where the printed algorithm cannot be taken literally (Alg. 2):
  * the per-length cost p(l) l (1 - alpha) is in tokens while the available
    budget b - alpha is a ratio: the budget is taken in tokens, (b - alpha)
    times the total prompt tokens, and the cost of a length is the extra
    device prefill of moving it from the tail wait to wait 0, (1 - alpha)
    count(l) l;
  * the equation for the partial wait w* has the wrong monotonic direction as
    printed; it is read as "the extra device prefill of that length at wait
    w*, (1 - alpha - F(w*)) count(l) l, equals what is left of the budget",
    and w* is the smallest server TTFT of the trace whose F reaches the
    required level (so the budget is never exceeded);
  * F^-1(q) is the nearest-rank order statistic, rank ceil(q N); rank 0 gives
    a wait of 0.

Pins (tests/test_oracle_solve.py): exhaustive search over all (threshold,
partial wait) pairs on tiny traces (feasible and maximal), the realised
device share of the evaluated policy against the budget, closed forms for
single-length traces, Alg. 3 against the sort-and-prefix-sum solve and the
bisection search of disco_oracle.c.
"""
from fractions import Fraction
import math

import numpy as np


def inverse_cdf(sorted_s: np.ndarray, q: Fraction):
    """F^-1(q) on the empirical distribution: (rank, value), rank = ceil(q N); rank 0 -> wait 0."""
    n = len(sorted_s)
    k = math.ceil(q * n)
    k = min(k, n)
    if k <= 0:
        return 0, np.float32(0.0)
    return k, np.float32(sorted_s[k - 1])


def solve_server_constrained(prompt_len: np.ndarray, b: Fraction) -> dict:
    """Alg. 3 / Eq. 3 in discrete form: the smallest threshold L such that the prompts that still use the
    server (l >= L) hold at most the share b of the prompt tokens; prompts below it run on the device alone."""
    lengths, counts = np.unique(np.asarray(prompt_len, np.int64), return_counts=True)
    total = sum(int(l) * int(c) for l, c in zip(lengths, counts))
    l_max = int(lengths[-1]) if len(lengths) else 0
    server_tokens = total                         # threshold 0: every prompt races
    l_th = 0
    for l, c in zip(lengths, counts):             # raise the threshold past one length of the support at a time
        if Fraction(server_tokens) <= b * total:
            break
        server_tokens -= int(l) * int(c)
        l_th = int(l) + 1
    return {"mode": 0, "l_th": min(l_th, l_max + 1), "server_tokens": server_tokens, "total_tokens": total}


def solve_device_constrained(prompt_len: np.ndarray, srv_ttft: np.ndarray, b: Fraction, alpha: Fraction) -> dict:
    """Alg. 2.  Returns the wait map as the policy record's fields: wait 0 for l <= l_th, w_mid for l == l_mid
    (-1: none), w_tail otherwise."""
    n = len(prompt_len)
    s_sorted = np.sort(np.asarray(srv_ttft, np.float32), kind="stable")
    lengths, counts = np.unique(np.asarray(prompt_len, np.int64), return_counts=True)
    total = sum(int(l) * int(c) for l, c in zip(lengths, counts))
    # Phase 1: tail protection
    rank_tail, w_tail = inverse_cdf(s_sorted, 1 - min(alpha, b))
    out = {"mode": 1, "l_th": -1, "l_mid": -1, "w_mid": np.float32(0.0), "w_tail": w_tail,
           "rank_tail": rank_tail, "rank_mid": 0, "zero_wait_tokens": 0, "total_tokens": total}
    if b <= alpha:
        return out                                 # the tail wait for every length
    # Phase 2: spend the rest on immediate starts, shortest prompts first
    available = (b - alpha) * total                # tokens
    for l, c in zip(lengths, counts):
        mass = int(l) * int(c)
        length_cost = (1 - alpha) * mass
        if available >= length_cost:
            out["l_th"] = int(l)
            out["zero_wait_tokens"] += mass
            available -= length_cost
        else:
            # partial wait: (1 - alpha - F(w*)) mass = available
            level = (1 - alpha) - available / mass
            out["rank_mid"], out["w_mid"] = inverse_cdf(s_sorted, level)
            out["l_mid"] = int(l)
            break
    return out


def expected_device_tokens(prompt_len: np.ndarray, srv_ttft: np.ndarray, pol: dict) -> Fraction:
    """E[I_d(l) l] N under the independence model: every length starts the device with probability
    1 - F(w(l)).  Used by the pins, not by the solve."""
    n = len(srv_ttft)
    s = np.asarray(srv_ttft, np.float32)
    lengths, counts = np.unique(np.asarray(prompt_len, np.int64), return_counts=True)
    acc = Fraction(0)
    for l, c in zip(lengths, counts):
        if l <= pol["l_th"]:
            w = np.float32(0.0)
        elif l == pol["l_mid"]:
            w = pol["w_mid"]
        else:
            w = pol["w_tail"]
        started = int((s > w).sum())
        acc += Fraction(started, n) * int(l) * int(c)
    return acc
