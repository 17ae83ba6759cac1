"""Pins of the oracle's closed-form policy solves (Alg. 2: device-constrained
wait times; Alg. 3 / Eq. 3: server-constrained length threshold).

Independent of the solves' own loops: exhaustive search over every policy of
the algorithm's family on tiny traces, the device's realised share of the
prompt tokens when the solved policy is evaluated by the dispatch oracle,
hand-worked single-length cases, and Alg. 3 against a numpy sort-and-cumsum
solve and against the bisection search."""
from fractions import Fraction as F
import math

import numpy as np
import pytest

import disco_inputs as DI
from oracle import disco_solve as S


@pytest.mark.parametrize("seed", range(12))
def test_alg2_is_the_most_aggressive_feasible_policy_of_its_family(seed):
    """Exhaustive search.  Family: zero wait for the k shortest lengths, the tail wait for the others except that
    length k may wait until the server's r-th smallest TTFT (start probability 1 - r/n).  Accounting of Alg. 2:
    a zero-wait length costs its tokens, the partial one (1 - r/n) of them, a tail length alpha of them.  The
    solve must return the largest k affordable with everything else at the tail wait and, for it, the smallest
    affordable r."""
    rng = np.random.default_rng(seed)
    n = int(rng.integers(6, 14))
    prompt = rng.choice([2, 3, 5, 8], n).astype(np.int32)
    s = rng.permutation(np.arange(1, n + 1)).astype(np.float32) / np.float32(8)        # distinct server TTFTs
    if seed % 3 == 0:
        s[rng.integers(0, n, 3)] = s[0]                                                  # ties
    lengths, counts = np.unique(prompt.astype(np.int64), return_counts=True)
    mass = [int(l) * int(c) for l, c in zip(lengths, counts)]
    total = sum(mass)
    s_sorted = np.sort(s)
    for b, alpha in ((F(1, 2), F(1, 5)), (F(3, 4), F(1, 10)), (F(2, 5), F(1, 3)), (F(9, 10), F(1, 4)), (F(1), F(1, 7)),
                     (F(11, 20), F(1, 2))):
        pol = S.solve_device_constrained(prompt, s, b, alpha)
        rank_tail = math.ceil((1 - alpha) * n)
        assert pol["rank_tail"] == rank_tail and pol["w_tail"] == s_sorted[rank_tail - 1]
        k = max(k for k in range(len(lengths) + 1) if sum(mass[:k]) + alpha * sum(mass[k:]) <= b * total)
        r = None
        if k < len(lengths):
            r = min(r for r in range(0, rank_tail + 1)
                    if sum(mass[:k]) + (1 - F(r, n)) * mass[k] + alpha * sum(mass[k + 1:]) <= b * total)
        best = (k, r)
        assert pol["l_th"] == (int(lengths[k - 1]) if k else -1), (seed, b, alpha, pol, best)
        assert pol["zero_wait_tokens"] == sum(mass[:k])
        if k < len(lengths):
            assert pol["l_mid"] == int(lengths[k]) and pol["rank_mid"] == r and r >= 1, (seed, b, alpha, pol, best)
            assert pol["w_mid"] == s_sorted[r - 1]
        else:
            assert pol["l_mid"] == -1


def test_alg2_phase1_only_when_the_budget_is_within_the_tail_ratio():
    rng = np.random.default_rng(5)
    s = rng.lognormal(-1, 0.7, 1000).astype(np.float32)
    prompt = rng.integers(1, 500, 1000).astype(np.int32)
    for b, alpha in ((F(1, 20), F(1, 10)), (F(1, 10), F(1, 10)), (F(0), F(1, 10))):
        pol = S.solve_device_constrained(prompt, s, b, alpha)
        assert pol["l_th"] == -1 and pol["l_mid"] == -1
        # w_tail is the (1 - b) quantile: at most b N requests see no server token by then
        assert int((s > pol["w_tail"]).sum()) <= b * 1000 < int((s >= pol["w_tail"]).sum()) or b == 0
    assert S.solve_device_constrained(prompt, s, F(0), F(1, 10))["w_tail"] == s.max()     # never start the device


def test_alg2_single_length_closed_form():
    # 1000 prompts of 100 tokens, server TTFTs 1/1024 .. 1000/1024: F(i/1024) = i/1000
    s = (np.arange(1, 1001, dtype=np.float32) / np.float32(1024))[np.random.default_rng(0).permutation(1000)]
    prompt = np.full(1000, 100, np.int32)
    pol = S.solve_device_constrained(prompt, s, F(1, 2), F(1, 10))
    # tail: F^-1(0.9) = 900/1024; phase 2: 0.4 of the tokens left, a zero wait would cost 0.9: partial wait with
    # 0.9 - F(w*) = 0.4, F(w*) = 0.5
    assert pol["rank_tail"] == 900 and pol["w_tail"] == np.float32(900 / 1024)
    assert pol["l_th"] == -1 and pol["l_mid"] == 100 and pol["rank_mid"] == 500 and pol["w_mid"] == np.float32(500 / 1024)
    full = S.solve_device_constrained(prompt, s, F(1), F(1, 10))
    assert full["l_th"] == 100 and full["l_mid"] == -1 and full["zero_wait_tokens"] == 100_000


@pytest.mark.parametrize("b,alpha", [(F(1, 20), F(1, 10)), (F(3, 10), F(1, 10)), (F(7, 10), F(1, 20)), (F(1), F(1, 10))])
def test_alg2_realised_device_share_meets_the_budget(oracle, b, alpha):
    """Evaluate the solved policy request by request: the device's share of the prompt tokens is b up to the
    sampling noise of the independence assumption (server TTFT and prompt length are independent in the trace)."""
    tr = oracle.gen_trace(DI.config(0, n_req=200_000, seed=9)["gen"])
    pol = S.solve_device_constrained(tr["prompt_len"], tr["srv_ttft"], b, alpha)
    p = oracle.Policy(mode=1, l_th=pol["l_th"], l_mid=pol["l_mid"], w_mid=float(pol["w_mid"]), w_tail=float(pol["w_tail"]))
    r = oracle.dispatch(tr, [p], materialise=False)
    total = int(tr["prompt_len"].astype(np.int64).sum())
    share = int(r["d_pre"][0]) / total
    assert abs(share - float(b)) < 0.004, (share, float(b))
    # and never above the model's accounting, which prices the tail at alpha although F(w_tail) >= 1 - alpha
    assert S.expected_device_tokens(tr["prompt_len"], tr["srv_ttft"], pol) <= b * total


def test_alg2_is_monotone_in_the_budget():
    rng = np.random.default_rng(2)
    s = rng.lognormal(-1, 0.7, 5000).astype(np.float32)
    prompt = np.clip(rng.lognormal(5, 1, 5000), 1, 4000).astype(np.int32)
    prev = (-2, np.float32(np.inf))
    for j in range(1, 21):
        pol = S.solve_device_constrained(prompt, s, F(j, 20), F(1, 10))
        key = (pol["l_th"], -pol["w_mid"] if pol["l_mid"] >= 0 else np.float32(0))
        assert pol["l_th"] >= prev[0]
        prev = (pol["l_th"], pol["w_mid"])


@pytest.mark.parametrize("seed", range(4))
def test_alg3_matches_sort_and_cumsum_and_the_bisection(oracle, seed):
    tr = oracle.gen_trace(DI.config(0, n_req=20_000, seed=seed)["gen"])
    l = tr["prompt_len"].astype(np.int64)
    total = int(l.sum())
    lmax = int(l.max())
    for j in range(16):
        b = F(j, 15)
        pol = S.solve_server_constrained(tr["prompt_len"], b)
        # numpy: thresholds worth trying are 0 and one past each length of the trace; take the smallest that fits
        cand = np.unique(np.concatenate([[0], np.unique(l) + 1]))
        fits = [int(L) for L in cand if int(l[l >= L].sum()) * b.denominator <= b.numerator * total]
        assert pol["l_th"] == min(fits), (j, pol["l_th"], min(fits))
        assert int(l[l >= pol["l_th"]].sum()) == pol["server_tokens"]
        assert pol["server_tokens"] * b.denominator <= b.numerator * total
        if pol["l_th"] > 0:                      # minimal: one less lets too many tokens through
            assert int(l[l >= pol["l_th"] - 1].sum()) * b.denominator > b.numerator * total
        steps = max(1, (lmax + 1).bit_length())
        l_bis, _, _ = oracle.search_lth(tr, oracle.Policy(mode=0), 0, lmax + 1, steps, "server_prefill_tok", DI.COST_S,
                                        float(b) * total)
        if abs(float(b) * total - round(float(b) * total)) > 1e-6 or j in (0, 15):   # the bisection compares in fp64
            assert l_bis == pol["l_th"], (j, l_bis, pol["l_th"])
