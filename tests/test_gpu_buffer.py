"""GPU parity of the buffer-based, cost-triggered migration (Sec. 4.3) against
the oracle: per-pair hand-off index, source tokens, last delivery, delayed
tokens (bit-exact), per-column token totals (exact), delivered offsets of one
column (bit-exact), and the statistics incl. TBT order statistics and the mean
number of delayed tokens per migrated request."""
import math

import numpy as np
import pytest
import torch

import disco_inputs as DI
from test_gpu_parity import check_migration, check_stats, both

pytestmark = pytest.mark.gpu


def buffer_policies():
    inf = math.inf
    return [
        dict(mode=0, l_th=0, mig_mode=2),                         # race everything, server -> device hand-offs
        dict(mode=0, l_th=20, mig_mode=2),
        dict(mode=0, l_th=10 ** 9, mig_mode=2),                   # device only: never a hand-off in this mode
        dict(mode=1, l_th=-1, w_tail=0.0, mig_mode=2),            # race everything, device -> server hand-offs
        dict(mode=1, l_th=-1, w_tail=inf, mig_mode=2),            # server only: never a hand-off in this mode
        dict(mode=1, l_th=10, beta=DI.f32(0.02), w_tail=DI.f32(0.5), mig_mode=2),
        dict(mode=0, l_th=240, mig_mode=1),                       # lag trigger next to buffer columns
        dict(mode=1, l_th=-1, w_tail=DI.f32(0.35), mig_mode=0),
    ]


def slow_prefill(tr, factor=64.0):
    """Short prompts and a slow device prefill: the server wins many races and re-prefilling is cheap."""
    tr = dict(tr)
    tr["prompt_len"] = (tr["prompt_len"] % 48 + 1).astype(np.int32)
    tr["dev_pre_spt"] = (tr["dev_pre_spt"] * np.float32(factor)).astype(np.float32)
    return tr


@pytest.mark.parametrize("n_req,max_out,cost", [(0, 10, "S"), (1, 1, "S"), (1, 2, "D"), (300, 120, "S"), (300, 120, "D"),
                                                (900, 400, "S"), (900, 400, "D"), (257, 1500, "D")])
def test_buffer_migration_matches_oracle(B, oracle, n_req, max_out, cost):
    print(f"buffer migration parity n_req={n_req} max_out={max_out} cost={cost}", flush=True)
    cost = DI.COST_S if cost == "S" else DI.COST_D
    tr = slow_prefill(DI.handmade_trace(23 + n_req, n_req, tokens=True, max_out=max_out, stall_p=0.02, ties=True))
    # with the deliveries of a column the general kernel walks every pair; without them the buffer pairs are settled
    # from the cost bound, the probe of the first tokens and the streaming walk's summaries
    for col in (0, 3, None):
        _, acc, want = check_migration(B, oracle, tr, buffer_policies(), DI.TAU, DI.KAPPA_LAG, delivered_col=col, cost=cost)
    if n_req >= 300:
        # both hand-off directions occur under the price that favours the target
        j = 0 if cost is DI.COST_S else 3
        assert want["n_migrated"][j] > 20, want["n_migrated"]
        assert want["n_migrated"][2] == 0 and want["n_migrated"][4] == 0


def test_buffer_migration_without_rates_never_hands_off(B, oracle):
    print("buffer migration parity without rates", flush=True)
    tr = slow_prefill(DI.handmade_trace(5, 400, tokens=True, max_out=120, stall_p=0.01))
    _, acc, want = check_migration(B, oracle, tr, buffer_policies()[:6], DI.TAU, DI.KAPPA_LAG, delivered_col=0, cost=None)
    assert (want["n_migrated"] == 0).all() and (acc["n_migrated"] == 0).all()


def test_buffer_migration_constant_gap_server(B, oracle):
    # no per-token trace: server arrivals t * srv_tbt, as source and as target
    print("buffer migration parity constant-gap", flush=True)
    tr = oracle.gen_trace(DI.config(0, n_req=2_001, seed=5)["gen"])
    tr["tok_arr"] = None
    for cost in (DI.COST_S, DI.COST_D):
        _, acc, want = check_migration(B, oracle, tr, buffer_policies(), DI.TAU, DI.KAPPA_LAG, delivered_col=3, cost=cost)
    # a slow server target: tokens are late after the hand-off
    tr["srv_tbt"] = (tr["srv_tbt"] * np.float32(6.0)).astype(np.float32)
    _, acc, want = check_migration(B, oracle, tr, buffer_policies(), DI.TAU, DI.KAPPA_LAG, delivered_col=3, cost=DI.COST_D)
    assert want["delay_sum"][3] > 0
    check_migration(B, oracle, tr, buffer_policies(), DI.TAU, DI.KAPPA_LAG, delivered_col=None, cost=DI.COST_D)


def test_buffer_migration_late_handoffs(B, oracle):
    """Sources whose gaps hover around the pacing interval fill the buffer slowly: hand-offs deep inside long
    requests (chunks after the first), in both directions, and late tokens behind a slow target."""
    print("buffer migration parity late hand-offs", flush=True)
    tau = 0.2
    rng = np.random.default_rng(19)
    tr = DI.handmade_trace(201, 240, tokens=True, max_out=1500, stall_p=0.0)
    l0 = tr["prompt_len"]
    tr["prompt_len"] = np.where(np.arange(len(l0)) % 2 == 1, 500 + l0 % 400, l0 % 200 + 1).astype(np.int32)
    n, off = tr["output_len"], tr["tok_off"]
    gaps = rng.lognormal(math.log(tau) - 0.25, 0.5, int(off[-1])).astype(np.float32)     # mean a little below tau
    arr = np.empty(int(off[-1]), np.float32)
    for i in range(len(n)):
        a, b = int(off[i]), int(off[i + 1])
        arr[a] = 0
        arr[a + 1:b] = np.cumsum(gaps[a + 1:b], dtype=np.float32)
    tr = dict(tr, tok_arr=arr)
    tr["srv_ttft"] = (tr["srv_ttft"] * np.float32(8.0)).astype(np.float32)               # long hand-off to the server
    tr["dev_dec_spt"] = rng.uniform(0.17, 0.26, len(n)).astype(np.float32)               # device near the pacing interval
    tr["dev_pre_spt"] = (tr["dev_dec_spt"] / np.float32(40.0)).astype(np.float32)
    specs = [dict(mode=0, l_th=0, mig_mode=2), dict(mode=1, l_th=-1, w_tail=0.0, mig_mode=2),
             dict(mode=1, l_th=-1, w_tail=math.inf, mig_mode=1)]
    for cost, col in ((DI.COST_S, 0), (DI.COST_D, 1)):
        _, acc, want = check_migration(B, oracle, tr, specs, tau, 3.0, delivered_col=col, cost=cost)
        check_migration(B, oracle, tr, specs, tau, 3.0, delivered_col=None, cost=cost)       # hand-offs beyond the probed tokens
        m = want["mig_idx"][col]
        assert (m >= 256).sum() > 5, (col, (m >= 0).sum(), (m >= 256).sum())
        assert want["delay_sum"][col] > 0
        check_stats(B, oracle, tr, specs, cost, tau=tau, kappa=3.0)


def test_buffer_handoff_to_devices_barely_faster_than_the_pacing(B, oracle):
    """Devices whose gap is tau (1 - 2^-k), k = 6 .. 23: behind a hand-off the target's arrivals creep ahead of the
    pacing slots by less and less, down to where fp32 rounding decides whether a token is late.  The statistics walk
    ends at the hand-off where it can prove the tail paced and walks on otherwise; both must give the oracle's bits."""
    print("buffer migration parity, device gap just below tau", flush=True)
    tau = 0.2
    rng = np.random.default_rng(23)
    tr = DI.handmade_trace(211, 360, tokens=True, max_out=1500, stall_p=0.0)
    tr["prompt_len"] = (tr["prompt_len"] % 500 + 1).astype(np.int32)
    n, off = tr["output_len"], tr["tok_off"]
    gaps = rng.lognormal(math.log(tau) - 0.35, 0.45, int(off[-1])).astype(np.float32)
    arr = np.empty(int(off[-1]), np.float32)
    for i in range(len(n)):
        a, b = int(off[i]), int(off[i + 1])
        arr[a] = 0
        arr[a + 1:b] = np.cumsum(gaps[a + 1:b], dtype=np.float32)
    tr = dict(tr, tok_arr=arr)
    k = 6 + np.arange(len(n)) % 18
    tr["dev_dec_spt"] = (np.float32(tau) * (np.float32(1.0) - np.exp2(-k.astype(np.float32)))).astype(np.float32)
    tr["dev_pre_spt"] = (tr["dev_dec_spt"] / np.float32(10.0)).astype(np.float32)      # the server wins the races
    specs = [dict(mode=0, l_th=0, mig_mode=2), dict(mode=0, l_th=60, mig_mode=2)]
    _, acc, want = check_migration(B, oracle, tr, specs, tau, 3.0, delivered_col=0, cost=DI.COST_S)
    check_migration(B, oracle, tr, specs, tau, 3.0, delivered_col=None, cost=DI.COST_S)
    m = want["mig_idx"][0]
    assert (m >= 0).sum() > 100 and (m >= 256).sum() > 3, ((m >= 0).sum(), (m >= 256).sum())
    assert ((m >= 0) & (m < 128)).sum() > 20          # ... and hand-offs the probe of the first tokens sees
    check_stats(B, oracle, tr, specs, DI.COST_S, tau=tau, kappa=3.0)


@pytest.mark.parametrize("cost", ["S", "D"])
def test_buffer_stats(B, oracle, cost):
    print(f"buffer statistics parity cost={cost}", flush=True)
    cost = DI.COST_S if cost == "S" else DI.COST_D
    tr = slow_prefill(DI.handmade_trace(31, 1200, tokens=True, max_out=200, stall_p=0.03))
    got, want = check_stats(B, oracle, tr, buffer_policies(), cost, tau=DI.TAU, kappa=DI.KAPPA_LAG,
                            quantiles=((50, 100), (99, 100), (999, 1000)))
    assert max(w["n_migrated"] for w in want) > 50
    # server re-prefill tokens of device -> server hand-offs are part of the server's prefill count
    if cost is DI.COST_D:
        assert want[3]["s_pre"] > oracle.stats(tr, [oracle.Policy(mode=1, l_th=-1, w_tail=0.0)], cost)[0]["s_pre"]


def test_buffer_many_columns(B, oracle):
    """40 columns of both hand-off directions and both prices: the per-column totals of the buffer pairs are added by
    column lanes that each read every request of a batch (no sub-groups left at more than 32 columns), on a request
    count that fills the last batch only partly."""
    print("buffer parity 40 columns", flush=True)
    rng = np.random.default_rng(77)
    tr = slow_prefill(DI.handmade_trace(57, 1003, tokens=True, max_out=180, stall_p=0.02))
    specs = []
    for j in range(40):
        if j % 2 == 0:
            specs.append(dict(mode=0, l_th=int(rng.integers(0, 60)), mig_mode=2 if j % 6 else 1))
        else:
            specs.append(dict(mode=1, l_th=int(rng.integers(-1, 30)), w_tail=DI.f32(rng.uniform(0, 0.8)), mig_mode=2 if j % 5 else 0))
    for cost in (DI.COST_S, DI.COST_D):
        _, acc, want = check_migration(B, oracle, tr, specs, DI.TAU, DI.KAPPA_LAG, delivered_col=None, cost=cost)
        assert max(want["n_migrated"]) > 20
    check_stats(B, oracle, tr, specs, DI.COST_S, tau=DI.TAU, kappa=DI.KAPPA_LAG)


def test_buffer_columns_in_a_device_resident_table(B, oracle):
    """The table never visits the host: the library cannot inspect it and picks the kernel on the device."""
    print("buffer migration parity device-resident table", flush=True)
    tr = slow_prefill(DI.handmade_trace(41, 500, tokens=True, max_out=150, stall_p=0.02))
    for specs in (buffer_policies(), [dict(mode=0, l_th=0, mig_mode=1), dict(mode=1, l_th=-1, w_tail=0.0, mig_mode=0)]):
        rec = np.zeros(len(specs), B.POLICY_DTYPE)
        for j, p in enumerate(both(B, oracle, specs)[0]):
            rec[j] = (p.mode, p.l_th, p.l_mid, p.w_mid, p.beta, p.w_tail, p.mig_mode, 0)
        buf = torch.from_numpy(rec.view(np.uint8).copy()).cuda()
        check_migration(B, oracle, tr, specs, DI.TAU, DI.KAPPA_LAG, delivered_col=None, cost=DI.COST_S,
                        policies=B.DevicePolicies(buf, len(specs)))
