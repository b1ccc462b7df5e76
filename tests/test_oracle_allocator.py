"""Pins of the allocator oracle (oracle/allocator.py) against what the paper prints and what
queueing theory fixes.  CPU only."""
import math
import os

import numpy as np
import pytest

from oracle import allocator as A

GOLD = os.path.join(os.path.dirname(__file__), "golden", "worked_example.txt")


def load_golden():
    g = {}
    with open(GOLD) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                g[k.strip()] = float(v)
    return g


def example(**over):
    g = load_golden()
    # a curve whose largest point meeting 20 ms yields the printed 1700 tokens/s (34 / 0.020)
    kw = dict(tp_total=g["tp_total_tokens_per_min"] / 60.0, l_in=g["l_in"], l_out=g["l_out"],
              ttft_slo=g["ttft_s"], tpot_slo=g["tpot_s"], prefill_max_tps=g["tp_prefill_max_tps"],
              decode_batch=[8, 16, 34, 64], decode_tpot_s=[0.012, 0.015, 0.020, 0.031],
              t_overhead_s=g["t_overhead_s"])
    kw.update(over)
    return kw


def test_worked_example_matches_printed_values():
    g = load_golden()
    r = A.allocate(**example())
    # Formula (13): 28300 - 6144/1.9, printed rounded to 25000
    assert r["tp_prefill_eff"] == pytest.approx(28300 - 6144 / 1.9, rel=1e-15)
    assert abs(r["tp_prefill_eff"] - g["printed_tp_prefill_eff"]) / g["printed_tp_prefill_eff"] < 0.005
    assert r["tp_decode_eff"] == pytest.approx(g["tp_decode_tps"], rel=1e-12)
    assert r["decode_batch"] == 34
    assert abs(r["ratio_pd"] - g["printed_ratio_pd"]) < 0.01
    assert r["n_prefill"] == g["printed_n_prefill"]
    assert r["n_decode"] == g["printed_n_decode"]
    # the real-valued counts behind "three" and "four"
    assert r["n_prefill_real"] == pytest.approx(3.0688, abs=5e-4)
    assert r["n_decode_real"] == pytest.approx(3.7707, abs=5e-4)


def test_printed_counts_need_round_to_nearest():
    # ceil would give 4P4D and floor 3P3D; only nearest reproduces the printed 3P4D
    r = A.allocate(**example())
    assert (math.ceil(r["n_prefill_real"]), math.ceil(r["n_decode_real"])) == (4, 4)
    assert (math.floor(r["n_prefill_real"]), math.floor(r["n_decode_real"])) == (3, 3)
    rc = A.allocate(**example(rounding=1))
    assert (rc["n_prefill"], rc["n_decode"]) == (4, 4)


def test_3p4d_predicted_capacity_close_to_measured():
    g = load_golden()
    r = A.allocate(**example())
    l_in, l_out = g["l_in"], g["l_out"]
    cap = min(3 * r["tp_prefill_eff"] * (l_in + l_out) / l_in,
              4 * r["tp_decode_eff"] * (l_in + l_out) / l_out) * 60 / 1e6
    assert abs(cap - g["printed_3p4d_capacity_mtpm"]) < 0.15


def test_mm1_sojourn_identity():
    # Eq. (13) substituted into lambda = TP/L_in and mu = TPhat/L_in gives 1/(mu-lambda) = TTFT - T_ov
    for tphat, l_in, ttft, tov in [(28300, 6144, 2.0, 0.1), (1e5, 2048, 0.5, 0.0), (5e4, 128, 1.0, 0.25)]:
        tp = A.effective_prefill_throughput(tphat, l_in, ttft, tov)
        mu = A.service_rate(tphat, l_in)
        lam = tp / l_in
        assert A.mm1_sojourn(mu, lam) == pytest.approx(ttft - tov, rel=1e-12)
        rho = A.utilisation(lam, mu)
        assert 0 < rho < 1
        assert tphat * rho == pytest.approx(tp, rel=1e-12)          # Eq. (11)


def test_balance_and_ratio_identities():
    r = A.allocate(**example())
    g = load_golden()
    assert r["n_prefill_real"] / r["n_decode_real"] == pytest.approx(r["ratio_pd"], rel=1e-13)
    t_p = g["l_in"] / (r["tp_prefill_eff"] * r["n_prefill_real"])   # Eq. (2) per request
    t_d = g["l_out"] / (r["tp_decode_eff"] * r["n_decode_real"])    # Eq. (3) per request
    assert t_p == pytest.approx(t_d, rel=1e-13)                      # Eq. (4)
    # Eq. (1): N_req (L_in+L_out) / T_total with T_total = t_p per request
    assert (g["l_in"] + g["l_out"]) / t_p == pytest.approx(g["tp_total_tokens_per_min"] / 60, rel=1e-13)


def test_ratio_independent_of_total_throughput():
    a = A.allocate(**example(tp_total=1e4))
    b = A.allocate(**example(tp_total=7e5))
    assert a["ratio_pd"] == b["ratio_pd"]


def test_monotone_in_total_throughput_and_slos():
    prev = (0, 0)
    for tp in np.linspace(1e3, 4e5, 200):
        r = A.allocate(**example(tp_total=float(tp)))
        cur = (r["n_prefill"], r["n_decode"])
        assert cur[0] >= prev[0] and cur[1] >= prev[1]
        prev = cur
    prev = None
    for ttft in np.linspace(0.4, 10.0, 100):        # looser TTFT -> higher TP_prefill -> fewer P
        r = A.allocate(**example(ttft_slo=float(ttft)))
        if prev is not None:
            assert r["n_prefill"] <= prev["n_prefill"]
            assert r["tp_prefill_eff"] >= prev["tp_prefill_eff"]
        prev = r
    # a curve whose b/TPOT rises with b: looser TPOT -> fewer D
    curve_b = [1, 2, 4, 8, 16, 32, 64, 128]
    curve_t = [0.010, 0.0105, 0.011, 0.012, 0.014, 0.019, 0.03, 0.05]
    prev = None
    for tpot in np.linspace(0.010, 0.06, 60):
        r = A.allocate(**example(tpot_slo=float(tpot), decode_batch=curve_b, decode_tpot_s=curve_t))
        if prev is not None:
            assert r["n_decode"] <= prev["n_decode"]
        prev = r


def test_higher_peak_gives_higher_utilisation_at_same_ttft():
    lo = A.effective_prefill_throughput(20000, 6144, 2.0, 0.1) / 20000
    hi = A.effective_prefill_throughput(40000, 6144, 2.0, 0.1) / 40000
    assert hi > lo


def test_decode_point_selection_rules():
    # inclusive bound, unsorted input, duplicates keep the smaller TPOT, non-monotone curve
    b, t, tp = A.decode_operating_point([16, 4, 8, 8, 32], [0.03, 0.01, 0.025, 0.02, 0.019], 0.02)
    assert (b, t) == (32, 0.019) and tp == 32 / 0.019
    b, t, _ = A.decode_operating_point([4, 8], [0.01, 0.02], 0.02)
    assert b == 8
    with pytest.raises(A.TPOTInfeasible):
        A.decode_operating_point([4, 8], [0.03, 0.04], 0.02)


def test_infeasible_and_invalid_inputs():
    with pytest.raises(A.TTFTInfeasible):
        A.allocate(**example(ttft_slo=0.1))              # T_s = 0
    with pytest.raises(A.TTFTInfeasible):
        A.allocate(**example(ttft_slo=0.1 + 6144 / 28300))  # bare compute time equals T_s
    with pytest.raises(ValueError):
        A.allocate(**example(tp_total=-1.0))
    with pytest.raises(ValueError):
        A.allocate(**example(l_in=float("nan")))
    with pytest.raises(ValueError):
        A.allocate(**example(decode_batch=[], decode_tpot_s=[]))


def test_rounding_rule():
    assert A.round_count(0.2) == 1 and A.round_count(2.5) == 3 and A.round_count(2.4999) == 2
    assert A.round_count(3.5) == 4      # half up, not banker's
    assert A.round_count(2.0, 1) == 2 and A.round_count(2.0000001, 1) == 3 and A.round_count(0.1, 1) == 1


def test_fifo_replay_brute_force_and_mm1_limit():
    # brute force: event-by-event simulation with an explicit queue
    rng = np.random.default_rng(3)
    arr = np.cumsum(rng.exponential(1.0, 200))
    srv = rng.exponential(0.7, 200)
    t, free_at, ref = 0.0, 0.0, []
    for a, s in zip(arr, srv):
        start = max(a, free_at)
        free_at = start + s
        ref.append(free_at - a)
    assert np.allclose(A.fifo_replay(arr, srv), ref, rtol=0, atol=1e-12)
    # long run with exponential service converges to 1/(mu - lambda)
    n, lam, mu = 400000, 0.6, 1.0
    rng = np.random.default_rng(11)
    arr = np.cumsum(rng.exponential(1 / lam, n))
    srv = rng.exponential(1 / mu, n)
    mean = float(np.mean(A.fifo_replay(arr, srv)))
    assert mean == pytest.approx(A.mm1_sojourn(mu, lam), rel=0.03)
    # Pollaczek-Khinchine reduces to M/M/1 for exponential service (E[S^2] = 2/mu^2)
    assert A.mg1_sojourn(lam, 1 / mu, 2 / mu ** 2) == pytest.approx(A.mm1_sojourn(mu, lam), rel=1e-12)
    # ... and to the M/D/1 value for constant service
    assert A.mg1_sojourn(0.5, 1.0, 1.0) == pytest.approx(1.0 + 0.5 / (2 * 0.5), rel=1e-12)


# ---- queue-model variants -------------------------------------------------------------------------

def brute_batched(arrivals, batch_service, max_batch):
    """Event-by-event simulation with an explicit queue, written independently of the oracle's loop."""
    n = len(arrivals)
    done = [None] * n
    queue, t, nxt, busy_until, serving = [], 0.0, 0, None, []
    while any(d is None for d in done):
        # next event: an arrival or the end of the running batch
        ta = arrivals[nxt] if nxt < n else math.inf
        tb = busy_until if busy_until is not None else math.inf
        if tb <= ta:
            t = tb
            for j in serving:
                done[j] = t - arrivals[j]
            serving, busy_until = [], None
        else:
            t = ta
            queue.append(nxt)
            nxt += 1
            while nxt < n and arrivals[nxt] == t:
                queue.append(nxt)
                nxt += 1
        if busy_until is None and queue:
            serving, queue = queue[:max_batch], queue[max_batch:]
            busy_until = t + batch_service[len(serving) - 1]
    return done


def test_batched_replay_against_event_simulation_and_unbatched():
    rng = np.random.default_rng(3)
    for trial in range(40):
        n = int(rng.integers(1, 60))
        arr = np.cumsum(rng.exponential(1.0, n)).tolist()
        if trial % 5 == 0:
            arr = sorted(round(a, 0) for a in arr)              # ties in arrival time
        mb = int(rng.integers(1, 5))
        bs = np.cumsum(rng.uniform(0.2, 1.5, mb)).tolist()      # longer batches take longer
        got = A.fifo_replay_batched(arr, bs, mb)
        ref = brute_batched(arr, bs, mb)
        assert np.allclose(got, ref, rtol=0, atol=1e-12), trial
    arr = np.cumsum(rng.exponential(0.7, 200)).tolist()
    assert A.fifo_replay_batched(arr, [0.6], 1) == A.fifo_replay(arr, [0.6] * 200)


def test_batching_never_hurts_when_a_batch_costs_no_more_than_its_requests_in_turn():
    rng = np.random.default_rng(4)
    arr = np.cumsum(rng.exponential(0.5, 3000)).tolist()
    one = np.mean(A.fifo_replay_batched(arr, [0.45], 1))
    three = np.mean(A.fifo_replay_batched(arr, [0.45, 0.9, 1.35], 3))      # exactly additive cost
    sub = np.mean(A.fifo_replay_batched(arr, [0.45, 0.8, 1.1], 3))         # batching is cheaper
    assert sub < three
    assert sub < one


def test_dp_groups_reduce_to_eq13_and_keep_the_mm1_identity():
    tp, l_in, ttft, tov = 28300.0, 6144.0, 2.0, 0.1
    assert A.effective_prefill_throughput_dp(tp, l_in, ttft, tov, 1) == A.effective_prefill_throughput(tp, l_in, ttft, tov)
    for g in (2, 4, 8):
        total = A.effective_prefill_throughput_dp(tp, l_in, ttft, tov, g)
        lam_g, mu_g = (total / g) / l_in, (tp / g) / l_in       # per-group rates, Eq. (9)
        assert abs(A.mm1_sojourn(mu_g, lam_g) - (ttft - tov)) < 1e-9
        assert total < A.effective_prefill_throughput(tp, l_in, ttft, tov)   # each split queue idles more
    with pytest.raises(A.TTFTInfeasible):
        A.effective_prefill_throughput_dp(tp, l_in, ttft, tov, 16)           # 28300/16 < 6144/1.9


def test_stage_allocation_reduces_to_eqs_5_6_and_balances_every_stage():
    # the worked example's two stages
    real, cnt = A.allocate_stages(5e6 / 60.0, 6144.0, 512.0, [6144.0, 512.0], [25066.315789473683, 1700.0])
    ref = A.allocate(5e6 / 60.0, 6144.0, 512.0, 2.0, 0.02, 28300.0, [34], [0.02], 0.1)
    assert real[0] == ref["n_prefill_real"] and real[1] == ref["n_decode_real"] and cnt == [3, 4]
    # three stages (encode: 2 images per request at 40 images/s per instance): stage times equal, Eq. (4)
    tp_total, l_in, l_out = 2.0e5, 3000.0, 400.0
    work, tps = [2.0, 3000.0, 400.0], [40.0, 21000.0, 1500.0]
    real, cnt = A.allocate_stages(tp_total, l_in, l_out, work, tps, rounding=1)
    req_rate = tp_total / (l_in + l_out)
    for w, t, n in zip(work, tps, real):
        assert abs(req_rate * w / (t * n) - 1.0) < 1e-12      # each stage exactly saturated
    assert cnt == [math.ceil(n) for n in real]
    with pytest.raises(ValueError):
        A.allocate_stages(tp_total, l_in, l_out, [1.0], [1.0, 2.0])


def test_kv_transfer_overhead_closed_forms_and_effect_on_the_worked_example():
    """The modelled overhead of Eq. (8): hand-computed byte counts, linearity in the prompt length,
    and the paper's worked example recovered when the model is set to give its 100 ms."""
    # 8B-shaped model: 32 layers x 2 (K and V) x 8 kv heads x 128 x 2 bytes = 131072 bytes per token
    t = A.kv_transfer_overhead(6144, 32, 8, 128, 2, 50e9)
    assert t == pytest.approx(6144 * 131072 / 50e9, rel=1e-15)
    assert t == pytest.approx(0.016106127, rel=1e-6)
    # an 8-bit cache halves the variable part, the fixed part stays
    assert A.kv_transfer_overhead(6144, 32, 8, 128, 1, 50e9, 0.01) == pytest.approx(0.01 + t / 2, rel=1e-15)
    assert A.kv_transfer_overhead(0, 32, 8, 128, 2, 50e9, 0.03) == 0.03
    assert A.kv_transfer_overhead(2 * 6144, 32, 8, 128, 2, 50e9) == pytest.approx(2 * t, rel=1e-15)
    # a link rate that makes the 6144-token transfer take 100 ms reproduces the example's Eq. (13)
    bw = 6144 * 131072 / 0.1
    tov = A.kv_transfer_overhead(6144, 32, 8, 128, 2, bw)
    assert tov == pytest.approx(0.1, rel=1e-15)
    assert A.effective_prefill_throughput(28300.0, 6144.0, 2.0, tov) == pytest.approx(25066.3, abs=0.05)
    # a larger overhead always lowers the effective prefill throughput (Eq. (13))
    tp = [A.effective_prefill_throughput(28300.0, 6144.0, 2.0, A.kv_transfer_overhead(6144, 32, 8, 128, 2, r))
          for r in (5e9, 10e9, 50e9, 400e9)]
    assert tp == sorted(tp)
