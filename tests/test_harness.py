"""Host logic of the sweep harness (no GPU): the algorithmic work that every roofline fraction is
quoted against, and the search for the largest batch that meets the TPOT target (section "Acquire
decode throughput under TPOT constraints": determine the batch size that satisfies the target TPOT)."""
import numpy as np
import pytest

import pd_inputs as I
from paper_2603_04716_amd import harness as H

LLAMA = I.CONFIGS["llama8b"]
MOE = I.CONFIGS["moe"]


def test_layer_params_of_the_8b_shape():
    attn, ffn = H.layer_params(LLAMA)
    assert attn == 4096 * 6144 + 4096 * 4096 == 41_943_040
    assert ffn == 3 * 4096 * 14336 == 176_160_768
    assert attn + ffn == 218_103_808


@pytest.mark.parametrize("l_in,tflop", [(1024, 3.642), (2048, 3.711), (4096, 3.848)])
def test_prefill_flops_8192_tokens(l_in, tflop):
    """2 P_layer T + sum over sequences of 2 Hq hd L (L + 1), written out with integers."""
    n = 8192 // l_in
    want = 2 * 218_103_808 * 8192 + n * 2 * 32 * 128 * l_in * (l_in + 1)
    got = H.prefill_flops(LLAMA, [l_in] * n)
    assert got == float(want)
    assert abs(got / 1e12 - tflop) < 5e-4          # the figures the roofline fractions are quoted on


def test_prefill_flops_ragged_and_empty_sequences():
    lens = [0, 1, 37, 500]
    want = 2 * 218_103_808 * 538 + sum(2 * 32 * 128 * L * (L + 1) for L in lens)
    assert H.prefill_flops(LLAMA, lens) == float(want)
    assert H.prefill_flops(LLAMA, []) == 0.0


def test_prefill_flops_mixture_of_experts():
    """top-2 of 8 experts: two FFNs per token plus the router product."""
    T = 8192
    want = 2 * (41_943_040 + 2 * 176_160_768) * T + 4 * 2 * 32 * 128 * 2048 * 2049 + 2 * 4096 * 8 * T
    got = H.prefill_flops(MOE, [2048] * 4)
    assert got == float(want)
    # expert products 5.77 TFLOP + attention projections 0.69 + causal attention 0.14 (+ router)
    assert abs(got / 1e12 - (5.772 + 0.687 + 0.1375 + 0.0005)) < 1e-3


@pytest.mark.parametrize("B,gb", [(1, 0.445), (8, 0.503), (64, 0.973), (256, 2.584)])
def test_decode_bytes_kv2048(B, gb):
    """Weights once + every cached row once, the new row included: 2 Hkv hd 2 (S + 1) bytes per sequence."""
    want = 2 * 218_103_808 + B * 2 * 8 * 128 * 2 * 2049
    got = H.decode_bytes(LLAMA, [2048] * B)
    assert got == float(want)
    assert abs(got / 1e9 - gb) < 1.5e-3


def test_decode_bytes_variants():
    lens = [5, 4096, 16383]
    kv = sum(2 * 8 * 128 * (s + 1) for s in lens)
    assert H.decode_bytes(LLAMA, lens) == float(2 * 218_103_808 + 2 * kv)
    assert H.decode_bytes(LLAMA, lens, esz=1) == float(218_103_808 + kv)              # 8-bit weights and cache
    assert H.decode_bytes(LLAMA, lens, esz=2, kv_esz=1) == float(2 * 218_103_808 + kv)
    # mixture of experts: attention weights + the experts actually touched
    assert H.decode_bytes(MOE, [4096] * 8, experts_touched=8) == float(
        2 * (41_943_040 + 8 * 176_160_768) + 8 * 2 * 8 * 128 * 2 * 4097)
    # expected distinct experts at batch 8 with top-2 of 8: 8 (1 - 0.75^8) = 7.2 -> 2.76 GB
    assert abs(H.decode_bytes(MOE, [4096] * 8, experts_touched=8 * (1 - 0.75 ** 8)) / 1e9 - 2.76) < 0.01


def brute_force(tpot, slo, b_max):
    ok = [b for b in range(1, b_max + 1) if tpot(b) <= slo]
    return max(ok) if ok else 0


@pytest.mark.parametrize("b_max", [1, 2, 7, 64, 100, 128, 257])
def test_largest_feasible_batch_monotone_curves_equal_brute_force(b_max):
    rng = np.random.default_rng(b_max)
    for trial in range(40):
        base, slope = rng.uniform(0.001, 0.01), rng.uniform(1e-5, 4e-4)
        steps = np.cumsum(rng.uniform(0, slope, b_max + 1))      # strictly increasing, uneven
        tpot = lambda b: base + steps[b]
        slo = float(rng.choice([base + steps[rng.integers(1, b_max + 1)], 0.02, 0.05, base * 0.5]))
        calls = []

        def measure(b):
            calls.append(b)
            return tpot(b)

        got, t, pts = H.largest_feasible_batch(measure, slo, b_max)
        assert got == brute_force(tpot, slo, b_max)
        assert (t is None) if got == 0 else (t == tpot(got))
        assert len(calls) == len(set(calls))                     # every batch measured once
        assert [b for b, _ in pts] == sorted(calls) and all(v == tpot(b) for b, v in pts)
        assert all(1 <= b <= b_max for b in calls)
        assert len(calls) <= 2 * int(np.ceil(np.log2(b_max + 1))) + 2


def test_largest_feasible_batch_boundaries():
    flat = lambda b: 0.01
    assert H.largest_feasible_batch(flat, 0.01, 128)[0] == 128          # inclusive target, cap reached
    assert H.largest_feasible_batch(flat, 0.009, 128)[:2] == (0, None)   # nothing feasible
    assert H.largest_feasible_batch(lambda b: 0.001 * b, 0.0775, 100)[0] == 77
    assert H.largest_feasible_batch(lambda b: 0.001 * b, 1.0, 100)[0] == 100   # b_max not a power of two


def test_largest_feasible_batch_non_monotone_curve_returns_a_valid_boundary():
    """With a noisy curve there may be several feasible / infeasible boundaries.  What the search
    promises then: the batch it returns was measured feasible, the next one was measured infeasible
    (or is the cap), and no power of two below it was measured infeasible."""
    rng = np.random.default_rng(3)
    for trial in range(60):
        b_max = int(rng.integers(2, 200))
        noise = rng.normal(0, 0.0008, b_max + 2)
        tpot = lambda b: 0.002 + 1.5e-4 * b + noise[b]
        slo = float(rng.uniform(0.003, 0.03))
        got, t, pts = H.largest_feasible_batch(tpot, slo, b_max)
        seen = dict(pts)
        if got == 0:
            assert seen[1] > slo
            continue
        assert seen[got] <= slo and t == seen[got]
        assert got == b_max or seen[got + 1] > slo
        p = 1
        while p <= got:
            assert seen[p] <= slo
            p *= 2
