"""CPU-only checks of the C-ABI library: it loads without a GPU, exports every symbol pd.h
declares, and its host entry points (allocator, FIFO replay, M/M/1) agree with the oracle bit for
bit on the same inputs."""
import math
import os
import re

import numpy as np
import pytest

import paper_2603_04716_amd as pd
from oracle import allocator as A

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "pd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pd_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_symbols()
    assert "pd_prefill" in names and "pd_decode_step" in names and "pd_allocate" in names
    for n in names:
        assert hasattr(pd.lib, n), n
    assert set(names) == set(pd.EXPORTS)


def curve(rng, n):
    b = sorted(set(int(x) for x in rng.integers(1, 512, n)))
    t = np.cumsum(rng.uniform(1e-4, 5e-3, len(b))) + 2e-3
    return b, [float(x) for x in t]


def test_allocator_bit_exact_against_oracle_random():
    rng = np.random.default_rng(0)
    checked = 0
    for i in range(3000):
        b, t = curve(rng, int(rng.integers(1, 12)))
        kw = dict(tp_total=float(rng.uniform(1e3, 1e6)), l_in=float(rng.integers(16, 16384)),
                  l_out=float(rng.integers(1, 4096)), ttft_slo=float(rng.uniform(0.05, 5)),
                  tpot_slo=float(rng.uniform(2e-3, 4e-2)), prefill_max_tps=float(rng.uniform(1e3, 3e5)),
                  decode_batch=b, decode_tpot_s=t, t_overhead_s=float(rng.uniform(0, 0.2)),
                  rounding=int(rng.integers(0, 2)))
        try:
            ref = A.allocate(**kw)
        except A.TTFTInfeasible:
            with pytest.raises(pd.PdError) as e:
                pd.pd_allocate(kw["tp_total"], kw["l_in"], kw["l_out"], kw["ttft_slo"], kw["tpot_slo"],
                               kw["prefill_max_tps"], b, t, kw["t_overhead_s"], kw["rounding"])
            assert e.value.status == pd.PD_ERR_TTFT_INFEASIBLE
            continue
        except A.TPOTInfeasible:
            with pytest.raises(pd.PdError) as e:
                pd.pd_allocate(kw["tp_total"], kw["l_in"], kw["l_out"], kw["ttft_slo"], kw["tpot_slo"],
                               kw["prefill_max_tps"], b, t, kw["t_overhead_s"], kw["rounding"])
            assert e.value.status == pd.PD_ERR_TPOT_INFEASIBLE
            continue
        got = pd.pd_allocate(kw["tp_total"], kw["l_in"], kw["l_out"], kw["ttft_slo"], kw["tpot_slo"],
                             kw["prefill_max_tps"], b, t, kw["t_overhead_s"], kw["rounding"])
        for k, v in ref.items():
            assert got[k] == v, (i, k, got[k], v)      # bit-exact doubles and counts
        checked += 1
    assert checked > 1000


def test_allocator_worked_example_and_unsorted_duplicates():
    got = pd.pd_allocate(5e6 / 60, 6144, 512, 2.0, 0.020, 28300, [64, 34, 8, 16, 34], [0.031, 0.020, 0.012, 0.015, 0.025], 0.1)
    assert (got["n_prefill"], got["n_decode"]) == (3, 4)
    assert got["decode_batch"] == 34 and got["decode_tpot_s"] == 0.020
    assert got["curve_non_monotone"] == 0
    got = pd.pd_allocate(5e6 / 60, 6144, 512, 2.0, 0.020, 28300, [8, 16, 32], [0.012, 0.011, 0.019], 0.1)
    assert got["curve_non_monotone"] == 1 and got["decode_batch"] == 32


def test_allocator_rejects_bad_input_and_leaves_output():
    for args in [(-1, 6144, 512, 2, 0.02, 28300, [8], [0.01]), (1e4, math.nan, 512, 2, 0.02, 28300, [8], [0.01]),
                 (1e4, 6144, 512, 2, 0.02, 28300, [], []), (1e4, 6144, 512, 2, 0.02, 28300, [0], [0.01]),
                 (1e4, 6144, 512, 2, 0.02, 28300, [8], [math.inf])]:
        with pytest.raises(pd.PdError) as e:
            pd.pd_allocate(*args)
        assert e.value.status == pd.PD_ERR_INVALID_ARG
    import ctypes as C
    out = pd.pd_allocation()
    out.n_prefill = 77
    cv = pd.pd_measured_curves(28300.0, 1, (C.c_int32 * 1)(8), (C.c_double * 1)(0.5), 0.0, 0)
    st = pd.lib.pd_allocate(1e4, 6144.0, 512.0, 2.0, 0.02, C.byref(cv), C.byref(out))
    assert st == pd.PD_ERR_TPOT_INFEASIBLE and out.n_prefill == 77
    assert b"TPOT" in pd.lib.pd_last_error()
    assert pd.lib.pd_status_string(st) == b"TPOT target infeasible"


def test_fifo_replay_and_mm1_match_oracle():
    rng = np.random.default_rng(1)
    a = np.cumsum(rng.exponential(1.0, 500))
    s = rng.exponential(0.8, 500)
    assert pd.pd_fifo_replay(a, s) == A.fifo_replay(a, s)
    assert pd.pd_fifo_replay([], []) == []
    with pytest.raises(pd.PdError):
        pd.pd_fifo_replay([1.0, 0.5], [0.1, 0.1])         # arrivals must be ordered
    assert pd.pd_mm1_sojourn(28300, 6144, 2.0) == A.mm1_sojourn(A.service_rate(28300, 6144), 2.0)
    with pytest.raises(pd.PdError) as e:
        pd.pd_mm1_sojourn(28300, 6144, 28300 / 6144)
    assert e.value.status == pd.PD_ERR_TTFT_INFEASIBLE


def test_queue_variants_bit_exact_against_oracle():
    rng = np.random.default_rng(11)
    for trial in range(200):
        n = int(rng.integers(0, 80))
        arr = np.cumsum(rng.exponential(1.0, n)).tolist()
        if trial % 4 == 0:
            arr = sorted(round(a, 0) for a in arr)
        mb = int(rng.integers(1, 6))
        bs = np.cumsum(rng.uniform(0.1, 1.5, mb)).tolist()
        assert pd.pd_fifo_replay_batched(arr, bs, mb) == A.fifo_replay_batched(arr, bs, mb)
    for trial in range(500):
        tp, l_in = float(rng.uniform(1e3, 3e5)), float(rng.integers(16, 16384))
        ttft, tov, g = float(rng.uniform(0.05, 5)), float(rng.uniform(0, 0.2)), int(rng.integers(1, 9))
        try:
            ref = A.effective_prefill_throughput_dp(tp, l_in, ttft, tov, g)
        except A.TTFTInfeasible:
            with pytest.raises(pd.PdError) as e:
                pd.pd_prefill_throughput_dp(tp, l_in, ttft, tov, g)
            assert e.value.status == pd.PD_ERR_TTFT_INFEASIBLE
            continue
        assert pd.pd_prefill_throughput_dp(tp, l_in, ttft, tov, g) == ref
        lam, ms = float(rng.uniform(0.1, 5)), float(rng.uniform(0.01, 0.15))
        ms2 = ms * ms * float(rng.uniform(1.0, 3.0))
        assert pd.pd_mg1_sojourn(lam, ms, ms2) == A.mg1_sojourn(lam, ms, ms2)
        l_in = float(rng.uniform(0, 20000))
        args = (l_in, int(rng.integers(1, 100)), int(rng.integers(1, 65)), int(rng.integers(1, 257)),
                float(rng.choice([1.0, 2.0, 4.0])), float(rng.uniform(1e9, 1e12)), float(rng.uniform(0, 0.2)))
        assert pd.pd_kv_transfer_overhead(*args) == A.kv_transfer_overhead(*args)
    for bad in [(-1.0, 32, 8, 128, 2.0, 5e10, 0.0), (10.0, 0, 8, 128, 2.0, 5e10, 0.0), (10.0, 32, 8, 128, 2.0, 0.0, 0.0),
                (10.0, 32, 8, 128, 2.0, 5e10, -0.1), (float("nan"), 32, 8, 128, 2.0, 5e10, 0.0)]:
        with pytest.raises(pd.PdError) as e:
            pd.pd_kv_transfer_overhead(*bad)
        assert e.value.status == pd.PD_ERR_INVALID_ARG
    with pytest.raises(pd.PdError):
        pd.pd_fifo_replay_batched([2.0, 1.0], [0.5], 1)              # arrivals not sorted
    with pytest.raises(pd.PdError):
        pd.pd_mg1_sojourn(10.0, 0.2, 0.05)                           # utilisation 2


def test_stage_allocation_bit_exact_against_oracle():
    rng = np.random.default_rng(12)
    for trial in range(500):
        n = int(rng.integers(1, 5))
        tp, l_in, l_out = float(rng.uniform(1e3, 1e6)), float(rng.integers(16, 16384)), float(rng.integers(1, 4096))
        work = [float(rng.uniform(1, 8000)) for _ in range(n)]
        tps = [float(rng.uniform(10, 1e5)) for _ in range(n)]
        rounding = int(rng.integers(0, 2))
        assert pd.pd_allocate_stages(tp, l_in, l_out, work, tps, rounding) == \
            tuple(A.allocate_stages(tp, l_in, l_out, work, tps, rounding))
    with pytest.raises(pd.PdError):
        pd.pd_allocate_stages(1e5, 100.0, 10.0, [1.0, -2.0], [5.0, 5.0])


def test_device_entry_points_reject_bad_arguments_before_touching_a_device():
    """Argument checks come first, so they hold on a machine without a GPU: NULL handles and pointers,
    impossible shapes (the non-NULL pointers below are never dereferenced)."""
    import ctypes as C
    lib = pd.lib
    fake = C.c_void_p(0x1000)
    ffake = C.cast(fake, C.POINTER(C.c_float))
    h = C.c_void_p()
    assert lib.pd_layer_create(None, None, C.byref(h)) == pd.PD_ERR_INVALID_ARG
    assert lib.pd_layer_create_w8(None, None, C.byref(h)) == pd.PD_ERR_INVALID_ARG
    assert lib.pd_layer_create_w8a8(None, None, C.byref(h)) == pd.PD_ERR_INVALID_ARG
    assert lib.pd_quantize_rows_e4m3(None, C.c_int32(4), C.c_int32(8), fake, ffake, None) == pd.PD_ERR_INVALID_ARG
    assert lib.pd_quantize_rows_e4m3(fake, C.c_int32(4), C.c_int32(12), fake, ffake, None) == pd.PD_ERR_INVALID_ARG
    assert lib.pd_quantize_rows_e4m3(fake, C.c_int32(-1), C.c_int32(8), fake, ffake, None) == pd.PD_ERR_INVALID_ARG
    args = lambda M, N, K: (fake, ffake, fake, ffake, C.c_int32(M), C.c_int32(N), C.c_int32(K), fake, None)
    assert lib.pd_gemm_e4m3(None, ffake, fake, ffake, C.c_int32(4), C.c_int32(16), C.c_int32(128), fake, None) == pd.PD_ERR_INVALID_ARG
    for M, N, K in ((0, 16, 128), (4, 24, 128), (4, 16, 192), (4, 16, 64)):
        assert lib.pd_gemm_e4m3(*args(M, N, K)) == pd.PD_ERR_SHAPE
    assert b"multiple of 128" in lib.pd_last_error()
    for create in (lib.pd_head_create, lib.pd_head_create_w8):
        assert create(C.c_int32(64), C.c_int32(32), C.c_float(1e-6), C.c_int(pd.PD_BF16), None, None, fake,
                      C.c_int32(4), C.byref(h)) == pd.PD_ERR_INVALID_ARG
        assert create(C.c_int32(0), C.c_int32(32), C.c_float(1e-6), C.c_int(pd.PD_BF16), fake, None, fake,
                      C.c_int32(4), C.byref(h)) == pd.PD_ERR_SHAPE
    assert lib.pd_lm_head(None, fake, C.c_int32(1), fake, None) == pd.PD_ERR_INVALID_ARG
    assert lib.pd_embed(None, fake, C.c_int32(1), fake, None) == pd.PD_ERR_INVALID_ARG
