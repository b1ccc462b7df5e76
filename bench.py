#!/usr/bin/env python3
"""Benchmark of the P/D hot path on one MI355X.

One "step" is one pass of the whole path on the Llama-8B-shaped bf16 layer: a prefill of 8192
tokens (4 sequences of 2048; back-to-back calls, median per-call time), decode steps at every batch of the sweep 1..320 over a
2048-token KV cache, and the allocation model on the curves just measured (per-layer times
scaled by 32 layers).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # dense bf16 matrix peak of MI355X
HBM_PEAK_GBPS = 8000.0
N_LAYERS = 32
L_IN, N_SEQ = 2048, 4              # prefill workload: 4 x 2048 = 8192 tokens
KV_LEN = 2048
# powers of two, refined around the batch where the 20 ms TPOT line is crossed, and past it, so that the
# largest feasible batch is set by the TPOT target and not by the end of the sweep
BATCHES = [1, 2, 4, 8, 16, 32, 64, 128, 192, 224, 256, 272, 288, 320]
TTFT_SLO, TPOT_SLO, L_OUT = 2.0, 0.020, 512.0
PREFILL_REPS = 12                  # back-to-back prefill calls per step (each the full 8192 tokens); median
DECODE_REPS = 3                    # decode steps per batch size per step; median
# Fabric-side traffic (L2 misses: fetched + written bytes) of one launch of the dominant kernel, from
# the FETCH_SIZE / WRITE_SIZE counters scaled by a plain copy (paper_2603_04716_amd/traffic_probe.py).
# Valid only for the kernel source the counters were taken on.
TRAFFIC = {"source": os.path.join("paper_2603_04716_amd", "csrc", "gemm_mfma.hip"),
           "sha256": "f1c3318cdf941103c39b45af982604ebc15103bbdc17a1d66b7331c2e1057cdc",
           "bytes_per_launch": 3054.4e6}


def counted_traffic():
    import hashlib
    try:
        with open(os.path.join(ROOT, TRAFFIC["source"]), "rb") as f:
            same = hashlib.sha256(f.read()).hexdigest() == TRAFFIC["sha256"]
    except OSError:
        same = False
    return TRAFFIC["bytes_per_launch"] if same else None


def cpu_baseline(cfg, weights):
    """The oracle, as it stands, timed on a bounded sample: prefill of 2 x 2048 tokens (two of the
    step's four sequences) through the full 8B-shaped layer on the host cores."""
    import numpy as np
    import pd_inputs as I
    from oracle import layer as O
    n = 2 * L_IN
    x = I.hidden(n, cfg["d_model"], seed=99, dtype="bf16")
    L = O.Layer(cfg, weights)
    t0 = time.perf_counter()
    O.prefill(L, x, np.array([0, n // 2, n], np.int32))
    dt = time.perf_counter() - t0
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    cores = min(cores, os.cpu_count() or cores)
    return {"value": n / (dt * N_LAYERS), "unit": "prefill tokens/s (32-layer model)", "cores": cores,
            "kind": "oracle", "sample": f"prefill of 2x{n // 2} tokens through the full 8B-shaped layer, {dt:.1f} s"}


def fp8_section(cfg, weights, x, cu, kd, vd):
    """The same layer with 8-bit (E4M3) weights, activations (calls of more than 256 rows) and KV cache:
    prefill rate, decode curve and the allocation they give.  Reported beside the bf16 figures, never
    as `value`."""
    import torch
    import pd_inputs as I
    import paper_2603_04716_amd as pd
    from paper_2603_04716_amd import harness as H
    layer = H.Layer(cfg, weights, a8=True)
    T = x.shape[0]
    t_pre = layer.time_prefill(x, cu, iters=10, warmup=12)   # the clock settles over the first calls after a pause
    batches = sorted(set(BATCHES + [320, 384, 448, 512, 576]))
    bmax = max(batches)
    cache = layer.new_cache(bmax, KV_LEN + 8, fp8_scales=(0.5, 0.125))
    layer.fill_cache(cache, [KV_LEN] * bmax, kd, vd)
    xdec = H._dev(I.hidden(bmax, cfg["d_model"], seed=12, dtype="bf16"), "bf16")
    curve, tpot = [], []
    for B in batches:
        run = layer.make_decode_step(cache, xdec[:B].contiguous(), [KV_LEN] * B)
        ms = H.median([run() for _ in range(7)])
        tpot.append(N_LAYERS * ms * 1e-3)
        # bytes a step must read: codes of the weights (the bf16 copy for 129 .. 256 rows), 8-bit cache
        by = H.decode_bytes(cfg, [KV_LEN] * B, esz=2 if 128 < B <= 256 else 1, kv_esz=1)
        curve.append({"batch": B, "ms_per_layer": round(ms, 4), "tpot_ms": round(N_LAYERS * ms, 3),
                      "tok_s": round(B / (N_LAYERS * ms * 1e-3), 1),
                      "hbm_frac": round(by / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)})
    tp_hat = T / (N_LAYERS * t_pre * 1e-3)
    alloc = pd.pd_allocate(5e6 / 60.0, float(L_IN), L_OUT, TTFT_SLO, TPOT_SLO, tp_hat, batches, tpot)
    star = next(c for c in curve if c["batch"] == alloc["decode_batch"])
    fl = H.prefill_flops(cfg, [L_IN] * N_SEQ)
    layer.close()
    return {"what": "E4M3 weights (power-of-two row scales), E4M3 activations in calls of more than 256 rows, "
                    "E4M3 KV cache (static scales); fp32 accumulation",
            "prefill": {"ms_per_layer": round(t_pre, 4), "tok_s_model": round(tp_hat, 1),
                        "tflops": round(fl / (t_pre * 1e-3) / 1e12, 1),
                        "mfma_frac_of_8bit_peak": round(fl / (t_pre * 1e-3) / 1e12 / 5000.0, 4)},
            "decode": {"max_feasible_batch": alloc["decode_batch"], "tpot_ms": star["tpot_ms"], "tok_s": star["tok_s"],
                       "curve": curve},
            "allocation": {k2: alloc[k2] for k2 in ("n_prefill", "n_decode", "ratio_pd", "tp_prefill_eff", "tp_decode_eff")}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-fp8", action="store_true", help="skip the 8-bit section reported beside the bf16 figures")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the other configurations reported beside the headline (prefill at 8 x 1024 and 2 x 4096, "
                         "long-context decode at KV 4096 / 8192 / 16384)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path uses no second device and no collectives; "
              "run it with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import pd_inputs as I
    import paper_2603_04716_amd as pd
    from paper_2603_04716_amd import harness as H

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    cfg = I.CONFIGS["llama8b"]
    weights = I.layer_weights(cfg)
    layer = H.Layer(cfg, weights)
    T = L_IN * N_SEQ
    x = H._dev(I.hidden(T, cfg["d_model"], seed=10, dtype="bf16"), "bf16")
    out = torch.empty_like(x)
    cu = [L_IN * i for i in range(N_SEQ + 1)]
    pd.pd_layer_reserve(layer.h, T)

    # decode state: every slot holds the same seeded N(0,1) keys / values
    bmax = max(BATCHES)
    cache = layer.new_cache(bmax, KV_LEN + 8)
    k, v = I.kv_fill(cfg["n_kv_heads"], KV_LEN, cfg["head_dim"], seed=11, dtype="bf16")
    kd, vd = H._dev(k, "bf16"), H._dev(v, "bf16")
    layer.fill_cache(cache, [KV_LEN] * bmax, kd, vd)
    xdec = H._dev(I.hidden(bmax, cfg["d_model"], seed=12, dtype="bf16"), "bf16")
    runs = {B: layer.make_decode_step(cache, xdec[:B].contiguous(), [KV_LEN] * B, use_graph=not args.no_graph)
            for B in BATCHES}
    torch.cuda.synchronize()

    prof = {}            # step name -> list of ms (prefill call)
    dec_prof = {}        # (B, name) -> list of ms (un-graphed profiled decode step, outside the timed region)

    def one_step(record):
        # prefill: PREFILL_REPS back-to-back calls with an event after each (the sustained regime of
        # a prefill instance; the first calls after a pause run below the settled clock).  Every other
        # call also has the library's per-kernel events on: those give the kernel durations, the
        # calls without them give the rate, so that event gaps stay out of it.
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(PREFILL_REPS + 1)]
        entries, plain = [], []
        ev[0].record()
        for i in range(PREFILL_REPS):
            profiled = i % 2 == 1
            if profiled:
                pd.pd_profile_enable(layer.h, True)
            pd.pd_prefill(layer.h, x, cu, out)
            ev[i + 1].record()
            if profiled:
                entries += pd.pd_profile_read(layer.h)
                pd.pd_profile_enable(layer.h, False)
            else:
                plain.append(i)
        ev[-1].synchronize()
        t_pre = H.median([ev[i].elapsed_time(ev[i + 1]) for i in plain])
        t_dec = {B: H.median([runs[B]() for _ in range(DECODE_REPS)]) for B in BATCHES}
        # allocation model on the curves just measured (instance = 32 layers of this layer)
        tp_hat = T / (N_LAYERS * t_pre * 1e-3)
        tpot = [N_LAYERS * t_dec[B] * 1e-3 for B in BATCHES]
        alloc = pd.pd_allocate(5e6 / 60.0, float(L_IN), L_OUT, TTFT_SLO, TPOT_SLO, tp_hat, BATCHES, tpot)
        if record:
            for name, ms in entries:
                prof.setdefault(name, []).append(ms)
        return t_pre, t_dec, alloc

    for _ in range(args.warmup):
        one_step(False)
    torch.cuda.synchronize()
    t_pre_all, t_dec_all, alloc = [], {B: [] for B in BATCHES}, None
    t0 = time.perf_counter()
    for _ in range(args.steps):
        t_pre, t_dec, alloc = one_step(True)
        t_pre_all.append(t_pre)
        for B in BATCHES:
            t_dec_all[B].append(t_dec[B])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # per-kernel durations of a decode step (events between kernels; not part of the timed region)
    slots_all = list(range(bmax))
    pd.pd_profile_enable(layer.h, True)
    for B in (1, 8, 64, 256):
        for _ in range(3):
            pd.pd_kv_cache_set_lens(cache, slots_all[:B], [KV_LEN] * B)
            pd.pd_decode_step(layer.h, xdec[:B].contiguous(), slots_all[:B], cache, runs[B].out)
            for name, ms in pd.pd_profile_read(layer.h):
                dec_prof.setdefault((B, name), []).append(ms)
    pd.pd_profile_enable(layer.h, False)

    med = H.median
    t_pre = med(t_pre_all)
    t_dec = {B: med(t_dec_all[B]) for B in BATCHES}
    prefill_tps_layer = T / (t_pre * 1e-3)
    prefill_tps = prefill_tps_layer / N_LAYERS
    fl = H.prefill_flops(cfg, [L_IN] * N_SEQ)
    curve = []
    for B in BATCHES:
        by = H.decode_bytes(cfg, [KV_LEN] * B)
        curve.append({"batch": B, "ms_per_layer": round(t_dec[B], 4), "tpot_ms": round(N_LAYERS * t_dec[B], 3),
                      "tok_s": round(B / (N_LAYERS * t_dec[B] * 1e-3), 1),
                      "hbm_gbps": round(by / (t_dec[B] * 1e-3) / 1e9, 1),
                      "hbm_frac": round(by / (t_dec[B] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)})
    b_star = alloc["decode_batch"]
    star = next(c for c in curve if c["batch"] == b_star)

    # dominant kernel of the step: the fused gate/up + SwiGLU GEMM of the prefill pass
    d, f = cfg["d_model"], cfg["d_ff"]
    gu_ms = float(np.mean(prof["gate_up_swiglu"]))   # average launch over the timed region
    gu_flops = 2.0 * T * (2 * f) * d
    kernels = {}
    gemm_flops = {"qkv_proj": 2.0 * T * (cfg["n_q_heads"] + 2 * cfg["n_kv_heads"]) * cfg["head_dim"] * d,
                  "o_proj_residual": 2.0 * T * d * cfg["n_q_heads"] * cfg["head_dim"],
                  "gate_up_swiglu": gu_flops, "down_residual": 2.0 * T * d * f,
                  "prefill_attention": N_SEQ * 2.0 * cfg["n_q_heads"] * cfg["head_dim"] * L_IN * (L_IN + 1)}
    for name, ms in prof.items():
        e = {"ms": round(med(ms), 4)}
        if name in gemm_flops:
            e["tflops"] = round(gemm_flops[name] / (med(ms) * 1e-3) / 1e12, 1)
            e["mfma_frac"] = round(e["tflops"] / MFMA_BF16_PEAK_TFLOPS, 4)
        kernels["prefill." + name] = e
    kv_bytes = lambda B: 2.0 * cfg["n_kv_heads"] * cfg["head_dim"] * 2 * (KV_LEN + 1) * B
    attn_p, ffn_p = H.layer_params(cfg)
    w_bytes = {"qkv_proj": 2.0 * d * (cfg["n_q_heads"] + 2 * cfg["n_kv_heads"]) * cfg["head_dim"],
               "o_proj_residual": 2.0 * d * cfg["n_q_heads"] * cfg["head_dim"],
               "gate_up_swiglu": 4.0 * d * f, "down_residual": 2.0 * d * f}
    for (B, name), ms in dec_prof.items():
        e = {"ms": round(med(ms), 4)}
        by = kv_bytes(B) if name == "decode_attention" else w_bytes.get(name)
        if by:
            e["gbps"] = round(by / (med(ms) * 1e-3) / 1e9, 1)
            e["hbm_frac"] = round(e["gbps"] / HBM_PEAK_GBPS, 4)
        kernels[f"decode_b{B}." + name] = e

    line = {
        "metric": "prefill tok/s & decode tok/s at max TPOT-feasible batch; % MFMA/HBM roofline",
        "value": round(prefill_tps, 1),
        "unit": "prefill tokens/s (32-layer model, one GPU)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall / args.steps * 1e3, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "llama8b-shaped layer, bf16: prefill 4x2048 tokens; decode batch 1..320 at KV 2048; "
                               "per-layer time x32", "n_layers_scaling": N_LAYERS, "l_in": L_IN, "kv_len": KV_LEN,
                   "ttft_slo_s": TTFT_SLO, "tpot_slo_s": TPOT_SLO, "l_out": L_OUT, "decode_graph": not args.no_graph,
                   "prefill_calls_per_step": PREFILL_REPS, "decode_calls_per_batch_per_step": DECODE_REPS,
                   "timing": "median of per-call event times"},
        "prefill": {"ms_per_layer": round(t_pre, 4), "tok_s_per_layer": round(prefill_tps_layer, 1),
                    "tok_s_model": round(prefill_tps, 1), "tflops": round(fl / (t_pre * 1e-3) / 1e12, 1),
                    "mfma_frac": round(fl / (t_pre * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)},
        "decode": {"max_feasible_batch": b_star, "tpot_ms": star["tpot_ms"], "tok_s": star["tok_s"],
                   "hbm_gbps": star["hbm_gbps"], "hbm_frac": star["hbm_frac"], "curve": curve},
        "allocation": {k2: alloc[k2] for k2 in ("n_prefill", "n_decode", "ratio_pd", "tp_prefill_eff", "tp_decode_eff")},
        "roofline": {"bound": "mfma", "kernel": "gemm_mfma_kernel (gate/up + SwiGLU, M=8192 N=28672 K=4096)",
                     "achieved": round(gu_flops / (gu_ms * 1e-3) / 1e12, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(gu_flops / (gu_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                     "traffic": counted_traffic(), "traffic_unit": "bytes per launch (L2 <-> fabric, counters)",
                     "algorithmic_bytes": 2.0 * (T * d + 2 * f * d + T * f), "avg_launch_ms": round(gu_ms, 4)},
        "kernels": kernels,
    }
    if not args.no_extra:
        # what the matrix pipe alone sustains on operands distributed like this benchmark's (a loop of
        # nothing but MFMAs on registers, same run): the launch runs at the chip's power limit, which
        # depends on the operand values, so this is context for `frac`, which stays against the published peak
        from paper_2603_04716_amd import mfma_ceiling_probe as MC
        ceil_tf = MC.sustained_tflops(*MC.benchmark_operands(), iters=60000, reps=5, warmup=2)
        line["roofline"]["mfma_only_loop_on_these_operand_values"] = {
            "tflops": round(ceil_tf, 1), "achieved_over_it": round(line["roofline"]["achieved"] / ceil_tf, 4)}
        # the benchmark's other single-GPU configurations, measured by the same harness on the same layer
        # (reported beside the headline, never as `value`)
        from paper_2603_04716_amd import experiments as X
        pd.pd_kv_cache_destroy(cache)
        layer.caches.remove(cache)
        del runs
        torch.cuda.empty_cache()
        line["prefill_vs_l_in"] = X.prefill_points(cfg, layer, x, iters=8, warmup=6)
        line["long_context"] = X.longctx_cases(cfg, layer, modes=("uniform",), reps=5)
    layer.close()
    if not args.no_fp8:
        line["fp8"] = fp8_section(cfg, weights, x, cu, kd, vd)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(cfg, weights)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
