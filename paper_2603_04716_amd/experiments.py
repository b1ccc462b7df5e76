"""Measurement runs that feed (and check) the allocation model, on one GPU.

    python -m paper_2603_04716_amd.experiments prefill      # max prefill throughput vs L_in
    python -m paper_2603_04716_amd.experiments longctx      # decode TPOT curves at KV 4096..16384, uniform + ragged,
                                                            # largest batch meeting TPOT 20/50/100 ms
    python -m paper_2603_04716_amd.experiments queue        # Poisson arrivals served FIFO by the GPU prefill,
                                                            # mean TTFT vs the M/M/1 prediction of Eq. (12)
    python -m paper_2603_04716_amd.experiments moe          # 8-expert top-2 layer: prefill + decode sweep
    python -m paper_2603_04716_amd.experiments fp8kv        # decode curve over the KV cache held as 8-bit E4M3
                                                            # codes beside the bf16 cache, KV 2048 and 8192
    python -m paper_2603_04716_amd.experiments w8           # small-batch decode with 8-bit projection weights
    python -m paper_2603_04716_amd.experiments operands     # the same prefill call on hidden states of different
                                                            # values (what the operand values cost the clock)
    python -m paper_2603_04716_amd.experiments kvxfer       # KV hand-off: cache export / import per layer, the
                                                            # modelled link, Eq. (13) with that overhead

Each run prints one JSON document.  Inputs are the seeded synthetic draws of pd_inputs.
"""
import json
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import pd_inputs as I  # noqa: E402
from . import binding as pd  # noqa: E402
from . import harness as H  # noqa: E402

N_LAYERS = 32
HBM_PEAK, MFMA_PEAK = 8e12, 2.5e15


def _layer(name):
    cfg = I.CONFIGS[name]
    return cfg, H.Layer(cfg, I.layer_weights(cfg))


def prefill_points(cfg, layer, x, rl=None, iters=10, warmup=3):
    """Maximum prefill throughput of x's tokens cut into sequences of 1024 / 2048 / 4096."""
    T = x.shape[0]
    pts = []
    for l_in in (1024, 2048, 4096):
        cu = I.uniform_cu_seqlens(T // l_in, l_in)
        ms = layer.time_prefill(x, cu, iters=iters, warmup=warmup, router_logits=rl)
        fl = H.prefill_flops(cfg, [l_in] * (T // l_in))
        pts.append({"l_in": l_in, "ms_per_layer": round(ms, 4), "tok_s_model": round(T / (N_LAYERS * ms * 1e-3), 1),
                    "tflops": round(fl / (ms * 1e-3) / 1e12, 1), "mfma_frac": round(fl / (ms * 1e-3) / MFMA_PEAK, 4)})
    return pts


def run_prefill(name="llama8b"):
    cfg, layer = _layer(name)
    T = 8192
    x = H._dev(I.hidden(T, cfg["d_model"], seed=10, dtype="bf16"), "bf16")
    rl = torch.from_numpy(I.router_logits(T, cfg["n_experts"], seed=13)).cuda() if cfg["n_experts"] else None
    pts = prefill_points(cfg, layer, x, rl)
    layer.close()
    return {"experiment": "max prefill throughput vs input length", "layer": name, "tokens": T, "points": pts}


def longctx_cases(cfg, layer, modes=("uniform", "ragged"), reps=7, kv_lengths=(4096, 8192, 16384), bmax=128):
    """Decode TPOT against batch at long KV lengths and, per TPOT target, the largest batch that meets
    it (powers of two, then bisection): section "Acquire decode throughput under TPOT constraints"."""
    hkv, hd, d = cfg["n_kv_heads"], cfg["head_dim"], cfg["d_model"]
    cases = []
    xall = H._dev(I.hidden(bmax, d, seed=12, dtype="bf16"), "bf16")
    for S in kv_lengths:
        cache = layer.new_cache(bmax, S + 8)
        k, v = I.kv_fill(hkv, S, hd, seed=11, dtype="bf16")
        kd, vd = H._dev(k, "bf16"), H._dev(v, "bf16")
        for mode in modes:
            lens_all = np.full(bmax, S, np.int32) if mode == "uniform" else I.ragged_kv_lengths(bmax, S, seed=S)
            layer.fill_cache(cache, lens_all, kd, vd)
            cache_pts = {}

            def tpot(B):
                if B not in cache_pts:
                    run = layer.make_decode_step(cache, xall[:B].contiguous(), lens_all[:B])
                    ms = H.median([run() for _ in range(reps)])
                    cache_pts[B] = ms
                return N_LAYERS * cache_pts[B] * 1e-3

            curve = []
            for B in (1, 2, 4, 8, 16, 32, 64, 128):
                if B > bmax:
                    break
                t = tpot(B)
                by = H.decode_bytes(cfg, lens_all[:B])
                curve.append({"batch": B, "tpot_ms": round(t * 1e3, 3), "tok_s": round(B / t, 1),
                              "hbm_frac": round(by / (t / N_LAYERS) / HBM_PEAK, 4)})
            targets = []
            for slo in (0.020, 0.050, 0.100):
                b, t, _ = H.largest_feasible_batch(tpot, slo, bmax)
                e = {"tpot_slo_ms": slo * 1e3, "max_batch": b}
                if b:
                    by = H.decode_bytes(cfg, lens_all[:b])
                    e.update(tpot_ms=round(t * 1e3, 3), tok_s=round(b / t, 1),
                             hbm_gbps=round(by / (t / N_LAYERS) / 1e9, 1),
                             hbm_frac=round(by / (t / N_LAYERS) / HBM_PEAK, 4), capped=(b == bmax))
                targets.append(e)
            cases.append({"kv_capacity": S, "lengths": mode, "mean_kv": float(np.mean(lens_all)),
                          "curve": curve, "targets": targets})
        layer.free_cache(cache)
        del kd, vd
    return cases


def run_longctx():
    cfg, layer = _layer("llama8b")
    out = {"experiment": "long-context decode: TPOT vs batch, uniform and ragged KV", "cases": longctx_cases(cfg, layer)}
    layer.close()
    return out


def run_queue(n_req=2000):
    cfg, layer = _layer("llama8b")
    d = cfg["d_model"]
    lens = I.request_lengths(n_req, seed=3)
    xbuf = H._dev(I.hidden(int(lens.max()), d, seed=14, dtype="bf16"), "bf16")   # timing is value-independent
    out_buf = torch.empty_like(xbuf)
    pd.pd_layer_reserve(layer.h, int(lens.max()))
    # service time of every request = measured GPU time of its own prefill (x 32 layers)
    uniq = np.unique(lens)
    svc_ms = {}
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for L in uniq:
        L = int(L)
        reps = 3
        pd.pd_prefill(layer.h, xbuf[:L], [0, L], out_buf[:L])
        e0.record()
        for _ in range(reps):
            pd.pd_prefill(layer.h, xbuf[:L], [0, L], out_buf[:L])
        e1.record()
        e1.synchronize()
        svc_ms[L] = e0.elapsed_time(e1) / reps
    service = np.array([N_LAYERS * svc_ms[int(L)] * 1e-3 for L in lens])
    # saturated pass: back-to-back service of the same 2000 requests
    tp_hat = float(lens.sum() / service.sum())
    mean_l = float(lens.mean())
    mu = tp_hat / mean_l                                 # Eq. (9) on the drawn lengths = 1 / mean service
    res = {"experiment": "FIFO prefill queue vs M/M/1", "requests": n_req, "mean_l_in": mean_l,
           "tp_prefill_max_tok_s": round(tp_hat, 1), "mu_req_s": round(mu, 4), "rates": []}
    for f in (0.3, 0.5, 0.7, 0.9):
        lam = f * mu
        arr = I.poisson_arrivals(n_req, lam, seed=int(f * 100))
        soj = pd.pd_fifo_replay(arr, service)
        pred = pd.pd_mm1_sojourn(tp_hat, mean_l, lam)
        pk = pd.pd_mg1_sojourn(lam, float(service.mean()), float(np.mean(service ** 2)))   # Pollaczek-Khinchine
        res["rates"].append({"load": f, "lambda_req_s": round(lam, 4), "mean_ttft_s": round(float(np.mean(soj)), 5),
                             "mm1_pred_s": round(pred, 5), "ratio_measured_over_mm1": round(float(np.mean(soj)) / pred, 4),
                             "mg1_pk_s": round(pk, 5)})
    layer.close()
    return res


def run_moe():
    cfg, layer = _layer("moe")
    d, E = cfg["d_model"], cfg["n_experts"]
    res = run_prefill_on(layer, cfg)
    S, bmax = 4096, 256
    cache = layer.new_cache(bmax, S + 8)
    k, v = I.kv_fill(cfg["n_kv_heads"], S, cfg["head_dim"], seed=11, dtype="bf16")
    layer.fill_cache(cache, [S] * bmax, H._dev(k, "bf16"), H._dev(v, "bf16"))
    xall = H._dev(I.hidden(bmax, d, seed=12, dtype="bf16"), "bf16")
    rl_np = I.router_logits(bmax, E, seed=15)
    rl = torch.from_numpy(rl_np).cuda()
    curve = []
    for B in (1, 2, 4, 8, 16, 32, 64, 128, 256):
        run = layer.make_decode_step(cache, xall[:B].contiguous(), [S] * B, router_logits=rl[:B].contiguous())
        ms = H.median([run() for _ in range(7)])
        top2 = np.argsort(-rl_np[:B], 1, kind="stable")[:, :2]
        touched = len(np.unique(top2))
        by = H.decode_bytes(cfg, [S] * B, experts_touched=touched)
        curve.append({"batch": B, "experts_touched": touched, "ms_per_layer": round(ms, 4),
                      "tpot_ms": round(N_LAYERS * ms, 3), "tok_s": round(B / (N_LAYERS * ms * 1e-3), 1),
                      "hbm_frac": round(by / (ms * 1e-3) / HBM_PEAK, 4)})
    hist = np.bincount(np.argsort(-I.router_logits(8192, E, seed=13), 1, kind="stable")[:, :2].ravel(), minlength=E)
    res.update(decode_kv_len=S, decode_curve=curve, prefill_expert_load=hist.tolist())
    layer.close()
    return res


def run_prefill_on(layer, cfg):
    T, l_in = 8192, 2048
    x = H._dev(I.hidden(T, cfg["d_model"], seed=10, dtype="bf16"), "bf16")
    rl = torch.from_numpy(I.router_logits(T, cfg["n_experts"], seed=13)).cuda()
    cu = I.uniform_cu_seqlens(T // l_in, l_in)
    ms = layer.time_prefill(x, cu, iters=8, warmup=3, router_logits=rl)
    fl = H.prefill_flops(cfg, [l_in] * (T // l_in))
    pd.pd_profile_enable(layer.h, True)
    out = torch.empty_like(x)
    pd.pd_prefill(layer.h, x, cu, out, router_logits=rl)
    steps = pd.pd_profile_read(layer.h)
    pd.pd_profile_enable(layer.h, False)
    return {"experiment": "MoE layer (8 experts, top-2)", "prefill": {
        "tokens": T, "l_in": l_in, "ms_per_layer": round(ms, 4), "tok_s_model": round(T / (N_LAYERS * ms * 1e-3), 1),
        "tflops": round(fl / (ms * 1e-3) / 1e12, 1), "mfma_frac": round(fl / (ms * 1e-3) / MFMA_PEAK, 4),
        "steps_ms": {n: round(t, 4) for n, t in steps}}}


def run_chunk(l_in=8192, chunks=(256, 512, 1024, 2048, 4096, 8192), reps=5, fp8=False):
    """Prefill of one l_in-token prompt chunk by chunk (pd_prefill_chunk against the growing cached
    prefix): throughput against the chunk size.  fp8: 8-bit weights, 8-bit activations in chunks of
    more than 256 tokens, 8-bit cache."""
    cfg = I.CONFIGS["llama8b"]
    layer = H.Layer(cfg, I.layer_weights(cfg), a8=fp8)
    x = H._dev(I.hidden(l_in, cfg["d_model"], seed=10, dtype="bf16"), "bf16")
    out = torch.empty_like(x)
    cache = layer.new_cache(1, l_in, fp8_scales=(0.5, 0.125) if fp8 else None)
    pd.pd_layer_reserve(layer.h, l_in)
    fl = H.prefill_flops(cfg, [l_in])
    pts = []
    for C in chunks:
        def once():
            pd.pd_kv_cache_set_len(cache, 0, 0)
            for a in range(0, l_in, C):
                b = min(l_in, a + C)
                pd.pd_prefill_chunk(layer.h, x[a:b], [0, b - a], [0], cache, out[a:b])
        for _ in range(2):
            once()
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            once()
            e1.record()
            e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        ms = H.median(ts)
        pts.append({"chunk": C, "calls": (l_in + C - 1) // C, "ms_per_layer": round(ms, 4),
                    "tok_s_model": round(l_in / (N_LAYERS * ms * 1e-3), 1),
                    "tflops": round(fl / (ms * 1e-3) / 1e12, 1), "mfma_frac": round(fl / (ms * 1e-3) / MFMA_PEAK, 4)})
    # the same prompt in one unchunked call, for reference
    ms_full = layer.time_prefill(x, [0, l_in], iters=5, warmup=2)
    layer.close()
    return {"experiment": "chunked prefill: throughput vs chunk size" + (" (8-bit weights, activations, cache)" if fp8 else ""),
            "l_in": l_in, "points": pts,
            "unchunked_ms_per_layer": round(ms_full, 4)}


def run_queue_fixed(n_req=2000):
    """The paper's own queue check: a fixed request input length, (a) chunked prefill size equal to
    it (requests served one by one), (b) a chunk several times larger (queued requests are batched
    into one prefill call).  Service times of batches of 1..k requests are measured on the GPU
    (x N_LAYERS), arrivals are Poisson, the queue is replayed in virtual time; mean TTFT beside
    Eq. (12) and the Pollaczek-Khinchine value for the constant service time."""
    cfg, layer = _layer("llama8b")
    d = cfg["d_model"]
    out = {"experiment": "queue check at a fixed input length, chunk = L_in and chunk = k L_in", "requests": n_req,
           "cases": []}
    for l_in, k in ((4096, 3), (6144, 4)):
        x = H._dev(I.hidden(l_in * k, d, seed=10, dtype="bf16"), "bf16")
        svc = []
        for b in range(1, k + 1):
            ms = layer.time_prefill(x[:l_in * b], I.uniform_cu_seqlens(b, l_in), iters=8, warmup=3)
            svc.append(N_LAYERS * ms * 1e-3)
        mu = 1.0 / svc[0]
        case = {"l_in": l_in, "chunk_batched": l_in * k, "batch_service_s": [round(t, 5) for t in svc],
                "tp_prefill_max_tok_s": round(l_in * mu, 1), "mu_req_s": round(mu, 4), "rates": []}
        for f in (0.3, 0.5, 0.7, 0.9):
            lam = f * mu
            arr = I.poisson_arrivals(n_req, lam, seed=int(100 * f) + l_in)
            one = pd.pd_fifo_replay_batched(arr, svc[:1], 1)
            bat = pd.pd_fifo_replay_batched(arr, svc, k)
            mm1 = pd.pd_mm1_sojourn(l_in * mu, l_in, lam)
            pk = pd.pd_mg1_sojourn(lam, svc[0], svc[0] * svc[0])
            case["rates"].append({"load": f, "lambda_req_s": round(lam, 4),
                                  "mean_ttft_chunk_eq_lin_s": round(float(np.mean(one)), 5),
                                  "mean_ttft_chunk_k_lin_s": round(float(np.mean(bat)), 5),
                                  "mm1_pred_s": round(mm1, 5), "md1_pk_s": round(pk, 5),
                                  "ratio_unbatched_over_mm1": round(float(np.mean(one)) / mm1, 4),
                                  "ratio_batched_over_mm1": round(float(np.mean(bat)) / mm1, 4)})
        out["cases"].append(case)
    layer.close()
    return out


def run_stack(n_layers=32, n_weight_sets=4, batches=(1, 8, 64, 256), kv_len=2048, fp8=False):
    """A real stack of n_layers resident layers (distinct device copies of a few seeded weight
    sets, one KV cache per layer), each layer's output feeding the next: measured prefill time and
    TPOT of the whole stack beside n_layers x the single-layer time that the sweeps scale up.
    fp8: the layers hold 8-bit weights, quantise activations in calls of more than 256 rows, and
    the caches hold 8-bit codes, the vocabulary projection holds 8-bit weights."""
    cfg = I.CONFIGS["llama8b"]
    d = cfg["d_model"]
    host_sets = [I.layer_weights(cfg, seed=s0) for s0 in range(n_weight_sets)]
    layers = [H.Layer(cfg, host_sets[i % n_weight_sets], a8=fp8) for i in range(n_layers)]
    del host_sets
    T, l_in = 8192, 2048
    cu = I.uniform_cu_seqlens(T // l_in, l_in)
    x = H._dev(I.hidden(T, d, seed=10, dtype="bf16"), "bf16")
    bufs = [torch.empty_like(x), torch.empty_like(x)]
    for L in layers:
        pd.pd_layer_reserve(L.h, T)
    # the stack's two ends: token embedding in front, final norm + vocabulary projection behind
    vocab = 128256
    hw = I.head_weights(d, vocab, seed=99, dtype="bf16")
    w_lm = H._dev(hw["w_lm"], "bf16")
    head = pd.pd_head_create(d, vocab, cfg["rms_eps"], "bf16", H._dev(hw["g_final"], "bf16"), w_lm, w_lm,
                             max_rows=max(max(batches), T // l_in), w8=fp8)
    del hw, w_lm
    ids = torch.from_numpy(np.random.default_rng(5).integers(0, vocab, T).astype(np.int32)).cuda()
    last_rows = torch.tensor([l_in * (i + 1) - 1 for i in range(T // l_in)], device="cuda")
    logits_p = torch.empty((T // l_in, vocab), dtype=torch.bfloat16, device="cuda")
    xe = torch.empty_like(x)

    def prefill_stack(ends=False):
        src = x
        if ends:
            pd.pd_embed(head, ids, xe)
            src = xe
        for i, L in enumerate(layers):
            pd.pd_prefill(L.h, src, cu, bufs[i & 1])
            src = bufs[i & 1]
        if ends:       # only the last token of each prompt is projected onto the vocabulary
            pd.pd_lm_head(head, src.index_select(0, last_rows), logits_p)

    def timed(fn, reps):
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        return H.median(ts)

    prefill_stack()
    ms_stack = timed(prefill_stack, 5)
    prefill_stack(True)
    ms_model = timed(lambda: prefill_stack(True), 5)
    ms_one = layers[0].time_prefill(x, cu, iters=10, warmup=3)
    res = {"experiment": "resident layer stack vs single layer scaled up" + (" (8-bit weights, activations, cache)" if fp8 else ""),
           "n_layers": n_layers,
           "prefill": {"tokens": T, "l_in": l_in, "stack_ms": round(ms_stack, 3),
                       "single_layer_ms_x_layers": round(ms_one * n_layers, 3),
                       "with_embedding_and_lm_head_ms": round(ms_model, 3),
                       "tok_s_stack": round(T / (ms_stack * 1e-3), 1),
                       "tok_s_scaled": round(T / (ms_one * n_layers * 1e-3), 1)}, "decode": []}
    finite = bool(torch.isfinite(bufs[(n_layers - 1) & 1].float()).all())
    res["prefill"]["output_finite"] = finite

    bmax = max(batches)
    k, v = I.kv_fill(cfg["n_kv_heads"], kv_len, cfg["head_dim"], seed=11, dtype="bf16")
    kd, vd = H._dev(k, "bf16"), H._dev(v, "bf16")
    caches = [L.new_cache(bmax, kv_len + 8, fp8_scales=(0.5, 0.125) if fp8 else None) for L in layers]
    for L, c in zip(layers, caches):
        L.fill_cache(c, [kv_len] * bmax, kd, vd)
    xdec = H._dev(I.hidden(bmax, d, seed=12, dtype="bf16"), "bf16")
    for B in batches:
        slots, lens = list(range(B)), [kv_len] * B
        xb = xdec[:B].contiguous()
        dbuf = [torch.empty_like(xb), torch.empty_like(xb)]

        def rewind():
            for c in caches:
                pd.pd_kv_cache_set_lens(c, slots, lens)

        ids_b = ids[:B].contiguous()
        xeb = torch.empty_like(xb)
        logits = torch.empty((B, vocab), dtype=torch.bfloat16, device="cuda")

        def step(ends=False):
            src = xb
            if ends:
                pd.pd_embed(head, ids_b, xeb)
                src = xeb
            for i, (L, c) in enumerate(zip(layers, caches)):
                pd.pd_decode_step(L.h, src, slots, c, dbuf[i & 1])
                src = dbuf[i & 1]
            if ends:
                pd.pd_lm_head(head, src, logits)

        def graph_time(ends):
            for _ in range(2):
                rewind()
                step(ends)
            rewind()
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step(ends)
            torch.cuda.synchronize()
            ts = []
            for _ in range(3):                   # clocks settle over the first replays after a pause
                rewind()
                graph.replay()
            for _ in range(7):
                rewind()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                graph.replay()
                e1.record()
                e1.synchronize()
                ts.append(e0.elapsed_time(e1))
            del graph
            return H.median(ts)

        tpot = graph_time(False)
        tpot_model = graph_time(True)

        def ends_only():
            pd.pd_embed(head, ids_b, xeb)
            pd.pd_lm_head(head, xb, logits)

        ends_only()
        ends_ms = timed(ends_only, 15)
        one = layers[0].make_decode_step(caches[0], xb, lens)
        ms_one_d = H.median([one() for _ in range(7)])
        # 8-bit mode: one byte per cached element; one byte per weight where the codes are streamed (up to 128 rows)
        by = H.decode_bytes(cfg, lens, esz=1 if (fp8 and B <= 128) else 2, kv_esz=1 if fp8 else None) * n_layers
        res["decode"].append({"batch": B, "tpot_ms_stack": round(tpot, 3),
                              "tpot_ms_scaled": round(ms_one_d * n_layers, 3),
                              "tpot_ms_with_embedding_and_lm_head": round(tpot_model, 3),
                              "embedding_and_lm_head_alone_ms": round(ends_ms, 4),
                              "lm_head_weight_gbps": round((1.0 if (fp8 and B <= 128) else 2.0) * vocab * d / (ends_ms * 1e-3) / 1e9, 1),
                              "logits_finite": bool(torch.isfinite(logits.float()).all()),
                              "tok_s_stack": round(B / (tpot * 1e-3), 1),
                              "hbm_frac_stack": round(by / (tpot * 1e-3) / HBM_PEAK, 4)})
    for L in layers:
        L.close()
    pd.pd_head_destroy(head)
    return res


def run_fp8kv():
    """Decode TPOT curve and largest batch under TPOT 20 ms with the cache in bf16 and as E4M3 codes."""
    cfg, layer = _layer("llama8b")
    hkv, hd, d = cfg["n_kv_heads"], cfg["head_dim"], cfg["d_model"]
    out = {"experiment": "decode over a bf16 vs an 8-bit E4M3 KV cache", "cases": []}
    for S, bmax, batches in ((2048, 512, (64, 128, 256, 320, 384, 512)), (8192, 128, (16, 32, 64, 128))):
        xall = H._dev(I.hidden(bmax, d, seed=12, dtype="bf16"), "bf16")
        k, v = I.kv_fill(hkv, S, hd, seed=11, dtype="bf16")
        kd, vd = H._dev(k, "bf16"), H._dev(v, "bf16")
        for kind in ("bf16", "fp8_e4m3"):
            cache = layer.new_cache(bmax, S + 8, fp8_scales=None if kind == "bf16" else (0.5, 0.125))
            layer.fill_cache(cache, [S] * bmax, kd, vd)
            kv_esz = 2 if kind == "bf16" else 1
            pts = {}

            def tpot(B):
                if B not in pts:
                    run = layer.make_decode_step(cache, xall[:B].contiguous(), [S] * B)
                    pts[B] = H.median([run() for _ in range(7)])
                return N_LAYERS * pts[B] * 1e-3

            curve = []
            for B in batches:
                t = tpot(B)
                by = H.decode_bytes(cfg, [S] * B, kv_esz=kv_esz)
                curve.append({"batch": B, "ms_per_layer": round(pts[B], 4), "tpot_ms": round(t * 1e3, 3),
                              "tok_s": round(B / t, 1), "hbm_frac": round(by / (t / N_LAYERS) / HBM_PEAK, 4)})
            b, t, _ = H.largest_feasible_batch(tpot, 0.020, bmax)
            best = {"tpot_slo_ms": 20.0, "max_batch": b}
            if b:
                best.update(tpot_ms=round(t * 1e3, 3), tok_s=round(b / t, 1), capped=(b == bmax))
            # attention's own share at the largest batch of the curve, from the library's step timers
            B = batches[-1]
            slots = list(range(B))
            o = torch.empty_like(xall[:B])
            pd.pd_profile_enable(layer.h, True)
            att = []
            for _ in range(5):
                pd.pd_kv_cache_set_lens(cache, slots, [S] * B)
                pd.pd_decode_step(layer.h, xall[:B].contiguous(), slots, cache, o)
                torch.cuda.synchronize()
                att.append(dict(pd.pd_profile_read(layer.h))["decode_attention"])
            pd.pd_profile_enable(layer.h, False)
            att_ms = H.median(att)
            kv_bytes = 2.0 * hkv * hd * kv_esz * (S + 1) * B
            out["cases"].append({"kv_len": S, "cache": kind, "curve": curve, "target": best,
                                 "attention": {"batch": B, "ms": round(att_ms, 4),
                                               "cache_gbps": round(kv_bytes / (att_ms * 1e-3) / 1e9, 1)}})
            layer.free_cache(cache)
        del kd, vd, xall
    layer.close()
    return out


def run_w8():
    """Decode up to batch 128 with the projection weights as 8-bit codes beside bf16 weights (both with the
    bf16 cache and, for the 8-bit weights, also the 8-bit cache), KV 2048, with per-step timings."""
    cfg = I.CONFIGS["llama8b"]
    hkv, hd, d = cfg["n_kv_heads"], cfg["head_dim"], cfg["d_model"]
    S, bmax = 2048, 128
    batches = (1, 2, 4, 8, 16, 32, 64, 96, 128)
    host_w = I.layer_weights(cfg)
    xall = H._dev(I.hidden(bmax, d, seed=12, dtype="bf16"), "bf16")
    k, v = I.kv_fill(hkv, S, hd, seed=11, dtype="bf16")
    kd, vd = H._dev(k, "bf16"), H._dev(v, "bf16")
    attn_p, ffn_p = H.layer_params(cfg)
    out = {"experiment": "decode with 8-bit projection weights (skinny kernel <= 16 rows, wide kernel <= 128)",
           "kv_len": S, "cases": []}
    for w8, fp8kv in ((False, False), (True, False), (True, True)):
        layer = H.Layer(cfg, host_w, w8=w8)
        cache = layer.new_cache(bmax, S + 8, fp8_scales=(0.5, 0.125) if fp8kv else None)
        layer.fill_cache(cache, [S] * bmax, kd, vd)
        curve = []
        for B in batches:
            run = layer.make_decode_step(cache, xall[:B].contiguous(), [S] * B)
            ms = H.median([run() for _ in range(9)])
            wbytes = (attn_p + ffn_p) * (1 if (w8 and B <= 128) else 2)
            kvbytes = 2.0 * hkv * hd * (1 if fp8kv else 2) * (S + 1) * B
            curve.append({"batch": B, "ms_per_layer": round(ms, 4), "tpot_ms": round(N_LAYERS * ms, 3),
                          "tok_s": round(B / (N_LAYERS * ms * 1e-3), 1),
                          "hbm_frac": round((wbytes + kvbytes) / (ms * 1e-3) / HBM_PEAK, 4)})
        # per-step timings at B = 8
        B = 8
        slots = list(range(B))
        o = torch.empty_like(xall[:B])
        pd.pd_profile_enable(layer.h, True)
        acc = {}
        for it in range(7):
            pd.pd_kv_cache_set_lens(cache, slots, [S] * B)
            pd.pd_decode_step(layer.h, xall[:B].contiguous(), slots, cache, o)
            torch.cuda.synchronize()
            if it >= 2:
                for n, t in pd.pd_profile_read(layer.h):
                    acc.setdefault(n, []).append(t)
        pd.pd_profile_enable(layer.h, False)
        out["cases"].append({"weights": "e4m3 + row scales" if w8 else "bf16", "cache": "e4m3" if fp8kv else "bf16",
                             "curve": curve, "steps_us_b8": {n: round(1e3 * H.median(t), 1) for n, t in acc.items()}})
        layer.close()
    return out


def run_a8():
    """Prefill with 8-bit weights and 8-bit activations (codes x codes on the matrix cores for calls of
    more than 256 rows) beside the bf16 layer: 8192 tokens at three input lengths, per-step timings at
    4 x 2048, and the mid-sized calls of a chunked prefill."""
    cfg = I.CONFIGS["llama8b"]
    host_w = I.layer_weights(cfg)
    T = 8192
    x = H._dev(I.hidden(T, cfg["d_model"], seed=10, dtype="bf16"), "bf16")
    out = {"experiment": "prefill with 8-bit weights and activations (E4M3 x E4M3, fp32 accumulation)", "cases": []}
    for a8 in (False, True):
        layer = H.Layer(cfg, host_w, a8=a8)
        pts = []
        for l_in in (1024, 2048, 4096):
            cu = I.uniform_cu_seqlens(T // l_in, l_in)
            ms = layer.time_prefill(x, cu, iters=10, warmup=3)
            fl = H.prefill_flops(cfg, [l_in] * (T // l_in))
            pts.append({"l_in": l_in, "ms_per_layer": round(ms, 4), "tok_s_model": round(T / (N_LAYERS * ms * 1e-3), 1),
                        "tflops": round(fl / (ms * 1e-3) / 1e12, 1)})
        mid = []
        for rows in (512, 1024, 2048):
            cu = I.uniform_cu_seqlens(1, rows)
            ms = layer.time_prefill(x[:rows].contiguous(), cu, iters=10, warmup=3)
            mid.append({"tokens": rows, "ms_per_layer": round(ms, 4), "tok_s_model": round(rows / (N_LAYERS * ms * 1e-3), 1)})
        cu = I.uniform_cu_seqlens(4, 2048)
        pd.pd_profile_enable(layer.h, True)
        o = torch.empty_like(x)
        acc = {}
        for it in range(5):
            pd.pd_prefill(layer.h, x, cu, o)
            torch.cuda.synchronize()
            if it >= 2:
                for n, t in pd.pd_profile_read(layer.h):
                    acc.setdefault(n, []).append(t)
        pd.pd_profile_enable(layer.h, False)
        out["cases"].append({"layer": "e4m3 weights and activations" if a8 else "bf16", "points": pts, "single_sequence": mid,
                             "steps_ms_4x2048": {n: round(H.median(t), 4) for n, t in acc.items()}})
        layer.close()
    # the mixture-of-experts layer (8 experts, top-2), 4 x 2048 tokens, given router logits
    mcfg = I.CONFIGS["moe"]
    mw = I.layer_weights(mcfg)
    rl = torch.from_numpy(I.router_logits(T, mcfg["n_experts"], seed=13)).cuda()
    cu = I.uniform_cu_seqlens(4, 2048)
    fl = H.prefill_flops(mcfg, [2048] * 4)
    out["moe"] = []
    for a8 in (False, True):
        layer = H.Layer(mcfg, mw, a8=a8)
        ms = layer.time_prefill(x, cu, iters=8, warmup=3, router_logits=rl)
        pd.pd_profile_enable(layer.h, True)
        o = torch.empty_like(x)
        pd.pd_prefill(layer.h, x, cu, o, router_logits=rl)
        steps = pd.pd_profile_read(layer.h)
        pd.pd_profile_enable(layer.h, False)
        out["moe"].append({"layer": "e4m3 weights and activations" if a8 else "bf16", "ms_per_layer": round(ms, 4),
                           "tok_s_model": round(T / (N_LAYERS * ms * 1e-3), 1), "tflops": round(fl / (ms * 1e-3) / 1e12, 1),
                           "steps_ms": {n: round(t, 4) for n, t in steps}})
        layer.close()
    return out


def run_kvxfer():
    """The KV hand-off from a prefill to a decode instance as far as one GPU shows it: reading a
    sequence's keys and values out of the (blocked) cache into one contiguous buffer and writing
    such a buffer into another cache, per layer; the link itself is the model of
    pd_kv_transfer_overhead.  Then Eq. (13) with the modelled overhead instead of a given scalar."""
    cfg, layer = _layer("llama8b")
    hkv, hd, d = cfg["n_kv_heads"], cfg["head_dim"], cfg["d_model"]
    out = {"experiment": "KV hand-off: cache export / import on the GPU, modelled link, effect on Eq. (13)", "cases": []}
    T = 8192
    x = H._dev(I.hidden(T, d, seed=10, dtype="bf16"), "bf16")
    for l_in in (2048, 6144):
        src, dst = layer.new_cache(2, l_in), layer.new_cache(2, l_in)
        k, v = I.kv_fill(hkv, l_in, hd, seed=11, dtype="bf16")
        kd, vd = H._dev(k, "bf16"), H._dev(v, "bf16")
        pd.pd_kv_cache_set(src, 0, kd, vd)
        kb, vb = torch.empty_like(kd), torch.empty_like(vd)
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        exp_ms, imp_ms = [], []
        for _ in range(9):
            e0.record()
            pd.pd_kv_cache_get(src, 0, kb, vb)
            e1.record()
            pd.pd_kv_cache_set(dst, 1, kb, vb)
            e2.record()
            e2.synchronize()
            exp_ms.append(e0.elapsed_time(e1))
            imp_ms.append(e1.elapsed_time(e2))
        assert torch.equal(kb, kd) and torch.equal(vb, vd)
        layer_bytes = 2.0 * hkv * hd * 2 * l_in
        ex, im = H.median(exp_ms), H.median(imp_ms)
        n_seq = T // l_in if T % l_in == 0 else 1
        cu = I.uniform_cu_seqlens(n_seq, l_in)
        ms = layer.time_prefill(x[:n_seq * l_in].contiguous(), cu, iters=8, warmup=3)
        tp_max = n_seq * l_in / (N_LAYERS * ms * 1e-3)
        case = {"l_in": l_in, "kv_mb_per_layer": round(layer_bytes / 1e6, 2), "export_ms_per_layer": round(ex, 4),
                "import_ms_per_layer": round(im, 4), "export_gbps": round(2 * layer_bytes / (ex * 1e-3) / 1e9, 1),
                "import_gbps": round(2 * layer_bytes / (im * 1e-3) / 1e9, 1),
                "on_gpu_ms_model": round(N_LAYERS * (ex + im), 3), "prefill_max_tok_s": round(tp_max, 1), "links": []}
        for name, bw, esz in (("400 Gb/s, bf16 cache", 50e9, 2.0), ("400 Gb/s, 8-bit cache", 50e9, 1.0),
                              ("100 Gb/s, bf16 cache", 12.5e9, 2.0)):
            tov = pd.pd_kv_transfer_overhead(l_in, N_LAYERS, hkv, hd, esz, bw, N_LAYERS * (ex + im) * 1e-3)
            case["links"].append({"link": name, "t_overhead_ms": round(tov * 1e3, 2),
                                  "tp_prefill_eq13": round(pd.pd_prefill_throughput_dp(tp_max, l_in, 2.0, tov, 1), 1)})
        case["tp_prefill_eq13_no_overhead"] = round(pd.pd_prefill_throughput_dp(tp_max, l_in, 2.0, 0.0, 1), 1)
        out["cases"].append(case)
        layer.free_cache(src)
        layer.free_cache(dst)
    layer.close()
    return out


def run_operands():
    """The same prefill call (4 x 2048 tokens, 8B shape) on hidden states of different values: the work
    and the schedule are identical, only what the matrix pipe toggles differs.  Beside the register-only
    loop of mfma_ceiling_probe this separates what the kernels' schedule costs from what the operand
    values cost (the clock the chip sustains under its power limit)."""
    cfg, layer = _layer("llama8b")
    T, l_in = 8192, 2048
    x = H._dev(I.hidden(T, cfg["d_model"], seed=10, dtype="bf16"), "bf16")
    cu = I.uniform_cu_seqlens(T // l_in, l_in)
    fl = H.prefill_flops(cfg, [l_in] * (T // l_in))
    d, f = cfg["d_model"], cfg["d_ff"]
    gemm_fl = {"qkv_proj": 2.0 * T * (cfg["n_q_heads"] + 2 * cfg["n_kv_heads"]) * cfg["head_dim"] * d,
               "o_proj_residual": 2.0 * T * d * d, "gate_up_swiglu": 4.0 * T * f * d, "down_residual": 2.0 * T * d * f}
    out = {"experiment": "prefill of 4 x 2048 tokens against the values of the hidden states", "cases": []}
    for name, xx in (("N(0,1) (the benchmark's input)", x), ("all zeros", torch.zeros_like(x)),
                     ("all ones", torch.ones_like(x)), ("N(0,1) again", x)):
        ms = layer.time_prefill(xx, cu, iters=20, warmup=10)
        pd.pd_profile_enable(layer.h, True)
        o = torch.empty_like(xx)
        acc = {}
        for _ in range(4):
            pd.pd_prefill(layer.h, xx, cu, o)
            torch.cuda.synchronize()
            for n, t in pd.pd_profile_read(layer.h):
                acc.setdefault(n, []).append(t)
        pd.pd_profile_enable(layer.h, False)
        out["cases"].append({"hidden_states": name, "ms_per_layer": round(ms, 4),
                             "pflops": round(fl / (ms * 1e-3) / 1e15, 3),
                             "kernels_us": {n: round(H.median(v) * 1e3, 1) for n, v in acc.items()},
                             "gemm_pflops": {n: round(gemm_fl[n] / (H.median(acc[n]) * 1e-3) / 1e15, 3) for n in gemm_fl}})
    layer.close()
    return out


def main():
    which = sys.argv[1] if len(sys.argv) > 1 else "prefill"
    fn = {"prefill": run_prefill, "longctx": run_longctx, "queue": run_queue, "moe": run_moe,
          "chunk": run_chunk, "stack": run_stack, "queue_fixed": run_queue_fixed, "fp8kv": run_fp8kv, "kvxfer": run_kvxfer, "w8": run_w8, "a8": run_a8,
          "operands": run_operands, "stack_fp8": lambda: run_stack(batches=(1, 8, 64, 256, 448), fp8=True),
          "chunk_fp8": lambda: run_chunk(fp8=True)}[which]
    print(json.dumps(fn()))


if __name__ == "__main__":
    main()
