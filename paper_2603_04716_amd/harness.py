"""Host-side measurement harness: turns timings of pd_prefill / pd_decode_step into the curves
the allocation model consumes.

  maximum prefill throughput  TPhat(L_in) = T / (n_layers * t_layer)         (section "Acquire prefill
                                                                             throughput under TTFT constraints")
  TPOT(B) = n_layers * t_layer(B);  TP_decode(B) = B / TPOT(B)               (section "Acquire decode
                                                                             throughput under TPOT constraints")

Only argument marshalling, timing with events on the launch stream, and bookkeeping happen here;
every arithmetic step of the layer runs inside the library.
"""
import numpy as np
import torch

from . import binding as pd

# algorithmic work of one layer call (masked-out attention is not counted)


def layer_params(cfg):
    d, hq, hkv, hd, f = cfg["d_model"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"], cfg["d_ff"]
    attn = d * (hq + 2 * hkv) * hd + hq * hd * d
    ffn = 3 * d * f
    return attn, ffn


def prefill_flops(cfg, seq_lens):
    attn, ffn = layer_params(cfg)
    T = int(sum(seq_lens))
    k = cfg.get("top_k", 0) if cfg.get("n_experts", 0) else 1
    fl = 2.0 * (attn + k * ffn) * T
    fl += sum(2.0 * cfg["n_q_heads"] * cfg["head_dim"] * L * (L + 1) for L in seq_lens)
    if cfg.get("n_experts", 0):
        fl += 2.0 * cfg["d_model"] * cfg["n_experts"] * T
    return fl


def decode_bytes(cfg, kv_lens, experts_touched=None, esz=2, kv_esz=None):
    """Weights touched once + every cached key/value row once (the new row included); kv_esz:
    bytes per cached element when it differs from the weights' (1 for the 8-bit cache)."""
    kv_esz = esz if kv_esz is None else kv_esz
    attn, ffn = layer_params(cfg)
    n_ffn = experts_touched if cfg.get("n_experts", 0) else 1
    w = (attn + n_ffn * ffn) * esz
    kv = sum(2 * cfg["n_kv_heads"] * cfg["head_dim"] * kv_esz * (int(s) + 1) for s in kv_lens)
    return float(w + kv)


def _dev(a, dtype):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if dtype == "bf16" else t.contiguous()


class Layer:
    """Device copy of one seeded layer plus timing helpers."""

    def __init__(self, cfg, weights, w8=False, a8=False):
        self.cfg = cfg
        self.dtype = cfg["dtype"]
        self.tdtype = torch.bfloat16 if self.dtype == "bf16" else torch.float32
        dev_w = {k: _dev(v, self.dtype) for k, v in weights.items()}
        self.h = pd.pd_layer_create(cfg, dev_w, w8=w8 or a8, a8=a8)
        del dev_w
        torch.cuda.empty_cache()
        self.caches = []

    def close(self):
        for c in self.caches:
            pd.pd_kv_cache_destroy(c)
        self.caches = []
        pd.pd_layer_destroy(self.h)

    def new_cache(self, n_slots, max_len, fp8_scales=None):
        """fp8_scales = (k_scale, v_scale): the cache holds 8-bit E4M3 codes with these static scales."""
        if fp8_scales is None:
            c = pd.pd_kv_cache_create(self.h, n_slots, max_len)
        else:
            c = pd.pd_kv_cache_create_fp8(self.h, n_slots, max_len, *fp8_scales)
        self.caches.append(c)
        return c

    def free_cache(self, c):
        self.caches.remove(c)
        pd.pd_kv_cache_destroy(c)

    # ---- prefill ------------------------------------------------------------------------------------
    def time_prefill(self, x, cu_seqlens, iters=5, warmup=2, router_logits=None):
        """Mean milliseconds of one pd_prefill call (events on the launch stream)."""
        out = torch.empty_like(x)
        pd.pd_layer_reserve(self.h, x.shape[0])
        for _ in range(warmup):
            pd.pd_prefill(self.h, x, cu_seqlens, out, router_logits=router_logits)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(iters):
            pd.pd_prefill(self.h, x, cu_seqlens, out, router_logits=router_logits)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    # ---- decode --------------------------------------------------------------------------------------
    def fill_cache(self, cache, kv_lens, k, v):
        """Every slot i gets the first kv_lens[i] positions of the (shared) k, v tensors."""
        for i, n in enumerate(kv_lens):
            pd.pd_kv_cache_set(cache, i, k[:, :int(n)].contiguous(), v[:, :int(n)].contiguous())

    def make_decode_step(self, cache, x, kv_lens, router_logits=None, use_graph=True):
        """Returns run() that rewinds the slots to kv_lens (untimed) and then executes ONE decode
        step, timed with events on the launch stream; run() returns milliseconds."""
        B = x.shape[0]
        slots = list(range(B))
        lens = [int(n) for n in kv_lens]
        out = torch.empty_like(x)
        pd.pd_layer_reserve(self.h, B)
        for _ in range(2):                       # warm-up also grows the library's scratch buffers
            pd.pd_kv_cache_set_lens(cache, slots, lens)
            pd.pd_decode_step(self.h, x, slots, cache, out, router_logits)
        torch.cuda.synchronize()
        graph = None
        if use_graph:
            pd.pd_kv_cache_set_lens(cache, slots, lens)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                pd.pd_decode_step(self.h, x, slots, cache, out, router_logits)
            torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

        def run():
            pd.pd_kv_cache_set_lens(cache, slots, lens)
            e0.record()
            if graph is not None:
                graph.replay()
            else:
                pd.pd_decode_step(self.h, x, slots, cache, out, router_logits)
            e1.record()
            e1.synchronize()
            return e0.elapsed_time(e1)

        run.out = out
        run.graph = graph
        return run


def median(xs):
    return float(np.median(np.asarray(xs, np.float64)))


def decode_curve(layer, cache, batches, kv_len, x_all, iters=10, router_logits=None, use_graph=True):
    """[(B, ms per layer step)] for uniform KV length kv_len (cache slots already filled)."""
    pts = []
    for B in batches:
        run = layer.make_decode_step(cache, x_all[:B].contiguous(), [kv_len] * B,
                                     None if router_logits is None else router_logits[:B].contiguous(),
                                     use_graph)
        pts.append((B, median([run() for _ in range(iters)])))
    return pts


def largest_feasible_batch(measure_tpot_s, tpot_slo_s, b_max):
    """Largest integer batch in [1, b_max] whose measured TPOT meets the target: powers of two
    first, then bisection between the last feasible and the first infeasible batch.
    measure_tpot_s(B) -> seconds.  Returns (B, tpot, all measured points) or (0, None, points)."""
    pts = {}

    def m(b):
        if b not in pts:
            pts[b] = measure_tpot_s(b)
        return pts[b]

    lo, hi = 0, None
    b = 1
    while b <= b_max:
        if m(b) <= tpot_slo_s:
            lo = b
            if b == b_max:
                break
            b = min(2 * b, b_max)
        else:
            hi = b
            break
    if hi is not None:
        while hi - lo > 1:
            mid = (lo + hi) // 2
            if m(mid) <= tpot_slo_s:
                lo = mid
            else:
                hi = mid
    return lo, (pts[lo] if lo else None), sorted(pts.items())
