"""Helpers for the GPU parity tests: move seeded numpy inputs to the device in the layer's dtype,
call the C ABI through the binding, bring results back as fp32 numpy."""
import numpy as np
import torch

import paper_2603_04716_amd as pd
import pd_inputs as I

TOL = {"f32": 1e-5, "bf16": 2e-2}     # max-norm relative error bound per dtype


def to_dev(a, dtype):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if dtype == "bf16" else t.contiguous()


def to_np(t):
    return t.detach().float().cpu().numpy()


def relmax(got, ref):
    ref = np.asarray(ref, np.float64)
    return float(np.max(np.abs(np.asarray(got, np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-30))


class GpuLayer:
    def __init__(self, cfg, weights, w8=False, a8=False):
        self.cfg = cfg
        self.dtype = cfg["dtype"]
        self.dev_w = {k: to_dev(v, self.dtype) for k, v in weights.items()}
        self.h = pd.pd_layer_create(cfg, self.dev_w, w8=w8 or a8, a8=a8)
        self.caches = []

    def cache(self, n_slots, max_len, fp8_scales=None):
        if fp8_scales is None:
            c = pd.pd_kv_cache_create(self.h, n_slots, max_len)
        else:
            c = pd.pd_kv_cache_create_fp8(self.h, n_slots, max_len, *fp8_scales)
        self.caches.append(c)
        return c

    def prefill(self, x, cu, cache=None, slots=None, router_logits=None):
        xd = to_dev(x, self.dtype)
        out = torch.empty_like(xd)
        rl = None if router_logits is None else torch.from_numpy(router_logits).cuda().contiguous()
        pd.pd_prefill(self.h, xd, cu, out, cache, slots, rl)
        torch.cuda.synchronize()
        return to_np(out)

    def prefill_chunk(self, x, cu, slots, cache, router_logits=None):
        xd = to_dev(x, self.dtype)
        out = torch.empty_like(xd)
        rl = None if router_logits is None else torch.from_numpy(router_logits).cuda().contiguous()
        pd.pd_prefill_chunk(self.h, xd, cu, slots, cache, out, rl)
        torch.cuda.synchronize()
        return to_np(out)

    def decode(self, x, slots, cache, router_logits=None):
        xd = to_dev(x, self.dtype)
        out = torch.empty_like(xd)
        rl = None if router_logits is None else torch.from_numpy(router_logits).cuda().contiguous()
        pd.pd_decode_step(self.h, xd, slots, cache, out, rl)
        torch.cuda.synchronize()
        return to_np(out)

    def experts(self, rows):
        e = torch.empty((rows, self.cfg["top_k"]), dtype=torch.int32, device="cuda")
        pd.pd_last_expert_choice(self.h, rows, e)
        torch.cuda.synchronize()
        return e.cpu().numpy()

    def close(self):
        for c in self.caches:
            pd.pd_kv_cache_destroy(c)
        pd.pd_layer_destroy(self.h)
        self.caches = []
