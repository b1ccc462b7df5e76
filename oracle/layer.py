"""numpy front end of the C layer oracle (oracle/layer_oracle.c).

TEST INFRASTRUCTURE ONLY.  Only tests/, the smoke check and the bench's
cpu_baseline leg may import this module; it imports nothing from the GPU
package.  Arrays are fp32; the C code accumulates in double.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


class _Cfg(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ff", C.c_int32), ("n_experts", C.c_int32),
                ("top_k", C.c_int32), ("act8", C.c_int32), ("rms_eps", C.c_double), ("rope_base", C.c_double)]


_WNAMES = ["g_attn", "w_q", "w_k", "w_v", "w_o", "g_ffn", "w_gate", "w_up", "w_down", "w_router"]


class _Wts(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _WNAMES]


def lib():
    global _lib
    if _lib is None:
        path = _build.build()
        _lib = C.CDLL(path)
        _lib.orc_prefill.restype = C.c_int
        _lib.orc_decode_step.restype = C.c_int
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


class Layer:
    """One decoder layer: configuration + fp32 weights (dict of numpy arrays)."""

    def __init__(self, cfg: dict, weights: dict):
        self.cfg = dict(cfg)
        self.c = _Cfg(cfg["d_model"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"],
                      cfg["d_ff"], cfg.get("n_experts", 0), cfg.get("top_k", 0), 0,
                      float(cfg.get("rms_eps", 1e-6)), float(cfg.get("rope_base", 10000.0)))
        self.w = {}
        self.cw = _Wts()
        for n in _WNAMES:
            a = weights.get(n)
            if a is None:
                setattr(self.cw, n, None)
            else:
                self.w[n] = _f32(a)
                setattr(self.cw, n, self.w[n].ctypes.data)

    @property
    def d(self):
        return self.c.d_model

    def call_cfg(self, act8: bool):
        """The configuration of one call.  act8 is the caller's statement that THIS call quantises the
        input rows of its four projections (rounded to bf16, then like act_quantise_rows); pass weights
        from quantise_layer_weights with it.  Which calls of a layer quantise is for the caller to say."""
        c = _Cfg.from_buffer_copy(self.c)
        c.act8 = int(bool(act8))
        return c


class KVCache:
    """fp32 cache [n_slots][Hkv][max_len][hd] for keys (rotated) and values, plus lengths."""

    def __init__(self, layer: Layer, n_slots: int, max_len: int, fp8_scales=None):
        """fp8_scales = (k_scale, v_scale): the cache holds 8-bit E4M3 numbers with these static
        scales (every stored element reads back as scale * fp8(x / scale)); None: exact storage."""
        c = layer.c
        self.k = np.zeros((n_slots, c.n_kv_heads, max_len, c.head_dim), np.float32)
        self.v = np.zeros_like(self.k)
        self.lens = np.zeros(n_slots, np.int32)
        self.max_len = max_len
        self.fp8 = 0 if fp8_scales is None else 1
        self.k_scale, self.v_scale = (1.0, 1.0) if fp8_scales is None else map(float, fp8_scales)

    def q(self):
        return C.c_int(self.fp8), C.c_double(self.k_scale), C.c_double(self.v_scale)

    def set(self, slot, k, v):
        """k, v: [Hkv, len, hd] already-rotated keys and values."""
        n = k.shape[1]
        kk, vv = _f32(k).copy(), _f32(v).copy()
        if self.fp8:
            lib().orc_cache_quantise(_p(kk), C.c_size_t(kk.size), C.c_double(self.k_scale))
            lib().orc_cache_quantise(_p(vv), C.c_size_t(vv.size), C.c_double(self.v_scale))
        self.k[slot, :, :n] = kk
        self.v[slot, :, :n] = vv
        self.lens[slot] = n


def prefill(layer: Layer, x, cu_seqlens, router_logits=None, rows=None, cache: KVCache = None,
            slots=None, return_experts=False, act8=False):
    x = _f32(x)
    T, d = x.shape
    cu = _i32(cu_seqlens)
    n_seqs = len(cu) - 1
    rl = None if router_logits is None else _f32(router_logits)
    rows_a = None if rows is None else _i32(rows)
    n_out = T if rows is None else len(rows_a)
    out = np.zeros((n_out, d), np.float32)
    k = max(layer.c.top_k, 1)
    eidx = np.full((n_out, k), -1, np.int32)
    sl = None if slots is None else _i32(slots)
    rc = lib().orc_prefill(C.byref(layer.call_cfg(act8)), C.byref(layer.cw), _p(x), C.c_int(T), C.c_int(n_seqs),
                           _p(cu), _p(rl), _p(rows_a), C.c_int(n_out), _p(sl),
                           _p(cache.k) if cache is not None and sl is not None else None,
                           _p(cache.v) if cache is not None and sl is not None else None,
                           _p(cache.lens) if cache is not None and sl is not None else None,
                           C.c_int(cache.max_len if cache is not None else 0), _p(out), _p(eidx),
                           *(cache.q() if cache is not None else (C.c_int(0), C.c_double(1.0), C.c_double(1.0))))
    if rc != 0:
        raise ValueError(f"orc_prefill failed rc={rc}")
    return (out, eidx) if return_experts else out


def decode_step(layer: Layer, x, slots, cache: KVCache, router_logits=None, return_experts=False, act8=False):
    x = _f32(x)
    B, d = x.shape
    sl = _i32(slots)
    rl = None if router_logits is None else _f32(router_logits)
    out = np.zeros((B, d), np.float32)
    k = max(layer.c.top_k, 1)
    eidx = np.full((B, k), -1, np.int32)
    rc = lib().orc_decode_step(C.byref(layer.call_cfg(act8)), C.byref(layer.cw), _p(x), C.c_int(B), _p(sl),
                               _p(cache.k), _p(cache.v), _p(cache.lens), C.c_int(cache.max_len),
                               _p(rl), _p(out), _p(eidx), *cache.q())
    if rc == -2:
        raise OverflowError("KV cache capacity exceeded")
    if rc != 0:
        raise ValueError(f"orc_decode_step failed rc={rc}")
    return (out, eidx) if return_experts else out


def prefill_chunk(layer: Layer, x, cu_seqlens, slots, cache: KVCache, router_logits=None,
                  return_experts=False, act8=False):
    """Chunked prefill: sequence s continues cache slot slots[s]; its rows take the positions
    behind the cached prefix, are appended to the cache and attend over prefix + chunk."""
    x = _f32(x)
    T, d = x.shape
    cu = _i32(cu_seqlens)
    n_seqs = len(cu) - 1
    sl = _i32(slots)
    rl = None if router_logits is None else _f32(router_logits)
    out = np.zeros((T, d), np.float32)
    k = max(layer.c.top_k, 1)
    eidx = np.full((T, k), -1, np.int32)
    rc = lib().orc_prefill_chunk(C.byref(layer.call_cfg(act8)), C.byref(layer.cw), _p(x), C.c_int(T), C.c_int(n_seqs),
                                 _p(cu), _p(rl), _p(sl), _p(cache.k), _p(cache.v), _p(cache.lens),
                                 C.c_int(cache.max_len), _p(out), _p(eidx), *cache.q())
    if rc == -2:
        raise OverflowError("KV cache capacity exceeded")
    if rc != 0:
        raise ValueError(f"orc_prefill_chunk failed rc={rc}")
    return (out, eidx) if return_experts else out


def fp8_e4m3_encode(x):
    """uint8 E4M3 codes of an array (round to nearest even, saturating at +-448)."""
    a = np.ascontiguousarray(x, np.float64).ravel()
    f = lib().orc_fp8_e4m3_encode
    f.restype, f.argtypes = C.c_uint8, [C.c_double]
    return np.array([f(float(v)) for v in a], np.uint8).reshape(np.shape(x))


def fp8_e4m3_decode(codes):
    c = np.ascontiguousarray(codes, np.uint8).ravel()
    f = lib().orc_fp8_e4m3_decode
    f.restype, f.argtypes = C.c_double, [C.c_uint8]
    return np.array([f(int(v)) for v in c], np.float64).reshape(np.shape(codes))


# ---- stand-alone pieces (for pins) -------------------------------------------------------------

def rmsnorm(x, g, eps=1e-6):
    x = _f32(x)
    g = _f32(g)
    y = np.empty_like(x)
    lib().orc_rmsnorm(_p(x), _p(g), C.c_int(x.shape[0]), C.c_int(x.shape[1]), C.c_double(eps), _p(y))
    return y


def linear(x, W):
    x = _f32(x)
    W = _f32(W)
    y = np.empty((x.shape[0], W.shape[0]), np.float32)
    lib().orc_linear(_p(x), _p(W), C.c_int(x.shape[0]), C.c_int(x.shape[1]), C.c_int(W.shape[0]), _p(y))
    return y


W8_NAMES = ("w_q", "w_k", "w_v", "w_o", "w_gate", "w_up", "w_down")


def quantise_rows(W):
    """(W', scales): every row of W (last axis = input features) replaced by s * fp8(w / s) with the
    row's power-of-two scale s (smallest with max|row| / s <= 448)."""
    W = _f32(W).copy()
    K = W.shape[-1]
    n_rows = W.size // K
    scales = np.empty(n_rows, np.float32)
    lib().orc_quantise_rows(_p(W), C.c_int(n_rows), C.c_int(K), _p(scales))
    return W, scales.reshape(W.shape[:-1])


def act_quantise_rows(x):
    """(x', scales, codes) for activation rows: x rounded to bf16, then quantised like a weight row;
    codes are the E4M3 bytes of x / scale."""
    x = _f32(x).copy()
    K = x.shape[-1]
    n_rows = x.size // K
    scales = np.empty(n_rows, np.float32)
    codes = np.empty(x.shape, np.uint8)
    lib().orc_act_quantise_rows(_p(x), C.c_int(n_rows), C.c_int(K), _p(scales), codes.ctypes.data_as(C.c_void_p))
    return x, scales.reshape(x.shape[:-1]), codes


def gemm_e4m3(a_codes, a_scales, b_codes, b_scales):
    """c[m, n] = a_scales[m] b_scales[n] sum_k value(a_codes[m, k]) value(b_codes[n, k]) in float64:
    the product of two row-quantised matrices, written out."""
    table = fp8_e4m3_decode(np.arange(256, dtype=np.uint8))
    A = table[np.asarray(a_codes, np.uint8)] * np.asarray(a_scales, np.float64)[:, None]
    B = table[np.asarray(b_codes, np.uint8)] * np.asarray(b_scales, np.float64)[:, None]
    return A @ B.T


def quantise_layer_weights(weights):
    """The weight set an 8-bit-weight layer computes with: projection matrices quantised row by row,
    norm gains and router unchanged."""
    return {k: (quantise_rows(v)[0] if k in W8_NAMES and v is not None else v) for k, v in weights.items()}


def embed(table, ids):
    """hidden[t] = table[ids[t]]; raises on an id outside the table."""
    table, ids = _f32(table), _i32(ids)
    out = np.empty((ids.shape[0], table.shape[1]), np.float32)
    f = lib().orc_embed
    f.restype = C.c_int
    rc = f(_p(table), _p(ids), C.c_int(ids.shape[0]), C.c_int(table.shape[1]), C.c_int(table.shape[0]), _p(out))
    if rc != 0:
        raise ValueError("token id outside the embedding table")
    return out


def lm_head(hidden, g, W, eps=1e-6):
    """logits = RMSNorm(hidden; g, eps) @ W^T, W [V, d]."""
    hidden, g, W = _f32(hidden), _f32(g), _f32(W)
    out = np.empty((hidden.shape[0], W.shape[0]), np.float32)
    lib().orc_lm_head(_p(hidden), _p(g), _p(W), C.c_int(hidden.shape[0]), C.c_int(hidden.shape[1]),
                      C.c_int(W.shape[0]), C.c_double(eps), _p(out))
    return out


def rope(x, pos, base=10000.0):
    """x [T, H, hd] -> rotated copy."""
    y = _f32(x).copy()
    T, H, hd = y.shape
    pos = _i32(pos)
    lib().orc_rope(_p(y), C.c_int(T), C.c_int(H), C.c_int(hd), _p(pos), C.c_double(base))
    return y


def attention(q, k, v, cu_seqlens):
    """q [T,Hq,hd], k,v [T,Hkv,hd] -> o [T,Hq,hd], causal inside each sequence."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    cu = _i32(cu_seqlens)
    o = np.zeros_like(q)
    lib().orc_attention(_p(q), _p(k), _p(v), C.c_int(len(cu) - 1), _p(cu), C.c_int(q.shape[1]),
                        C.c_int(k.shape[1]), C.c_int(q.shape[2]), _p(o))
    return o


def route(logits, top_k):
    logits = _f32(logits)
    T, E = logits.shape
    idx = np.zeros((T, top_k), np.int32)
    wgt = np.zeros((T, top_k), np.float64)
    for t in range(T):
        lib().orc_route_row(_p(logits[t]), C.c_int(E), C.c_int(top_k), _p(idx[t]), _p(wgt[t]))
    return idx, wgt


def ffn_block(layer: Layer, h, router_logits=None, act8=False):
    h = _f32(h)
    rl = None if router_logits is None else _f32(router_logits)
    out = np.empty_like(h)
    lib().orc_ffn_block(C.byref(layer.call_cfg(act8)), C.byref(layer.cw), _p(h), C.c_int(h.shape[0]), _p(rl),
                        _p(out), None)
    return out
