"""ctypes binding of include/pd.h: same entry-point names, argument marshalling only.

Device tensors are torch tensors (used purely as owners of device memory); their raw pointers and
the current torch stream are handed to the library.  Every step of the path runs inside
libpd_mi355x.so; if that library is missing the import fails.
"""
import ctypes as C
import os

# PyTorch owns the device memory handed to the library, so both must bind to ONE HIP runtime
# instance: load torch (and with it the runtime it ships) before the library resolves its own
# dependency on libamdhip64.
import torch  # noqa: F401

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpd_mi355x.so")

PD_OK = 0
PD_ERR_INVALID_ARG, PD_ERR_SHAPE, PD_ERR_DTYPE, PD_ERR_OOM, PD_ERR_DEVICE = 1, 2, 3, 4, 5
PD_ERR_KV_CAPACITY, PD_ERR_TTFT_INFEASIBLE, PD_ERR_TPOT_INFEASIBLE = 6, 7, 8
PD_F32, PD_BF16 = 0, 1

EXPORTS = [
    "pd_layer_create", "pd_layer_create_w8", "pd_layer_create_w8a8", "pd_quantize_rows_e4m3", "pd_gemm_e4m3", "pd_layer_destroy", "pd_layer_reserve", "pd_kv_cache_create", "pd_kv_cache_create_fp8",
    "pd_kv_cache_destroy", "pd_kv_cache_set", "pd_kv_cache_set_len", "pd_kv_cache_len",
    "pd_kv_cache_set_lens", "pd_kv_cache_get", "pd_profile_enable", "pd_profile_read", "pd_stream_copy", "pd_mfma_probe", "pd_head_create", "pd_head_create_w8", "pd_head_destroy", "pd_embed", "pd_lm_head", "pd_prefill", "pd_prefill_chunk", "pd_decode_step", "pd_decode_step_noalloc", "pd_last_expert_choice", "pd_allocate",
    "pd_fifo_replay", "pd_mm1_sojourn", "pd_fifo_replay_batched", "pd_prefill_throughput_dp", "pd_mg1_sojourn", "pd_kv_transfer_overhead", "pd_allocate_stages", "pd_status_string", "pd_last_error",
]


class PdError(RuntimeError):
    def __init__(self, status, msg):
        super().__init__(f"pd status {status}: {msg}")
        self.status = status


class pd_layer_config(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ff", C.c_int32), ("n_experts", C.c_int32),
                ("top_k", C.c_int32), ("rms_eps", C.c_float), ("rope_base", C.c_float),
                ("dtype", C.c_int32)]


_WNAMES = ["g_attn", "w_q", "w_k", "w_v", "w_o", "g_ffn", "w_gate", "w_up", "w_down", "w_router"]


class pd_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _WNAMES]


class pd_tokens(C.Structure):
    _fields_ = [("hidden", C.c_void_p), ("n_seqs", C.c_int32), ("cu_seqlens", C.POINTER(C.c_int32)),
                ("slots", C.POINTER(C.c_int32)), ("router_logits", C.c_void_p)]


class pd_batch(C.Structure):
    _fields_ = [("hidden", C.c_void_p), ("batch", C.c_int32), ("slots", C.POINTER(C.c_int32)),
                ("router_logits", C.c_void_p)]


class pd_measured_curves(C.Structure):
    _fields_ = [("prefill_max_tps", C.c_double), ("n_decode", C.c_int32),
                ("decode_batch", C.POINTER(C.c_int32)), ("decode_tpot_s", C.POINTER(C.c_double)),
                ("t_overhead_s", C.c_double), ("rounding", C.c_int32)]


class pd_allocation(C.Structure):
    _fields_ = [("tp_prefill_eff", C.c_double), ("tp_decode_eff", C.c_double),
                ("decode_batch", C.c_int32), ("decode_tpot_s", C.c_double),
                ("n_prefill_real", C.c_double), ("n_decode_real", C.c_double),
                ("ratio_pd", C.c_double), ("n_prefill", C.c_int32), ("n_decode", C.c_int32),
                ("curve_non_monotone", C.c_int32)]


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python paper_2603_04716_amd/build.py` "
                      "(there is no fallback path)")
lib = C.CDLL(LIB_PATH)
for _n in EXPORTS:
    getattr(lib, _n)          # raises AttributeError if the library lacks a declared symbol
lib.pd_status_string.restype = C.c_char_p
lib.pd_last_error.restype = C.c_char_p
lib.pd_layer_destroy.restype = None
lib.pd_kv_cache_destroy.restype = None
lib.pd_layer_destroy.argtypes = [C.c_void_p]
lib.pd_kv_cache_destroy.argtypes = [C.c_void_p]
lib.pd_head_destroy.restype = None
lib.pd_head_destroy.argtypes = [C.c_void_p]
lib.pd_allocate.argtypes = [C.c_double] * 5 + [C.POINTER(pd_measured_curves), C.POINTER(pd_allocation)]
lib.pd_mm1_sojourn.argtypes = [C.c_double] * 3 + [C.POINTER(C.c_double)]
lib.pd_mg1_sojourn.argtypes = [C.c_double] * 3 + [C.POINTER(C.c_double)]
lib.pd_kv_transfer_overhead.argtypes = ([C.c_double] + [C.c_int32] * 3 + [C.c_double] * 3 + [C.POINTER(C.c_double)])
lib.pd_prefill_throughput_dp.argtypes = [C.c_double] * 4 + [C.c_int32, C.POINTER(C.c_double)]


def _check(status):
    if status != PD_OK:
        raise PdError(status, lib.pd_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _i32_array(values):
    values = [int(v) for v in values]
    return (C.c_int32 * max(len(values), 1))(*values)


def make_config(cfg: dict) -> pd_layer_config:
    return pd_layer_config(cfg["d_model"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"],
                           cfg["d_ff"], cfg.get("n_experts", 0), cfg.get("top_k", 0),
                           float(cfg.get("rms_eps", 1e-6)), float(cfg.get("rope_base", 10000.0)),
                           PD_BF16 if cfg.get("dtype", "f32") == "bf16" else PD_F32)


# ---- device entry points ---------------------------------------------------------------------------

def pd_layer_create(cfg: dict, weights: dict, w8=False, a8=False):
    """weights: name -> contiguous device torch tensor in the layer's dtype; w8: hold the projection
    matrices as 8-bit codes with per-row power-of-two scales (pd_layer_create_w8); a8: also quantise
    the activations of calls with more than 256 rows (pd_layer_create_w8a8)."""
    w = pd_layer_weights()
    for n in _WNAMES:
        t = weights.get(n)
        setattr(w, n, None if t is None else t.data_ptr())
    h = C.c_void_p()
    c = make_config(cfg)
    create = lib.pd_layer_create_w8a8 if a8 else lib.pd_layer_create_w8 if w8 else lib.pd_layer_create
    _check(create(C.byref(c), C.byref(w), C.byref(h)))
    return h


def pd_layer_destroy(layer):
    lib.pd_layer_destroy(layer)


def pd_quantize_rows_e4m3(x, codes, scales):
    """x [n_rows, n_cols] bf16 -> codes [n_rows, n_cols] uint8, scales [n_rows] fp32 (device tensors)."""
    _check(lib.pd_quantize_rows_e4m3(_ptr(x), C.c_int32(x.shape[0]), C.c_int32(x.shape[1]), _ptr(codes),
                                     C.cast(scales.data_ptr(), C.POINTER(C.c_float)), _stream()))


def pd_gemm_e4m3(a_codes, a_scales, b_codes, b_scales, out):
    """out [M, N] bf16 = (a_scales * value(a_codes [M, K])) (b_scales * value(b_codes [N, K]))^T (device tensors)."""
    M, K = a_codes.shape
    N = b_codes.shape[0]
    fp = C.POINTER(C.c_float)
    _check(lib.pd_gemm_e4m3(_ptr(a_codes), C.cast(a_scales.data_ptr(), fp), _ptr(b_codes), C.cast(b_scales.data_ptr(), fp),
                            C.c_int32(M), C.c_int32(N), C.c_int32(K), _ptr(out), _stream()))


def pd_layer_reserve(layer, max_tokens):
    _check(lib.pd_layer_reserve(layer, C.c_int32(max_tokens)))


def pd_kv_cache_create(layer, max_seqs, max_len):
    h = C.c_void_p()
    _check(lib.pd_kv_cache_create(layer, C.c_int32(max_seqs), C.c_int32(max_len), C.byref(h)))
    return h


def pd_kv_cache_create_fp8(layer, max_seqs, max_len, k_scale, v_scale):
    h = C.c_void_p()
    _check(lib.pd_kv_cache_create_fp8(layer, C.c_int32(max_seqs), C.c_int32(max_len), C.c_double(k_scale),
                                      C.c_double(v_scale), C.byref(h)))
    return h


def pd_kv_cache_destroy(cache):
    lib.pd_kv_cache_destroy(cache)


def pd_kv_cache_set(cache, slot, k, v):
    """k, v: device tensors [Hkv, len, hd]."""
    _check(lib.pd_kv_cache_set(cache, C.c_int32(slot), C.c_int32(k.shape[1]), _ptr(k), _ptr(v), _stream()))


def pd_kv_cache_set_len(cache, slot, length):
    _check(lib.pd_kv_cache_set_len(cache, C.c_int32(slot), C.c_int32(length), _stream()))


def pd_kv_cache_set_lens(cache, slots, lens):
    _check(lib.pd_kv_cache_set_lens(cache, C.c_int32(len(slots)), _i32_array(slots), _i32_array(lens), _stream()))


def pd_profile_enable(layer, on=True):
    _check(lib.pd_profile_enable(layer, C.c_int32(1 if on else 0)))


def pd_profile_read(layer, max_entries=64):
    """[(step name, milliseconds)] of the last pd_prefill / pd_decode_step on this layer."""
    names = (C.c_char_p * max_entries)()
    ms = (C.c_float * max_entries)()
    n = C.c_int32()
    _check(lib.pd_profile_read(layer, C.c_int32(max_entries), names, ms, C.byref(n)))
    return [(names[i].decode(), float(ms[i])) for i in range(n.value)]


def pd_head_create(d_model, vocab, rms_eps, dtype, g_final, w_lm, w_embed=None, max_rows=256, w8=False):
    """dtype: "f32" / "bf16"; tensors are device tensors of that dtype; w8: hold w_lm as 8-bit codes with
    per-row power-of-two scales (pd_head_create_w8)."""
    h = C.c_void_p()
    create = lib.pd_head_create_w8 if w8 else lib.pd_head_create
    _check(create(C.c_int32(d_model), C.c_int32(vocab), C.c_float(rms_eps),
                              C.c_int(PD_BF16 if dtype == "bf16" else PD_F32), _ptr(g_final),
                              None if w_embed is None else _ptr(w_embed), _ptr(w_lm), C.c_int32(max_rows), C.byref(h)))
    return h


def pd_head_destroy(head):
    lib.pd_head_destroy(head)


def pd_embed(head, token_ids, hidden):
    """token_ids: device int32 tensor [T]; hidden: device tensor [T, d_model]."""
    _check(lib.pd_embed(head, _ptr(token_ids), C.c_int32(token_ids.shape[0]), _ptr(hidden), _stream()))


def pd_lm_head(head, hidden, logits):
    _check(lib.pd_lm_head(head, _ptr(hidden), C.c_int32(hidden.shape[0]), _ptr(logits), _stream()))


def pd_stream_copy(dst, src):
    """dst <- src by the library's plain copy kernel (same byte size, multiple of 16)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("pd_stream_copy: size mismatch")
    _check(lib.pd_stream_copy(_ptr(dst), _ptr(src), C.c_int64(nbytes), _stream()))


def pd_mfma_probe(a_vals, b_vals, n_workgroups, iters, sink):
    """Register-only matrix-instruction loop on the given operand values (bf16 tensors of 16384 and 8192 elements)."""
    if a_vals.numel() != 16384 or b_vals.numel() != 8192 or sink.numel() < n_workgroups * 512:
        raise ValueError("pd_mfma_probe: a_vals 16384, b_vals 8192 bf16 elements, sink n_workgroups * 512 floats")
    _check(lib.pd_mfma_probe(_ptr(a_vals), _ptr(b_vals), C.c_int32(n_workgroups), C.c_int32(iters), _ptr(sink), _stream()))


def pd_kv_cache_len(cache, slot):
    n = C.c_int32()
    _check(lib.pd_kv_cache_len(cache, C.c_int32(slot), C.byref(n)))
    return n.value


def pd_kv_cache_get(cache, slot, k, v):
    _check(lib.pd_kv_cache_get(cache, C.c_int32(slot), C.c_int32(k.shape[1]), _ptr(k), _ptr(v), _stream()))


def pd_prefill(layer, hidden, cu_seqlens, out, cache=None, slots=None, router_logits=None):
    cu = _i32_array(cu_seqlens)
    sl = None if slots is None else _i32_array(slots)
    tk = pd_tokens(None if hidden is None else hidden.data_ptr(), len(cu_seqlens) - 1, cu,
                   sl if sl is not None else C.POINTER(C.c_int32)(),
                   None if router_logits is None else router_logits.data_ptr())
    _check(lib.pd_prefill(layer, C.byref(tk), cache, _ptr(out), _stream()))
    return out


def pd_prefill_chunk(layer, hidden, cu_seqlens, slots, cache, out, router_logits=None):
    cu = _i32_array(cu_seqlens)
    sl = _i32_array(slots)
    tk = pd_tokens(None if hidden is None else hidden.data_ptr(), len(cu_seqlens) - 1, cu, sl,
                   None if router_logits is None else router_logits.data_ptr())
    _check(lib.pd_prefill_chunk(layer, C.byref(tk), cache, _ptr(out), _stream()))
    return out


def pd_decode_step(layer, hidden, slots, cache, out, router_logits=None):
    sl = _i32_array(slots)
    bt = pd_batch(hidden.data_ptr(), len(slots), sl,
                  None if router_logits is None else router_logits.data_ptr())
    _check(lib.pd_decode_step(layer, C.byref(bt), cache, _ptr(out), _stream()))
    return out


def pd_decode_step_noalloc(layer, hidden, slots, cache, out, router_logits=None):
    sl = _i32_array(slots)
    bt = pd_batch(hidden.data_ptr(), len(slots), sl,
                  None if router_logits is None else router_logits.data_ptr())
    _check(lib.pd_decode_step_noalloc(layer, C.byref(bt), cache, _ptr(out), _stream()))
    return out


def pd_last_expert_choice(layer, rows, expert_idx):
    _check(lib.pd_last_expert_choice(layer, C.c_int32(rows), _ptr(expert_idx), _stream()))
    return expert_idx


# ---- host entry points -----------------------------------------------------------------------------

def pd_allocate(tp_total_tps, l_in, l_out, ttft_slo_s, tpot_slo_s, prefill_max_tps, decode_batch,
                decode_tpot_s, t_overhead_s=0.0, rounding=0):
    n = len(decode_batch)
    b = _i32_array(decode_batch)
    t = (C.c_double * max(n, 1))(*[float(x) for x in decode_tpot_s])
    cv = pd_measured_curves(float(prefill_max_tps), n, b, t, float(t_overhead_s), int(rounding))
    out = pd_allocation()
    _check(lib.pd_allocate(float(tp_total_tps), float(l_in), float(l_out), float(ttft_slo_s),
                           float(tpot_slo_s), C.byref(cv), C.byref(out)))
    return {f[0]: getattr(out, f[0]) for f in pd_allocation._fields_}


def pd_fifo_replay(arrival_s, service_s):
    n = len(arrival_s)
    a = (C.c_double * max(n, 1))(*[float(x) for x in arrival_s])
    s = (C.c_double * max(n, 1))(*[float(x) for x in service_s])
    o = (C.c_double * max(n, 1))()
    _check(lib.pd_fifo_replay(C.c_int32(n), a, s, o))
    return [o[i] for i in range(n)]


def pd_mm1_sojourn(prefill_max_tps, l_in, lambda_rps):
    t = C.c_double()
    _check(lib.pd_mm1_sojourn(float(prefill_max_tps), float(l_in), float(lambda_rps), C.byref(t)))
    return t.value


def pd_fifo_replay_batched(arrival_s, batch_service_s, max_batch):
    n = len(arrival_s)
    a = (C.c_double * max(n, 1))(*[float(x) for x in arrival_s])
    bs = (C.c_double * max(len(batch_service_s), 1))(*[float(x) for x in batch_service_s])
    o = (C.c_double * max(n, 1))()
    if len(batch_service_s) < max_batch:
        raise ValueError("pd_fifo_replay_batched: batch_service_s shorter than max_batch")
    _check(lib.pd_fifo_replay_batched(C.c_int32(n), a, C.c_int32(max_batch), bs, o))
    return [o[i] for i in range(n)]


def pd_prefill_throughput_dp(prefill_max_tps, l_in, ttft_slo_s, t_overhead_s, dp_groups):
    t = C.c_double()
    _check(lib.pd_prefill_throughput_dp(float(prefill_max_tps), float(l_in), float(ttft_slo_s),
                                        float(t_overhead_s), C.c_int32(dp_groups), C.byref(t)))
    return t.value


def pd_mg1_sojourn(lambda_rps, mean_service_s, mean_service_sq_s2):
    t = C.c_double()
    _check(lib.pd_mg1_sojourn(float(lambda_rps), float(mean_service_s), float(mean_service_sq_s2), C.byref(t)))
    return t.value


def pd_kv_transfer_overhead(l_in, n_layers, n_kv_heads, head_dim, bytes_per_elem, link_bytes_per_s, fixed_s=0.0):
    t = C.c_double()
    _check(lib.pd_kv_transfer_overhead(float(l_in), C.c_int32(n_layers), C.c_int32(n_kv_heads), C.c_int32(head_dim),
                                       float(bytes_per_elem), float(link_bytes_per_s), float(fixed_s), C.byref(t)))
    return t.value


def pd_allocate_stages(tp_total_tps, l_in, l_out, work_per_request, stage_tps, rounding=0):
    n = len(work_per_request)
    if len(stage_tps) != n:
        raise ValueError("pd_allocate_stages: list lengths differ")
    w = (C.c_double * max(n, 1))(*[float(x) for x in work_per_request])
    t = (C.c_double * max(n, 1))(*[float(x) for x in stage_tps])
    real = (C.c_double * max(n, 1))()
    cnt = (C.c_int32 * max(n, 1))()
    _check(lib.pd_allocate_stages(C.c_int32(n), C.c_double(tp_total_tps), C.c_double(l_in), C.c_double(l_out),
                                  w, t, C.c_int32(rounding), real, cnt))
    return [real[i] for i in range(n)], [cnt[i] for i in range(n)]
