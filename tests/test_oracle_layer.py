"""Pins of the C layer oracle against things other than itself: an independent float64 composition
of PyTorch CPU library primitives, brute-force attention, decode == prefill of the extended
sequence, and textbook invariants.  CPU only."""
import numpy as np
import pytest
import torch

import pd_inputs as I
from oracle import layer as O


# ---- independent float64 composition of library routines ----------------------------------------

def torch_act_q(z):
    """Library form of the 8-bit activation rule: rows rounded to bf16, power-of-two scale that keeps
    the row inside +-448, the library's float8_e4m3fn conversion of z / s."""
    zb = z.to(torch.float32).to(torch.bfloat16).to(torch.float64)
    m = zb.abs().amax(dim=-1, keepdim=True)
    s = torch.where(m > 0, 2.0 ** torch.ceil(torch.log2(m / 448.0)), torch.ones_like(m))
    return (zb / s).to(torch.float32).to(torch.float8_e4m3fn).to(torch.float64) * s


def torch_layer(cfg, w, x, cu, router_logits=None, act_q=None):
    f64 = torch.float64
    aq = act_q if act_q is not None else (lambda z: z)
    W = {k: torch.from_numpy(np.asarray(v)).to(f64) for k, v in w.items()}
    x = torch.from_numpy(x).to(f64)
    d, hq, hkv, hd = cfg["d_model"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]

    def norm(a, g):
        return torch.nn.functional.rms_norm(a, (d,), g, cfg["rms_eps"])

    def rot(a, pos):            # a [L, H, hd]
        half = hd // 2
        inv = cfg["rope_base"] ** (-torch.arange(0, half, dtype=f64) * 2.0 / hd)
        ang = pos.to(f64)[:, None] * inv[None, :]
        c, s = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]
        a1, a2 = a[..., :half], a[..., half:]
        return torch.cat([a1 * c - a2 * s, a2 * c + a1 * s], dim=-1)

    y = aq(norm(x, W["g_attn"]))
    q = (y @ W["w_q"].T).view(-1, hq, hd)
    k = (y @ W["w_k"].T).view(-1, hkv, hd)
    v = (y @ W["w_v"].T).view(-1, hkv, hd)
    o = torch.zeros_like(q)
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        if b == a:
            continue
        pos = torch.arange(b - a)
        qs = rot(q[a:b], pos).transpose(0, 1)[None]
        ks = rot(k[a:b], pos).transpose(0, 1)[None].repeat_interleave(hq // hkv, dim=1)
        vs = v[a:b].transpose(0, 1)[None].repeat_interleave(hq // hkv, dim=1)
        os_ = torch.nn.functional.scaled_dot_product_attention(qs, ks, vs, is_causal=True)
        o[a:b] = os_[0].transpose(0, 1)
    h = x + aq(o.reshape(-1, hq * hd)) @ W["w_o"].T
    y2 = norm(h, W["g_ffn"])
    y2r = y2                  # the router reads the unquantised row
    y2 = aq(y2)

    def ffn(z, wg, wu, wd):
        return aq(torch.nn.functional.silu(z @ wg.T) * (z @ wu.T)) @ wd.T

    if cfg.get("n_experts", 0) == 0:
        out = h + ffn(y2, W["w_gate"], W["w_up"], W["w_down"])
    else:
        r = torch.from_numpy(router_logits).to(f64) if router_logits is not None else y2r @ W["w_router"].T
        p = torch.softmax(r, dim=-1)
        tv, ti = torch.topk(p, cfg["top_k"], dim=-1)
        tv = tv / tv.sum(-1, keepdim=True)
        out = h.clone()
        for t in range(x.shape[0]):
            for j in range(cfg["top_k"]):
                e = int(ti[t, j])
                out[t] += tv[t, j] * ffn(y2[t:t + 1], W["w_gate"][e], W["w_up"][e], W["w_down"][e])[0]
    return out.numpy()


def relmax(a, b):
    return float(np.max(np.abs(np.asarray(a, np.float64) - np.asarray(b, np.float64))) / np.max(np.abs(b)))


CASES = [
    dict(),                                              # GQA 4/2
    dict(n_q_heads=4, n_kv_heads=4),                     # MHA
    dict(n_q_heads=8, n_kv_heads=1, head_dim=16),        # MQA
    dict(d_model=96, n_q_heads=6, n_kv_heads=3, head_dim=8, d_ff=80),
]


@pytest.mark.parametrize("over", CASES)
def test_prefill_matches_float64_library_composition(over):
    cfg = I.small_config(**over)
    w = I.layer_weights(cfg, std=0.08)
    cu = np.array([0, 17, 17, 40, 41], np.int32)        # ragged, one empty, one single-token sequence
    x = I.hidden(int(cu[-1]), cfg["d_model"], seed=5)
    got = O.prefill(O.Layer(cfg, w), x, cu)
    ref = torch_layer(cfg, w, x, cu)
    assert relmax(got, ref) < 2e-6          # only the fp32 rounding of stored intermediates differs


def test_moe_matches_float64_library_composition():
    cfg = I.small_config(n_experts=4, top_k=2, d_ff=64)
    w = I.layer_weights(cfg, std=0.08, with_router=True)
    cu = np.array([0, 9, 24], np.int32)
    x = I.hidden(24, cfg["d_model"], seed=6)
    r = I.router_logits(24, 4, seed=8)
    L = O.Layer(cfg, w)
    assert relmax(O.prefill(L, x, cu, router_logits=r), torch_layer(cfg, w, x, cu, r)) < 2e-6
    # router computed from w_router when no logits are handed in
    assert relmax(O.prefill(L, x, cu), torch_layer(cfg, w, x, cu, None)) < 2e-6


# ---- brute force ----------------------------------------------------------------------------------

def test_attention_brute_force_tiny():
    rng = np.random.default_rng(0)
    T, hq, hkv, hd = 13, 4, 2, 8
    q = rng.standard_normal((T, hq, hd)).astype(np.float32)
    k = rng.standard_normal((T, hkv, hd)).astype(np.float32)
    v = rng.standard_normal((T, hkv, hd)).astype(np.float32)
    cu = np.array([0, 5, 13], np.int32)
    got = O.attention(q, k, v, cu)
    ref = np.zeros((T, hq, hd))
    for s in range(2):
        a, b = cu[s], cu[s + 1]
        for h in range(hq):
            S = q[a:b, h].astype(np.float64) @ k[a:b, h // 2].astype(np.float64).T / np.sqrt(hd)
            S = np.where(np.tril(np.ones_like(S)) > 0, S, -np.inf)
            P = np.exp(S - S.max(1, keepdims=True))
            P /= P.sum(1, keepdims=True)
            ref[a:b, h] = P @ v[a:b, h // 2].astype(np.float64)
    assert np.max(np.abs(got - ref)) < 1e-6


# ---- decode == prefill of the extended sequence ---------------------------------------------------

@pytest.mark.parametrize("over", [dict(), dict(n_q_heads=4, n_kv_heads=4), dict(n_experts=4, top_k=2, d_ff=64)])
def test_decode_equals_prefill_of_extended_sequence(over):
    cfg = I.small_config(**over)
    w = I.layer_weights(cfg, std=0.08, with_router=True)
    L = O.Layer(cfg, w)
    lens = [1, 6, 19]
    S_max = 24
    xs = [I.hidden(S_max, cfg["d_model"], seed=20 + i) for i in range(3)]
    cache = O.KVCache(L, n_slots=4, max_len=S_max)
    slots = [2, 0, 3]
    x0 = np.concatenate([xs[i][:lens[i]] for i in range(3)])
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    O.prefill(L, x0, cu, cache=cache, slots=slots)
    assert list(cache.lens[[2, 0, 3]]) == lens
    for step in range(3):                                   # three successive decode steps
        cur = [n + step for n in lens]
        xb = np.stack([xs[i][cur[i]] for i in range(3)])
        got = O.decode_step(L, xb, slots, cache)
        for i in range(3):
            full = O.prefill(L, xs[i][:cur[i] + 1], np.array([0, cur[i] + 1], np.int32))
            assert relmax(got[i], full[-1]) < 1e-6
        assert list(cache.lens[[2, 0, 3]]) == [n + 1 for n in cur]


def test_decode_capacity_error_leaves_state():
    cfg = I.small_config()
    L = O.Layer(cfg, I.layer_weights(cfg))
    cache = O.KVCache(L, 2, 4)
    O.prefill(L, I.hidden(4, cfg["d_model"], 1), np.array([0, 4], np.int32), cache=cache, slots=[1])
    before = cache.k.copy()
    with pytest.raises(OverflowError):
        O.decode_step(L, I.hidden(1, cfg["d_model"], 2), [1], cache)
    assert cache.lens[1] == 4 and np.array_equal(before, cache.k)


# ---- chunked prefill == unchunked prefill -------------------------------------------------------------

@pytest.mark.parametrize("over", [dict(), dict(n_q_heads=4, n_kv_heads=4), dict(n_experts=4, top_k=2, d_ff=64)])
def test_chunked_prefill_equals_unchunked(over):
    cfg = I.small_config(**over)
    w = I.layer_weights(cfg, std=0.08, with_router=True)
    L = O.Layer(cfg, w)
    lens = [13, 1, 22]
    xs = [I.hidden(n, cfg["d_model"], seed=40 + i) for i, n in enumerate(lens)]
    slots = [3, 0, 1]
    # three calls with ragged chunk lengths, one of them empty for a sequence
    plan = [[5, 1, 7], [8, 0, 4], [0, 0, 11]]
    cache = O.KVCache(L, n_slots=4, max_len=24)
    done = [0, 0, 0]
    got = [[] for _ in lens]
    for chunk in plan:
        x = np.concatenate([xs[i][done[i]:done[i] + chunk[i]] for i in range(3)])
        cu = np.concatenate([[0], np.cumsum(chunk)]).astype(np.int32)
        out = O.prefill_chunk(L, x, cu, slots, cache)
        for i in range(3):
            got[i].append(out[cu[i]:cu[i + 1]])
            done[i] += chunk[i]
        assert [int(cache.lens[s]) for s in slots] == done
    full_cache = O.KVCache(L, n_slots=4, max_len=24)
    for i in range(3):
        full = O.prefill(L, xs[i], np.array([0, lens[i]], np.int32), cache=full_cache, slots=[slots[i]])
        assert relmax(np.concatenate(got[i]), full) < 1e-6
        # and against the independent float64 composition of library routines
        ref = torch_layer(cfg, w, xs[i], [0, lens[i]])
        assert relmax(np.concatenate(got[i]), ref) < 2e-6
    for sl, n in zip(slots, lens):                           # the caches hold the same keys and values
        assert np.array_equal(cache.k[sl, :, :n], full_cache.k[sl, :, :n])
        assert np.array_equal(cache.v[sl, :, :n], full_cache.v[sl, :, :n])


def test_chunk_of_one_token_is_a_decode_step_and_empty_prefix_is_a_prefill():
    cfg = I.small_config()
    w = I.layer_weights(cfg, std=0.08)
    L = O.Layer(cfg, w)
    x = I.hidden(12, cfg["d_model"], seed=50)
    a, b = O.KVCache(L, 2, 16), O.KVCache(L, 2, 16)
    p1 = O.prefill(L, x[:9], np.array([0, 4, 9], np.int32), cache=a, slots=[1, 0])
    p2 = O.prefill_chunk(L, x[:9], np.array([0, 4, 9], np.int32), [1, 0], b)
    assert np.array_equal(p1, p2) and np.array_equal(a.k, b.k) and np.array_equal(a.lens, b.lens)
    d1 = O.decode_step(L, x[9:11], [0, 1], a)
    d2 = O.prefill_chunk(L, x[9:11], np.array([0, 1, 2], np.int32), [0, 1], b)
    assert np.array_equal(d1, d2) and np.array_equal(a.k, b.k) and np.array_equal(a.v, b.v)
    assert list(a.lens) == list(b.lens) == [6, 5]


def test_chunk_capacity_and_argument_errors_leave_state():
    cfg = I.small_config()
    L = O.Layer(cfg, I.layer_weights(cfg))
    cache = O.KVCache(L, 2, 6)
    O.prefill(L, I.hidden(4, cfg["d_model"], 1), np.array([0, 4], np.int32), cache=cache, slots=[1])
    before_k, before_len = cache.k.copy(), cache.lens.copy()
    with pytest.raises(OverflowError):
        O.prefill_chunk(L, I.hidden(4, cfg["d_model"], 2), np.array([0, 1, 4], np.int32), [0, 1], cache)
    with pytest.raises(ValueError):                          # repeated slot
        O.prefill_chunk(L, I.hidden(2, cfg["d_model"], 2), np.array([0, 1, 2], np.int32), [1, 1], cache)
    assert np.array_equal(before_k, cache.k) and np.array_equal(before_len, cache.lens)
    O.prefill_chunk(L, I.hidden(2, cfg["d_model"], 2), np.array([0, 2], np.int32), [1], cache)   # exactly full
    assert cache.lens[1] == 6


# ---- invariants -------------------------------------------------------------------------------------

def test_rmsnorm_unit_rms_and_gain():
    x = I.hidden(9, 64, 3) * 5
    y = O.rmsnorm(x, np.ones(64, np.float32), 1e-6)
    assert np.allclose(np.sqrt((y.astype(np.float64) ** 2).mean(1)), 1.0, atol=1e-6)
    g = np.linspace(0.5, 2, 64).astype(np.float32)
    assert np.allclose(O.rmsnorm(x, g, 1e-6), y * g, rtol=2e-7, atol=0)
    # eps sits inside the square root: a zero row stays zero and tiny rows scale by 1/sqrt(eps)
    z = np.full((1, 64), 1e-6, np.float32)
    assert np.allclose(O.rmsnorm(z, np.ones(64, np.float32), 1e-2), z / np.sqrt(1e-12 + 1e-2), rtol=1e-6)


def test_rope_properties():
    rng = np.random.default_rng(1)
    hd = 16
    q = rng.standard_normal((1, 1, hd)).astype(np.float32)
    k = rng.standard_normal((1, 1, hd)).astype(np.float32)
    assert np.array_equal(O.rope(q, [0]), q)                      # position 0 is the identity
    r = O.rope(q, [37])
    half = hd // 2
    n0 = q[0, 0, :half] ** 2 + q[0, 0, half:] ** 2
    n1 = r[0, 0, :half] ** 2 + r[0, 0, half:] ** 2
    assert np.allclose(n0, n1, rtol=1e-6)                         # each (i, i+hd/2) pair keeps its norm
    dots = [float((O.rope(q, [m]).astype(np.float64) * O.rope(k, [n]).astype(np.float64)).sum())
            for m, n in [(5, 2), (40, 37), (103, 100)]]
    assert np.allclose(dots, dots[0], atol=1e-5)                  # depends on m - n only
    # closed form for the first pair (theta_0 = 1) and the last pair (theta = base^(-(hd-2)/hd))
    p = 3
    th = 10000.0 ** (-(hd - 2) / hd)
    a, b = float(q[0, 0, 0]), float(q[0, 0, half])
    r3 = O.rope(q, [p])
    assert r3[0, 0, 0] == pytest.approx(a * np.cos(p) - b * np.sin(p), rel=1e-6)
    assert r3[0, 0, half] == pytest.approx(b * np.cos(p) + a * np.sin(p), rel=1e-6)
    a, b = float(q[0, 0, half - 1]), float(q[0, 0, hd - 1])
    assert r3[0, 0, half - 1] == pytest.approx(a * np.cos(p * th) - b * np.sin(p * th), rel=1e-6)


def test_attention_single_key_and_uniform():
    rng = np.random.default_rng(2)
    q = rng.standard_normal((3, 2, 8)).astype(np.float32)
    k = rng.standard_normal((3, 2, 8)).astype(np.float32)
    v = rng.standard_normal((3, 2, 8)).astype(np.float32)
    o = O.attention(q, k, v, np.array([0, 3], np.int32))
    assert np.allclose(o[0], v[0], atol=1e-7)                     # first token sees only itself
    o = O.attention(q * 0, k, v, np.array([0, 3], np.int32))       # zero query -> uniform average
    assert np.allclose(o[2], v.mean(0), atol=1e-6)


def test_causality_and_batch_independence():
    cfg = I.small_config()
    L = O.Layer(cfg, I.layer_weights(cfg, std=0.08))
    x = I.hidden(30, cfg["d_model"], 9)
    cu = np.array([0, 12, 30], np.int32)
    base = O.prefill(L, x, cu)
    x2 = x.copy()
    x2[8:12] += 1.0                                               # perturb the tail of sequence 0
    pert = O.prefill(L, x2, cu)
    assert np.array_equal(base[:8], pert[:8])                     # earlier rows bit-identical
    assert np.array_equal(base[12:], pert[12:])                   # other sequence untouched
    assert not np.array_equal(base[8:12], pert[8:12])
    alone = O.prefill(L, x[12:], np.array([0, 18], np.int32))
    assert np.array_equal(alone, base[12:])                       # packed == alone


def test_gqa_equals_mha_with_duplicated_kv_heads():
    cfg = I.small_config(n_q_heads=4, n_kv_heads=2)
    w = I.layer_weights(cfg, std=0.08)
    hd, d = cfg["head_dim"], cfg["d_model"]
    w2 = dict(w)
    w2["w_k"] = np.repeat(w["w_k"].reshape(2, hd, d), 2, axis=0).reshape(4 * hd, d)
    w2["w_v"] = np.repeat(w["w_v"].reshape(2, hd, d), 2, axis=0).reshape(4 * hd, d)
    cfg2 = dict(cfg, n_kv_heads=4)
    x = I.hidden(21, d, 4)
    cu = np.array([0, 21], np.int32)
    assert np.array_equal(O.prefill(O.Layer(cfg, w), x, cu), O.prefill(O.Layer(cfg2, w2), x, cu))


def test_moe_special_cases_reduce_to_dense():
    cfg = I.small_config(d_ff=64)
    w = I.layer_weights(cfg, std=0.08)
    x = I.hidden(10, cfg["d_model"], 12)
    cu = np.array([0, 10], np.int32)
    dense = O.prefill(O.Layer(cfg, w), x, cu)
    # identical experts: the renormalised weights sum to 1
    cfgm = dict(cfg, n_experts=4, top_k=2)
    wm = dict(w)
    for n in ("w_gate", "w_up", "w_down"):
        wm[n] = np.repeat(w[n][None], 4, axis=0)
    moe = O.prefill(O.Layer(cfgm, wm), x, cu, router_logits=I.router_logits(10, 4, 1))
    assert relmax(moe, dense) < 1e-6
    # one expert, top-1
    cfg1 = dict(cfg, n_experts=1, top_k=1)
    w1 = dict(w)
    for n in ("w_gate", "w_up", "w_down"):
        w1[n] = w[n][None]
    one = O.prefill(O.Layer(cfg1, w1), x, cu, router_logits=np.zeros((10, 1), np.float32))
    assert relmax(one, dense) < 1e-7


def test_router_top2_weights_and_tie_break():
    r = np.array([[0.0, 1.0, 3.0, 2.0], [1.0, 1.0, 1.0, 1.0], [2.0, 5.0, 5.0, 0.0]], np.float32)
    idx, wgt = O.route(r, 2)
    assert idx.tolist() == [[2, 3], [0, 1], [1, 2]]               # ties -> lower index first
    assert np.allclose(wgt.sum(1), 1.0)
    # renormalised softmax over all experts == softmax over the two chosen logits
    assert wgt[0, 0] == pytest.approx(np.exp(3) / (np.exp(3) + np.exp(2)), rel=1e-12)
    assert np.allclose(wgt[1], 0.5)


def test_ffn_zero_branches_and_silu_closed_form():
    # W_up = 0, W_down = 0 or W_gate = 0 (silu(0) = 0) each make the FFN add nothing: out == h.
    cfg = I.small_config(d_ff=32)
    w = I.layer_weights(cfg, std=0.08)
    h = I.hidden(5, cfg["d_model"], 2)
    for name in ("w_gate", "w_up", "w_down"):
        wz = dict(w)
        wz[name] = np.zeros_like(w[name])
        assert np.array_equal(O.ffn_block(O.Layer(cfg, wz), h), h)
    # silu closed form at one point: an FFN with F=1 and known scalars
    cfg1 = dict(cfg, d_model=2, n_q_heads=1, n_kv_heads=1, head_dim=2, d_ff=1)
    w1 = {"g_attn": np.ones(2, np.float32), "g_ffn": np.ones(2, np.float32),
          "w_q": np.zeros((2, 2), np.float32), "w_k": np.zeros((2, 2), np.float32),
          "w_v": np.zeros((2, 2), np.float32), "w_o": np.zeros((2, 2), np.float32),
          "w_gate": np.array([[1.0, 0.0]], np.float32), "w_up": np.array([[0.0, 1.0]], np.float32),
          "w_down": np.array([[1.0], [0.0]], np.float32)}
    hh = np.array([[3.0, 4.0]], np.float32)                        # rms = sqrt(12.5)
    y = hh.astype(np.float64) / np.sqrt(12.5 + 1e-6)
    z = y[0, 0]
    expect0 = 3.0 + (z / (1 + np.exp(-z))) * y[0, 1]
    out = O.ffn_block(O.Layer(cfg1, w1), hh)
    assert out[0, 0] == pytest.approx(expect0, rel=1e-6) and out[0, 1] == 4.0


def test_row_sampled_prefill_equals_full_rows():
    cfg = I.small_config()
    L = O.Layer(cfg, I.layer_weights(cfg, std=0.08))
    cu = np.array([0, 14, 33], np.int32)
    x = I.hidden(33, cfg["d_model"], 14)
    full = O.prefill(L, x, cu)
    rows = [32, 0, 13, 20]
    assert np.array_equal(O.prefill(L, x, cu, rows=rows), full[rows])


def test_linear_is_x_times_w_transposed():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((3, 7)).astype(np.float32)
    W = rng.standard_normal((5, 7)).astype(np.float32)
    assert np.allclose(O.linear(x, W), x.astype(np.float64) @ W.astype(np.float64).T, rtol=1e-6, atol=1e-6)


def test_input_module_bf16_rounding_is_rne():
    a = np.array([1.0, 1.00390625, 1.01171875, -3.1415927, 65504.0, 1e-8], np.float32)
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(I.round_to_bf16(a), ref)
    assert np.array_equal(I.bf16_bits_to_f32(I.f32_to_bf16_bits(a)), ref)


# ---- 8-bit E4M3 cache storage ---------------------------------------------------------------------

def test_fp8_e4m3_codec_against_the_format_and_a_library_conversion():
    codes = np.arange(256, dtype=np.uint8)
    vals = O.fp8_e4m3_decode(codes)
    # the format's landmarks: 1.0, largest finite, smallest normal, smallest subnormal, NaN codes
    assert vals[0x38] == 1.0 and vals[0x7E] == 448.0 and vals[0x08] == 2.0 ** -6 and vals[0x01] == 2.0 ** -9
    assert np.isnan(vals[0x7F]) and np.isnan(vals[0xFF]) and vals[0xFE] == -448.0
    finite = ~np.isnan(vals)
    assert np.array_equal(O.fp8_e4m3_encode(vals[finite]), codes[finite])          # round trip of every code
    pos = vals[:0x7F]
    assert np.all(np.diff(pos) > 0)                                                # strictly increasing
    # an independent conversion: PyTorch's CPU float8_e4m3fn cast (in range; it does not saturate)
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * rng.choice([1e-3, 0.05, 1.0, 30.0], 20000),
                        (pos[:-1] + pos[1:]) / 2, -(pos[:-1] + pos[1:]) / 2,     # exact ties
                        pos, -pos]).astype(np.float32)
    x = x[np.abs(x) <= 448.0]
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    mine = O.fp8_e4m3_encode(x)
    both_zero = (O.fp8_e4m3_decode(mine) == 0) & (O.fp8_e4m3_decode(lib) == 0)     # +0 / -0 of tiny inputs
    assert np.array_equal(mine[~both_zero], lib[~both_zero])
    # saturation and NaN
    assert list(O.fp8_e4m3_encode([1e9, -500.0, 448.0, 463.9, float("nan")])) == [0x7E, 0xFE, 0x7E, 0x7E, 0x7F]


def test_fp8_cache_stores_quantised_values_and_prefill_itself_is_unchanged():
    cfg = I.small_config()
    w = I.layer_weights(cfg, std=0.08)
    L = O.Layer(cfg, w)
    x = I.hidden(30, cfg["d_model"], seed=90)
    cu = np.array([0, 11, 30], np.int32)
    exact, q8 = O.KVCache(L, 2, 40), O.KVCache(L, 2, 40, fp8_scales=(0.5, 2.0))
    out_e = O.prefill(L, x, cu, cache=exact, slots=[0, 1])
    out_q = O.prefill(L, x, cu, cache=q8, slots=[0, 1])
    assert np.array_equal(out_e, out_q)                 # prefill attends over the fresh keys and values
    for cache_t, ref_t, s in ((q8.k, exact.k, 0.5), (q8.v, exact.v, 2.0)):
        lib = torch.from_numpy(ref_t / s).to(torch.float8_e4m3fn).float().numpy() * s
        assert np.array_equal(cache_t, lib.astype(np.float32))
    # decode and a chunk over the quantised cache: close to the exact run, not equal to it
    xn = I.hidden(2, cfg["d_model"], seed=91)
    d_e, d_q = O.decode_step(L, xn, [0, 1], exact), O.decode_step(L, xn, [0, 1], q8)
    assert 0 < relmax(d_q, d_e) < 0.05
    xc = I.hidden(7, cfg["d_model"], seed=92)
    c_e = O.prefill_chunk(L, xc, np.array([0, 3, 7], np.int32), [0, 1], exact)
    c_q = O.prefill_chunk(L, xc, np.array([0, 3, 7], np.int32), [0, 1], q8)
    assert 0 < relmax(c_q, c_e) < 0.05
    # the appended positions are quantised too: every stored element is a representable value
    for cache_t, s in ((q8.k, 0.5), (q8.v, 2.0)):
        held = cache_t[0, :, :int(q8.lens[0])] / s
        assert np.array_equal(O.fp8_e4m3_decode(O.fp8_e4m3_encode(held)).astype(np.float32), held)
    # set(): the benchmark fill goes through the same quantiser
    k, v = I.kv_fill(cfg["n_kv_heads"], 5, cfg["head_dim"], seed=3)
    q8.set(1, k, v)
    assert np.array_equal(q8.k[1, :, :5], torch.from_numpy(k / 0.5).to(torch.float8_e4m3fn).float().numpy() * 0.5)


# ---- stack ends: embedding and LM head -------------------------------------------------------------

def test_lm_head_against_library_composition_and_closed_forms():
    d, V, T = 96, 333, 7
    hw = I.head_weights(d, V, seed=3, std=0.1)
    x = I.hidden(T, d, seed=4)
    got = O.lm_head(x, hw["g_final"], hw["w_lm"], eps=1e-6)
    xt = torch.from_numpy(x).double()
    ref = torch.nn.functional.rms_norm(xt, (d,), torch.from_numpy(hw["g_final"]).double(), 1e-6) @ \
        torch.from_numpy(hw["w_lm"]).double().T
    assert np.max(np.abs(got - ref.numpy())) <= 2e-6 * float(ref.abs().max())
    # identity projection and unit gain: the logits are the unit-RMS rows themselves
    eye = np.eye(d, dtype=np.float32)
    y = O.lm_head(x, np.ones(d, np.float32), eye, eps=0.0)
    assert np.allclose(np.sqrt(np.mean(y.astype(np.float64) ** 2, axis=1)), 1.0, atol=1e-6)
    assert np.allclose(y * np.sqrt(np.mean(x.astype(np.float64) ** 2, axis=1))[:, None], x, atol=1e-5)
    # the norm removes the scale of the input (eps = 0); the gain scales one input channel
    assert np.allclose(O.lm_head(8.0 * x, hw["g_final"], hw["w_lm"], eps=0.0),
                       O.lm_head(x, hw["g_final"], hw["w_lm"], eps=0.0), rtol=1e-5, atol=1e-6)
    g2 = hw["g_final"].copy()
    g2[5] = 0.0
    w5 = hw["w_lm"].copy()
    w5[:, 5] = 0.0
    assert np.allclose(O.lm_head(x, g2, hw["w_lm"]), O.lm_head(x, hw["g_final"], w5), atol=1e-6)
    # a constant row c: every normalised element is c / sqrt(c^2 + eps); one-hot W row picks g_j times it
    c, eps = 0.5, 0.25
    row = np.full((1, d), c, np.float32)
    pick = np.zeros((1, d), np.float32)
    pick[0, 11] = 1.0
    assert O.lm_head(row, hw["g_final"], pick, eps=eps)[0, 0] == pytest.approx(
        c / np.sqrt(c * c + eps) * float(hw["g_final"][11]), rel=1e-6)


def test_embedding_is_a_row_lookup():
    d, V = 24, 50
    hw = I.head_weights(d, V, seed=5)
    ids = np.array([0, 49, 7, 7, 13], np.int32)
    assert np.array_equal(O.embed(hw["w_embed"], ids), hw["w_embed"][ids])
    for bad in ([3, 50], [-1, 2]):
        with pytest.raises(ValueError):
            O.embed(hw["w_embed"], np.array(bad, np.int32))


# ---- 8-bit weights ---------------------------------------------------------------------------------

def test_row_quantisation_scales_and_values():
    """Per-row power-of-two scales and E4M3 values of quantise_rows, against the format's own facts
    and a library conversion."""
    rng = np.random.default_rng(21)
    W = (rng.standard_normal((37, 200)) * np.exp(rng.uniform(-8, 3, (37, 1)))).astype(np.float32)
    W[5] = 0.0                                   # a row of zeros keeps scale 1
    W[6, :] = 0.0
    W[6, 17] = 448.0 * 2.0 ** -3                 # maximum exactly on a power-of-two boundary
    W[7, 3] = 448.0 * 2.0 ** -3 * (1 + 2.0 ** -20)    # and just above it
    Wq, s = O.quantise_rows(W)
    assert s[5] == 1.0 and np.all(Wq[5] == 0.0)
    assert s[6] == 2.0 ** -3 and Wq[6, 17] == W[6, 17]
    m = np.max(np.abs(W), axis=1)
    live = m > 0
    # powers of two, the smallest that keep the row inside +-448
    assert np.all(np.log2(s[live]) == np.round(np.log2(s[live])))
    assert np.all(m[live] / s[live] <= 448.0) and np.all(m[live] / (s[live] / 2) > 448.0)
    # every value is a representable E4M3 number times the scale: the library's conversion agrees
    t = torch.from_numpy(W / s[:, None]).to(torch.float8_e4m3fn).float().numpy() * s[:, None]
    assert np.array_equal(Wq, t.astype(np.float32))
    # nearest representable value: error at most half the local spacing (2^-3 relative at most), and
    # quantising twice changes nothing
    a = np.abs(W[live] / s[live, None])
    spacing = 2.0 ** (np.floor(np.log2(np.maximum(a, 2.0 ** -6))) - 3)
    assert np.all(np.abs(Wq[live] - W[live]) / s[live, None] <= spacing / 2 + 1e-12)
    Wq2, s2 = O.quantise_rows(Wq)
    assert np.array_equal(Wq2, Wq)
    # leading axes are rows too (mixture-of-experts weights [E, F, d])
    W3 = W[:36].reshape(3, 12, 200)
    assert np.array_equal(O.quantise_rows(W3)[0].reshape(36, 200), Wq[:36])


def test_layer_with_quantised_weights_is_the_layer_on_the_replaced_weights():
    cfg = I.small_config()
    w = I.layer_weights(cfg, std=0.1)
    wq = O.quantise_layer_weights(w)
    assert np.array_equal(wq["g_attn"], w["g_attn"]) and not np.array_equal(wq["w_q"], w["w_q"])
    x = I.hidden(9, cfg["d_model"], seed=2)
    cu = np.array([0, 4, 9], np.int32)
    a = O.prefill(O.Layer(cfg, wq), x, cu)
    b = O.prefill(O.Layer(cfg, w), x, cu)
    # the quantised layer is close to, and different from, the exact one (3 mantissa bits per weight)
    err = np.max(np.abs(a - b)) / np.max(np.abs(b))
    assert 1e-4 < err < 0.1


def test_activation_row_quantisation_against_library_conversions():
    """act_quantise_rows = round to bf16, then the weight-row rule: against torch's bfloat16 and
    float8_e4m3fn conversions (values, scales and code bytes), with planted boundary cases."""
    rng = np.random.default_rng(31)
    x = (rng.standard_normal((23, 136)) * np.exp(rng.uniform(-6, 4, (23, 1)))).astype(np.float32)
    x[3] = 0.0                                     # zero row: scale 1
    x[4, :] = 0.0
    x[4, 9] = 448.0 * 4.0                          # maximum exactly 448 * 2^2
    x[5, 2] = np.float32(448.0 * 4.0) * np.float32(1 + 2.0 ** -7)   # one bf16 step above: next scale
    x[6, 5] = 1.0 + 2.0 ** -9                      # rounds to 1.0 in bf16 before anything else
    xq, s, codes = O.act_quantise_rows(x)
    xb = torch.from_numpy(x).to(torch.bfloat16).float().numpy()
    assert s[3] == 1.0 and s[4] == 4.0 and s[5] == 8.0
    m = np.max(np.abs(xb), axis=1)
    live = m > 0
    assert np.all(np.log2(s[live]) == np.round(np.log2(s[live])))
    assert np.all(m[live] / s[live] <= 448.0) and np.all(m[live] / (s[live] / 2) > 448.0)
    t8 = torch.from_numpy(xb / s[:, None]).to(torch.float8_e4m3fn)
    assert np.array_equal(xq, t8.float().numpy() * s[:, None])
    assert np.array_equal(codes, t8.view(torch.uint8).numpy())
    # the bf16 rounding comes first: quantising the rounded rows as weights gives the same thing
    assert np.array_equal(xq, O.quantise_rows(xb)[0])
    assert xq[6, 5] == O.quantise_rows(np.where(np.arange(136) == 5, 1.0, xb[6]).astype(np.float32)[None])[0][0, 5]


def test_act8_call_matches_library_composition():
    """8-bit activations: in a call that says so the four projections see quantised input rows;
    against the float64 library composition with the library's conversions in the same four places."""
    cfg = I.small_config(d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ff=96)
    w = O.quantise_layer_weights(I.layer_weights(cfg, std=0.08))
    T = 70
    cu = np.array([0, 30, 31, T], np.int32)
    x = I.hidden(T, cfg["d_model"], seed=6)
    ol = O.Layer(cfg, w)
    got = O.prefill(ol, x, cu, act8=True)
    ref = torch_layer(cfg, w, x, cu, act_q=torch_act_q)
    assert relmax(got, ref) < 2e-6
    plain = O.prefill(ol, x, cu)
    assert 1e-4 < relmax(got, plain) < 0.2       # and it is not the layer without them
    assert np.array_equal(plain, O.prefill(ol, x, cu, act8=False))


def test_act8_moe_call_matches_library_composition():
    """Mixture of experts: the normalised row is quantised once per token after routing (the router
    reads it unquantised), the SwiGLU row once per (token, expert) pair."""
    cfg = I.small_config(d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ff=48, n_experts=4, top_k=2)
    w = O.quantise_layer_weights(I.layer_weights(cfg, std=0.08, with_router=True))
    T = 45
    cu = np.array([0, 20, T], np.int32)
    x = I.hidden(T, cfg["d_model"], seed=16)
    ol = O.Layer(cfg, w)
    for rl in (None, I.router_logits(T, 4, seed=17)):
        got = O.prefill(ol, x, cu, router_logits=rl, act8=True)
        ref = torch_layer(cfg, w, x, cu, router_logits=rl, act_q=torch_act_q)
        assert relmax(got, ref) < 2e-6
        assert relmax(got, O.prefill(ol, x, cu, router_logits=rl)) > 1e-4


def test_act8_is_a_statement_of_the_call_at_any_row_count():
    """Nothing inside the oracle decides which calls quantise: one row or many, prefill, decode and
    chunked prefill all follow the flag of the call; the flag changes nothing else (cache contents of
    a call without it stay exact)."""
    cfg = I.small_config()
    w = I.layer_weights(cfg, std=0.08)
    ol = O.Layer(cfg, w)
    for T in (1, 2, 40):
        cu = np.array([0, T], np.int32)
        x = I.hidden(T, cfg["d_model"], seed=7)
        assert not np.array_equal(O.prefill(ol, x, cu, act8=True), O.prefill(ol, x, cu))
    for B in (1, 3):
        ca, cp = O.KVCache(ol, B, 16), O.KVCache(ol, B, 16)
        xs = I.hidden(B, cfg["d_model"], seed=8)
        a = O.decode_step(ol, xs, list(range(B)), ca, act8=True)
        p = O.decode_step(ol, xs, list(range(B)), cp)
        assert not np.array_equal(a, p)
        # decode with the flag == prefill with the flag of the same one-token sequences
        cu = np.arange(B + 1, dtype=np.int32)
        assert relmax(a, O.prefill(ol, xs, cu, act8=True)) < 1e-6
    ca, cp = O.KVCache(ol, 1, 48), O.KVCache(ol, 1, 48)
    x = I.hidden(40, cfg["d_model"], seed=9)
    cuc = np.array([0, 40], np.int32)
    a = O.prefill_chunk(ol, x, cuc, [0], ca, act8=True)
    assert not np.array_equal(a, O.prefill_chunk(ol, x, cuc, [0], cp))
    assert relmax(a, O.prefill(ol, x, cuc, act8=True)) < 1e-6
    h = I.hidden(5, cfg["d_model"], seed=10)
    assert not np.array_equal(O.ffn_block(ol, h, act8=True), O.ffn_block(ol, h))


def test_gemm_e4m3_is_the_product_of_the_decoded_matrices():
    """Against the library's own reading of the bytes (float8_e4m3fn view) and a float64 matmul."""
    rng = np.random.default_rng(41)
    a = rng.integers(0, 256, (9, 64), dtype=np.uint8)
    b = rng.integers(0, 256, (5, 64), dtype=np.uint8)
    a[(a & 0x7f) == 0x7f] = 0x30                      # no NaN codes
    b[(b & 0x7f) == 0x7f] = 0xB1
    sa = 2.0 ** rng.integers(-6, 6, 9).astype(np.float32)
    sb = 2.0 ** rng.integers(-6, 6, 5).astype(np.float32)
    A = torch.from_numpy(a).view(torch.float8_e4m3fn).to(torch.float64) * torch.from_numpy(sa).to(torch.float64)[:, None]
    B = torch.from_numpy(b).view(torch.float8_e4m3fn).to(torch.float64) * torch.from_numpy(sb).to(torch.float64)[:, None]
    ref = (A @ B.T).numpy()
    got = O.gemm_e4m3(a, sa, b, sb)
    assert np.allclose(got, ref, rtol=1e-13, atol=0)
    # one-hot rows pick single products
    a1 = np.zeros((1, 64), np.uint8)
    a1[0, 7] = 0x38                                  # 1.0
    assert np.array_equal(O.gemm_e4m3(a1, np.ones(1), b, np.ones(5))[0], O.fp8_e4m3_decode(b[:, 7]))
