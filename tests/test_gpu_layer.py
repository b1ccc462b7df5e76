"""GPU parity: the HIP layer forward (through the C ABI) against the CPU oracle, element by
element, on the same seeded inputs.  Bound: max |gpu - ref| / max |ref| <= 1e-5 (fp32 layers),
<= 2e-2 (bf16 layers)."""
import numpy as np
import pytest
import torch

import paper_2603_04716_amd as pd
import pd_inputs as I
from oracle import layer as O
from gpu_util import GpuLayer, TOL, relmax, to_dev, to_np

pytestmark = pytest.mark.gpu


def both(cfg, std=0.02, with_router=False, seed=None):
    w = I.layer_weights(cfg, seed=seed, std=std, with_router=with_router)
    return O.Layer(cfg, w), GpuLayer(cfg, w)


def test_tiny_config_two_layers_prefill_and_decode():
    cfg = I.CONFIGS["tiny"]
    layers = [both(cfg, seed=cfg["seed"] + i) for i in range(2)]
    tol = TOL["f32"]
    # prefill: 4 sequences of 128 rows through both layers
    x = I.hidden(512, cfg["d_model"], seed=100)
    cu = I.uniform_cu_seqlens(4, 128)
    ref, got = x, x
    for ol, gl in layers:
        ref = O.prefill(ol, ref, cu)
        got = gl.prefill(got, cu)
        assert relmax(got, ref) <= tol
    # decode: batch 8, each sequence over a 128-token cache produced by its own prefill
    xp = I.hidden(8 * 128, cfg["d_model"], seed=101)
    cu8 = I.uniform_cu_seqlens(8, 128)
    slots = list(range(8))
    ocaches = [O.KVCache(ol, 8, 130) for ol, _ in layers]
    gcaches = [gl.cache(8, 130) for _, gl in layers]
    ref, got = xp, xp
    for (ol, gl), oc, gc in zip(layers, ocaches, gcaches):
        ref = O.prefill(ol, ref, cu8, cache=oc, slots=slots)
        got = gl.prefill(got, cu8, cache=gc, slots=slots)
        assert relmax(got, ref) <= tol
    for step in range(2):
        xn = I.hidden(8, cfg["d_model"], seed=102 + step)
        ref, got = xn, xn
        for (ol, gl), oc, gc in zip(layers, ocaches, gcaches):
            ref = O.decode_step(ol, ref, slots, oc)
            got = gl.decode(got, slots, gc)
            assert relmax(got, ref) <= tol
            assert pd.pd_kv_cache_len(gc, 3) == 129 + step
    for _, gl in layers:
        gl.close()


SMALL = [
    dict(),
    dict(n_q_heads=4, n_kv_heads=4),
    dict(n_q_heads=8, n_kv_heads=1, head_dim=16),
    dict(d_model=96, n_q_heads=6, n_kv_heads=3, head_dim=8, d_ff=80),
    dict(d_model=200, n_q_heads=2, n_kv_heads=1, head_dim=130, d_ff=72),
    dict(d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=128, d_ff=512),     # MFMA-eligible in bf16
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("over", SMALL)
def test_small_ragged_prefill_then_decode(over, dtype):
    cfg = I.small_config(dtype=dtype, **over)
    ol, gl = both(cfg, std=0.08)
    tol = TOL[dtype]
    cu = np.array([0, 70, 70, 199, 200, 333], np.int32)     # ragged, one empty, one single-token
    x = I.hidden(int(cu[-1]), cfg["d_model"], seed=5, dtype=dtype)
    slots = [4, 0, 2, 5, 1]
    oc, gc = O.KVCache(ol, 6, 140), gl.cache(6, 140)
    ref = O.prefill(ol, x, cu, cache=oc, slots=slots)
    got = gl.prefill(x, cu, cache=gc, slots=slots)
    assert relmax(got, ref) <= tol
    assert [pd.pd_kv_cache_len(gc, s) for s in slots] == [70, 0, 129, 1, 133]
    # without a cache the output is the same
    assert np.array_equal(gl.prefill(x, cu), got)
    for step in range(3):
        xn = I.hidden(5, cfg["d_model"], seed=50 + step, dtype=dtype)
        ref = O.decode_step(ol, xn, slots, oc)
        got = gl.decode(xn, slots, gc)
        assert relmax(got, ref) <= tol
    # cache contents: rotated keys and values of slot 2
    Hkv, hd = cfg["n_kv_heads"], cfg["head_dim"]
    n = 129 + 3
    k = torch.empty((Hkv, n, hd), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")
    v = torch.empty_like(k)
    pd.pd_kv_cache_get(gc, 2, k, v)
    torch.cuda.synchronize()
    assert relmax(to_np(k), oc.k[2, :, :n]) <= tol
    assert relmax(to_np(v), oc.v[2, :, :n]) <= tol
    gl.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_moe_small(dtype):
    cfg = I.small_config(dtype=dtype, n_experts=8, top_k=2, d_ff=96)
    ol, gl = both(cfg, std=0.08, with_router=True)
    tol = TOL[dtype]
    cu = np.array([0, 37, 150], np.int32)
    x = I.hidden(150, cfg["d_model"], seed=6, dtype=dtype)
    r = I.router_logits(150, 8, seed=9)
    r[3] = 0.25                                  # all-equal logits: ties resolve to experts 0, 1
    r[4, 5] = r[4, 2] = 3.0                      # two-way tie at the top
    r[5] = -5.0                                  # different logits whose probabilities round to the same double:
    r[5, 3], r[5, 1], r[5, 6] = 1.0, 1e-30, 2e-30        # a tie for the second place, the lower index wins
    ref, eref = O.prefill(ol, x, cu, router_logits=r, return_experts=True)
    assert list(eref[5]) == [3, 1]
    got = gl.prefill(x, cu, router_logits=r)
    assert np.array_equal(gl.experts(150), eref)            # integer decisions: bit-exact
    assert relmax(got, ref) <= tol
    if dtype == "f32":
        # router computed on the device from w_router (fp32 logits decide the experts; a bf16
        # layer could legitimately flip a near-tie, so only the fp32 layer is compared here)
        ref, eref = O.prefill(ol, x, cu, return_experts=True)
        got = gl.prefill(x, cu)
        assert np.array_equal(gl.experts(150), eref)
        assert relmax(got, ref) <= tol
    oc, gc = O.KVCache(ol, 2, 160), gl.cache(2, 160)
    O.prefill(ol, x, cu, router_logits=r, cache=oc, slots=[0, 1])
    gl.prefill(x, cu, cache=gc, slots=[0, 1], router_logits=r)
    xn = I.hidden(2, cfg["d_model"], seed=77, dtype=dtype)
    rn = I.router_logits(2, 8, seed=78)
    ref, eref = O.decode_step(ol, xn, [0, 1], oc, router_logits=rn, return_experts=True)
    got = gl.decode(xn, [0, 1], gc, router_logits=rn)
    assert np.array_equal(gl.experts(2), eref)
    assert relmax(got, ref) <= tol
    gl.close()


@pytest.mark.parametrize("hq,hkv", [(4, 1), (2, 2)])
def test_bf16_matrix_core_path_long_ragged(hq, hkv):
    """head_dim 128 in bf16 runs the MFMA GEMM and MFMA attention kernels: several query blocks and
    key tiles per sequence, ragged tails, a one-token and an empty sequence."""
    cfg = I.small_config(dtype="bf16", d_model=256, n_q_heads=hq, n_kv_heads=hkv, head_dim=128, d_ff=512)
    ol, gl = both(cfg, std=0.05)
    cu = np.array([0, 600, 601, 601, 858, 1243, 1307], np.int32)
    x = I.hidden(int(cu[-1]), cfg["d_model"], seed=21, dtype="bf16")
    slots = [0, 1, 2, 3, 4, 5]
    oc, gc = O.KVCache(ol, 6, 640), gl.cache(6, 640)
    ref = O.prefill(ol, x, cu, cache=oc, slots=slots)
    got = gl.prefill(x, cu, cache=gc, slots=slots)
    assert relmax(got, ref) <= TOL["bf16"]
    # per-sequence check as well, so that a short sequence cannot hide behind a large global max
    for s in range(6):
        a, b = cu[s], cu[s + 1]
        if b > a:
            assert relmax(got[a:b], ref[a:b]) <= TOL["bf16"]
    # 36 decode steps: appended tokens cross the 16-, 32- and 64-position block boundaries of the cache
    for step in range(36):
        xn = I.hidden(6, cfg["d_model"], seed=220 + step, dtype="bf16")
        ref = O.decode_step(ol, xn, slots, oc)
        got = gl.decode(xn, slots, gc)
        assert relmax(got, ref) <= TOL["bf16"], step
        for i in range(6):
            assert relmax(got[i], ref[i]) <= 2 * TOL["bf16"], (step, i)
    gl.close()


@pytest.mark.parametrize("B", [1, 3, 16, 17, 64, 65, 130, 256])
def test_bf16_decode_batch_sizes_ragged_cache(B):
    """Every decode GEMM variant (<=16 rows, <=64, <=128, <=256 with split-K) and the chunked decode
    attention, over caches of ragged length filled through pd_kv_cache_set."""
    cfg = I.small_config(dtype="bf16", d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=128, d_ff=512)
    ol, gl = both(cfg, std=0.05)
    rng = np.random.default_rng(B)
    lens = rng.integers(0, 300, B)
    lens[0] = 299
    cap = 320
    oc, gc = O.KVCache(ol, B, cap), gl.cache(B, cap)
    for i, n in enumerate(lens):
        k, v = I.kv_fill(2, int(n), 128, seed=1000 + i, dtype="bf16")
        oc.set(i, k, v)
        if n > 0:
            pd.pd_kv_cache_set(gc, i, to_dev(k, "bf16"), to_dev(v, "bf16"))
    slots = list(range(B))
    for step in range(2):
        xn = I.hidden(B, cfg["d_model"], seed=31 + step, dtype="bf16")
        ref = O.decode_step(ol, xn, slots, oc)
        got = gl.decode(xn, slots, gc)
        assert relmax(got, ref) <= TOL["bf16"]
        worst = max(relmax(got[i], ref[i]) for i in range(B))
        assert worst <= 2 * TOL["bf16"]
    gl.close()


@pytest.mark.parametrize("B", [17, 32, 33, 48, 64, 65, 100, 128])
@pytest.mark.parametrize("hq,hkv,d,F", [(4, 2, 512, 1024), (6, 2, 1024, 1536)])
def test_bf16_decode_mid_batches_wider_layers(B, hq, hkv, d, F):
    """Decode batches of 17 .. 128 rows on layers with inner dimensions of 512 .. 1536 (the wide
    register-operand kernel needs K in multiples of 512, the split-K tile kernels take the rest),
    groups of 2 and 3 query heads per kv head, ragged cache lengths including an empty and a
    block-aligned one; two steps, so the second attends over what the fused rotary embedding and
    append of the first wrote."""
    cfg = I.small_config(dtype="bf16", d_model=d, n_q_heads=hq, n_kv_heads=hkv, head_dim=128, d_ff=F)
    ol, gl = both(cfg, std=0.04)
    rng = np.random.default_rng(B + d)
    lens = rng.integers(0, 130, B)
    lens[0], lens[1] = 129, 63
    cap = 136
    oc, gc = O.KVCache(ol, B, cap), gl.cache(B, cap)
    k, v = I.kv_fill(hkv, 129, 128, seed=77, dtype="bf16")
    kd, vd = to_dev(k, "bf16"), to_dev(v, "bf16")
    for i, n in enumerate(lens):
        n = int(n)
        oc.set(i, k[:, :n], v[:, :n])
        if n > 0:
            pd.pd_kv_cache_set(gc, i, kd[:, :n].contiguous(), vd[:, :n].contiguous())
    slots = [int(s_) for s_ in rng.permutation(B)]
    for step in range(2):
        xn = I.hidden(B, d, seed=41 + step, dtype="bf16")
        ref = O.decode_step(ol, xn, slots, oc)
        got = gl.decode(xn, slots, gc)
        assert relmax(got, ref) <= TOL["bf16"]
        assert max(relmax(got[i], ref[i]) for i in range(B)) <= 2 * TOL["bf16"]
    gl.close()


def test_fp32_decode_beyond_rotary_table():
    """Positions past the precomputed rotary table (32768) take the on-the-fly double-precision
    path; fp32 bound 1e-5 must still hold there."""
    cfg = I.small_config(d_model=32, n_q_heads=2, n_kv_heads=1, head_dim=8, d_ff=32)
    ol, gl = both(cfg, std=0.1)
    n = 32767
    cap = n + 4
    k, v = I.kv_fill(1, n, 8, seed=9, dtype="f32")
    oc, gc = O.KVCache(ol, 1, cap), gl.cache(1, cap)
    oc.set(0, k, v)
    pd.pd_kv_cache_set(gc, 0, to_dev(k, "f32"), to_dev(v, "f32"))
    for step in range(3):                       # positions 32767 (table), 32768, 32769 (computed)
        xn = I.hidden(1, cfg["d_model"], seed=60 + step)
        assert relmax(gl.decode(xn, [0], gc), O.decode_step(ol, xn, [0], oc)) <= TOL["f32"]
    kk = torch.empty((1, n + 3, 8), dtype=torch.float32, device="cuda")
    vv = torch.empty_like(kk)
    pd.pd_kv_cache_get(gc, 0, kk, vv)
    torch.cuda.synchronize()
    assert relmax(to_np(kk)[:, n:], oc.k[0, :, n:n + 3]) <= TOL["f32"]
    gl.close()


@pytest.mark.parametrize("fp8", [False, True])
def test_bf16_decode_beyond_rotary_table(fp8):
    """The decode step of a bf16 layer on the matrix-core attention path rotates q and the new key inside
    the attention kernel and appends the key in a later launch: both read the rotary table up to
    position 32767 and compute the angle in double precision beyond it.  Three steps across that
    boundary, two sequences (one short, inside the table), outputs and appended keys against the oracle."""
    cfg = I.small_config(dtype="bf16", d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=128, d_ff=512)
    ol, gl = both(cfg, std=0.05)
    n = 32767
    cap = n + 4
    k, v = I.kv_fill(2, n, 128, seed=9, dtype="bf16")
    oc = O.KVCache(ol, 2, cap, fp8_scales=(0.5, 0.125) if fp8 else None)
    gc = gl.cache(2, cap, fp8_scales=(0.5, 0.125) if fp8 else None)
    oc.set(0, k, v)
    oc.set(1, k[:, :100], v[:, :100])
    pd.pd_kv_cache_set(gc, 0, to_dev(k, "bf16"), to_dev(v, "bf16"))
    pd.pd_kv_cache_set(gc, 1, to_dev(k[:, :100].copy(), "bf16"), to_dev(v[:, :100].copy(), "bf16"))
    for step in range(3):                       # slot 0: positions 32767 (table), 32768, 32769 (computed)
        xn = I.hidden(2, cfg["d_model"], seed=60 + step, dtype="bf16")
        ref = O.decode_step(ol, xn, [0, 1], oc)
        got = gl.decode(xn, [0, 1], gc)
        assert relmax(got, ref) <= TOL["bf16"]
        assert max(relmax(got[i], ref[i]) for i in range(2)) <= 2 * TOL["bf16"]
    kk = torch.empty((2, n + 3, 128), dtype=torch.bfloat16, device="cuda")
    vv = torch.empty_like(kk)
    pd.pd_kv_cache_get(gc, 0, kk, vv)
    torch.cuda.synchronize()
    # appended keys and values: within the bf16 bound of the oracle's, plus, in the 8-bit cache, the one
    # spacing of the representable values that rounding to a code can add
    for got, ref, scale in ((to_np(kk)[:, n:], oc.k[0, :, n:n + 3], oc.k_scale), (to_np(vv)[:, n:], oc.v[0, :, n:n + 3], oc.v_scale)):
        slack = TOL["bf16"] * np.max(np.abs(ref))
        if fp8:
            mag = np.maximum(np.maximum(np.abs(ref), np.abs(got)) / scale, 2.0 ** -6)
            slack = slack + scale * 2.0 ** (np.floor(np.log2(mag)) - 3)
        assert np.all(np.abs(got - ref) <= slack)
    gl.close()


def test_kv_cache_set_get_and_errors():
    cfg = I.small_config()
    ol, gl = both(cfg)
    gc = gl.cache(3, 16)
    k, v = I.kv_fill(cfg["n_kv_heads"], 10, cfg["head_dim"], seed=3, dtype="f32")
    kd, vd = to_dev(k, "f32"), to_dev(v, "f32")
    pd.pd_kv_cache_set(gc, 1, kd, vd)
    assert pd.pd_kv_cache_len(gc, 1) == 10
    k2, v2 = torch.empty_like(kd), torch.empty_like(vd)
    pd.pd_kv_cache_get(gc, 1, k2, v2)
    torch.cuda.synchronize()
    assert torch.equal(k2, kd) and torch.equal(v2, vd)
    # decode over a filled cache equals the oracle over the same contents
    oc = O.KVCache(ol, 3, 16)
    oc.set(1, k, v)
    xn = I.hidden(1, cfg["d_model"], seed=4)
    assert relmax(gl.decode(xn, [1], gc), O.decode_step(ol, xn, [1], oc)) <= TOL["f32"]
    # errors: full slot, repeated slot, slot out of range, too-long sequence; state unchanged
    pd.pd_kv_cache_set_len(gc, 2, 16)
    x2 = to_dev(I.hidden(2, cfg["d_model"], seed=5), "f32")
    out = torch.zeros_like(x2)
    for slots, status in [([1, 2], pd.PD_ERR_KV_CAPACITY), ([1, 1], pd.PD_ERR_INVALID_ARG), ([1, 3], pd.PD_ERR_INVALID_ARG)]:
        with pytest.raises(pd.PdError) as e:
            pd.pd_decode_step(gl.h, x2, slots, gc, out)
        assert e.value.status == status
    torch.cuda.synchronize()
    assert pd.pd_kv_cache_len(gc, 1) == 11 and float(out.abs().sum()) == 0.0
    xl = to_dev(I.hidden(17, cfg["d_model"], seed=6), "f32")
    with pytest.raises(pd.PdError) as e:
        pd.pd_prefill(gl.h, xl, [0, 17], torch.empty_like(xl), gc, [0])
    assert e.value.status == pd.PD_ERR_KV_CAPACITY
    with pytest.raises(pd.PdError) as e:
        pd.pd_prefill(gl.h, xl, [0, 9, 8, 17], torch.empty_like(xl))
    assert e.value.status == pd.PD_ERR_SHAPE
    # empty batch is a no-op
    pd.pd_prefill(gl.h, None, [0, 0], None)
    gl.close()


def test_layer_create_rejects_bad_shapes():
    cfg = I.small_config()
    w = {k: to_dev(v, "f32") for k, v in I.layer_weights(cfg).items()}
    for over, status in [(dict(head_dim=31), pd.PD_ERR_SHAPE), (dict(n_q_heads=3), pd.PD_ERR_SHAPE),
                         (dict(n_experts=4, top_k=5), pd.PD_ERR_SHAPE)]:
        with pytest.raises(pd.PdError) as e:
            pd.pd_layer_create(dict(cfg, **over), w)
        assert e.value.status == status
    w2 = dict(w)
    w2["w_o"] = None
    with pytest.raises(pd.PdError) as e:
        pd.pd_layer_create(cfg, w2)
    assert e.value.status == pd.PD_ERR_INVALID_ARG


def test_deterministic_across_runs():
    cfg = I.small_config(dtype="bf16")
    ol, gl = both(cfg, std=0.08)
    x = I.hidden(300, cfg["d_model"], seed=1, dtype="bf16")
    cu = np.array([0, 100, 300], np.int32)
    a = gl.prefill(x, cu)
    for _ in range(3):
        assert np.array_equal(gl.prefill(x, cu), a)
    gl.close()


def test_stream_copy_is_bit_exact_and_checks_arguments():
    rng = np.random.default_rng(5)
    src = torch.from_numpy(rng.integers(-2**31, 2**31 - 1, (1 << 20) + 12).astype(np.int32)).cuda()
    for n in (4, 4 * 257, (1 << 20) + 12):       # 16 bytes, a ragged tail, many grid strides
        dst = torch.zeros(n + 4, dtype=torch.int32, device="cuda")
        pd.pd_stream_copy(dst[:n], src[:n])
        torch.cuda.synchronize()
        assert torch.equal(dst[:n], src[:n])
        assert int(dst[n:].abs().max()) == 0     # nothing written past the end
    with pytest.raises(pd.PdError) as e:
        pd.pd_stream_copy(torch.zeros(6, dtype=torch.int32, device="cuda"), src[:6])   # 24 bytes
    assert e.value.status == pd.PD_ERR_INVALID_ARG
    with pytest.raises(pd.PdError):
        pd.pd_stream_copy(torch.zeros(9, dtype=torch.int32, device="cuda")[1:], src[:8])  # misaligned


def test_mfma_probe_sums_and_checks_arguments():
    """The register-only matrix-instruction loop (a measurement aid): what it leaves in its sink is a
    closed form.  A lane's sink value is the sum over its 8 accumulator blocks x 16 registers; with all
    operands 1 every accumulator element grows by the 16-deep contraction per instruction, so the value
    is 8 * 16 * 16 * iters.  With one A fragment set to 2 for every lane the four blocks fed by it double."""
    iters, n_wg = 37, 3
    a = torch.ones(16384, dtype=torch.bfloat16, device="cuda")
    b = torch.ones(8192, dtype=torch.bfloat16, device="cuda")
    sink = torch.zeros(n_wg * 512 + 5, dtype=torch.float32, device="cuda")
    pd.pd_mfma_probe(a, b, n_wg, iters, sink)
    torch.cuda.synchronize()
    assert torch.all(sink[:n_wg * 512] == 8 * 16 * 16 * iters) and torch.all(sink[n_wg * 512:] == 0)
    a2 = a.clone().view(512, 4, 8)
    a2[:, 1, :] = 2.0                                   # fragment 1 of every lane
    pd.pd_mfma_probe(a2.reshape(-1).contiguous(), b, n_wg, iters, sink)
    torch.cuda.synchronize()
    assert torch.all(sink[:n_wg * 512] == (6 + 2 * 2) * 16 * 16 * iters)
    import ctypes as C
    st = pd.lib.pd_mfma_probe(C.c_void_p(a.data_ptr()), C.c_void_p(b.data_ptr()), C.c_int32(0), C.c_int32(5),
                              C.c_void_p(sink.data_ptr()), None)
    assert st == pd.PD_ERR_INVALID_ARG
    st = pd.lib.pd_mfma_probe(C.c_void_p(a.data_ptr() + 2), C.c_void_p(b.data_ptr()), C.c_int32(1), C.c_int32(5),
                              C.c_void_p(sink.data_ptr()), None)
    assert st == pd.PD_ERR_INVALID_ARG


@pytest.mark.parametrize("B", [1, 3, 8, 9, 40])
def test_bf16_moe_decode_batch_sizes(B):
    """Mixture-of-experts decode on the matrix-core path: up to 16 (token, expert) pairs run the
    grouped skinny GEMM (only chosen experts are streamed), more run the grouped tiled GEMM with
    tiles sized by the mean group; routing decisions are compared bit for bit."""
    cfg = I.small_config(dtype="bf16", d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=128, d_ff=256,
                         n_experts=8, top_k=2)
    ol, gl = both(cfg, std=0.05)
    rng = np.random.default_rng(100 + B)
    lens = rng.integers(1, 200, B)
    cap = 208
    oc, gc = O.KVCache(ol, B, cap), gl.cache(B, cap)
    for i, n in enumerate(lens):
        k, v = I.kv_fill(2, int(n), 128, seed=2000 + i, dtype="bf16")
        oc.set(i, k, v)
        pd.pd_kv_cache_set(gc, i, to_dev(k, "bf16"), to_dev(v, "bf16"))
    slots = list(range(B))
    for step in range(2):
        xn = I.hidden(B, cfg["d_model"], seed=41 + step, dtype="bf16")
        rn = I.router_logits(B, 8, seed=51 + step)
        if B >= 3:
            rn[1] = rn[0]                         # two tokens with the same experts
            rn[2, :] = 0.5                        # all-equal logits: experts 0 and 1
        ref, eref = O.decode_step(ol, xn, slots, oc, router_logits=rn, return_experts=True)
        got = gl.decode(xn, slots, gc, router_logits=rn)
        assert np.array_equal(gl.experts(B), eref)
        assert relmax(got, ref) <= TOL["bf16"]
        assert max(relmax(got[i], ref[i]) for i in range(B)) <= 2 * TOL["bf16"]
    gl.close()


def test_bf16_moe_decode_all_tokens_on_two_experts():
    """20 tokens that all choose experts 3 and 5: groups of 20 rows, i.e. two passes of the grouped
    skinny GEMM over those experts' weights, and six experts that are never read."""
    cfg = I.small_config(dtype="bf16", d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=128, d_ff=256,
                         n_experts=8, top_k=2)
    ol, gl = both(cfg, std=0.05)
    B, cap = 20, 80
    oc, gc = O.KVCache(ol, B, cap), gl.cache(B, cap)
    for i in range(B):
        k, v = I.kv_fill(2, 10 + 3 * i, 128, seed=3000 + i, dtype="bf16")
        oc.set(i, k, v)
        pd.pd_kv_cache_set(gc, i, to_dev(k, "bf16"), to_dev(v, "bf16"))
    xn = I.hidden(B, cfg["d_model"], seed=43, dtype="bf16")
    rn = I.router_logits(B, 8, seed=53) * 0.1
    rn[:, 3] += 5.0
    rn[:, 5] += 4.0
    slots = list(range(B))
    ref, eref = O.decode_step(ol, xn, slots, oc, router_logits=rn, return_experts=True)
    got = gl.decode(xn, slots, gc, router_logits=rn)
    assert np.array_equal(eref, np.tile([3, 5], (B, 1)))
    assert np.array_equal(gl.experts(B), eref)
    assert relmax(got, ref) <= TOL["bf16"]
    assert max(relmax(got[i], ref[i]) for i in range(B)) <= 2 * TOL["bf16"]
    gl.close()
