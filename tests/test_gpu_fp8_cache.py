"""GPU parity of the KV cache held as 8-bit E4M3 codes with static scales: the codec bit for bit
against the oracle's, and decode / chunked prefill over such a cache against the oracle run with
the same cache semantics (bf16 bound 2e-2)."""
import numpy as np
import pytest
import torch

import paper_2603_04716_amd as pd
import pd_inputs as I
from oracle import layer as O
from gpu_util import GpuLayer, TOL, relmax, to_dev, to_np

pytestmark = pytest.mark.gpu


def both(cfg, std=0.05, seed=None, with_router=False):
    w = I.layer_weights(cfg, seed=seed, std=std, with_router=with_router)
    return O.Layer(cfg, w), GpuLayer(cfg, w)


def small(hq=4, hkv=2, **kw):
    return I.small_config(dtype="bf16", d_model=256, n_q_heads=hq, n_kv_heads=hkv, head_dim=128, d_ff=512, **kw)


def bf16_round(a):
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(torch.bfloat16).float().numpy()


def cache_mismatch(gl, gc, oc, slot, n):
    """Read-back of the first n positions of a slot against the oracle's cache: the fraction of
    elements that differ, and the largest difference in excess of what rounding to a code can add
    to the bf16 error of the unquantised value (one spacing of the representable values there)."""
    hkv = oc.k.shape[1]
    kk = torch.empty((hkv, n, 128), dtype=torch.bfloat16, device="cuda")
    vv = torch.empty_like(kk)
    pd.pd_kv_cache_get(gc, slot, kk, vv)
    torch.cuda.synchronize()
    frac, excess = 0.0, -1.0
    for got, ref, scale in ((to_np(kk), oc.k[slot, :, :n], oc.k_scale), (to_np(vv), oc.v[slot, :, :n], oc.v_scale)):
        ref = bf16_round(ref)
        diff = np.abs(got - ref) / scale
        mag = np.maximum(np.maximum(np.abs(ref), np.abs(got)) / scale, 2.0 ** -6)
        spacing = 2.0 ** (np.floor(np.log2(mag)) - 3)
        frac = max(frac, float(np.mean(diff > 0)))
        excess = max(excess, float(np.max(diff - spacing - TOL["bf16"] * np.max(np.abs(ref)) / scale)))
    return frac, excess


@pytest.mark.parametrize("scales", [(1.0, 1.0), (0.75, 0.0625), (3.0, 1.7)])
def test_codec_matches_the_oracle_on_every_bf16_value(scales):
    """pd_kv_cache_set then _get returns scale * fp8(x / scale) for every one of the 65536 bf16 bit
    patterns (ties, subnormals of both formats, saturation, infinities; NaNs aside), bit for bit
    the oracle's value rounded to bf16, for keys and values in every layout position class."""
    cfg = small()
    ol, gl = both(cfg)
    bits = np.arange(65536, dtype=np.uint32)
    vals = (bits << 16).astype(np.uint32).view(np.float32).copy()
    vals[np.isnan(vals)] = 0.0
    k = vals.reshape(2, 256, 128)
    v = np.random.default_rng(5).permutation(vals).reshape(2, 256, 128)
    oc, gc = O.KVCache(ol, 2, 256, fp8_scales=scales), gl.cache(2, 256, fp8_scales=scales)
    oc.set(1, k, v)
    pd.pd_kv_cache_set(gc, 1, to_dev(k, "bf16"), to_dev(v, "bf16"))
    kk = torch.empty((2, 256, 128), dtype=torch.bfloat16, device="cuda")
    vv = torch.empty_like(kk)
    pd.pd_kv_cache_get(gc, 1, kk, vv)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(kk), bf16_round(oc.k[1]))
    assert np.array_equal(to_np(vv), bf16_round(oc.v[1]))
    gl.close()


@pytest.mark.parametrize("hq,hkv", [(4, 2), (4, 1), (16, 1), (2, 2)])
def test_prefill_fills_and_decode_reads_the_fp8_cache(hq, hkv):
    """Prefill attends over fresh keys and values and stores codes; 40 decode steps then read only
    codes, crossing the 16- and 64-position block boundaries of the 8-bit layout."""
    cfg = small(hq, hkv)
    ol, gl = both(cfg)
    scales = (0.5, 0.25)
    cu = np.array([0, 150, 151, 151, 280, 343], np.int32)
    x = I.hidden(int(cu[-1]), cfg["d_model"], seed=71, dtype="bf16")
    slots = [4, 0, 1, 3, 2]
    oc, gc = O.KVCache(ol, 5, 200, fp8_scales=scales), gl.cache(5, 200, fp8_scales=scales)
    ref = O.prefill(ol, x, cu, cache=oc, slots=slots)
    got = gl.prefill(x, cu, cache=gc, slots=slots)
    assert relmax(got, ref) <= TOL["bf16"]
    # stored codes: the two sides round independently computed bf16 / fp64 values, so a small
    # fraction lands on another code, no further than the bf16 error plus one spacing
    frac, excess = cache_mismatch(gl, gc, oc, 4, 150)
    assert frac < 0.12 and excess <= 0.0, (frac, excess)
    for step in range(40):
        xn = I.hidden(5, cfg["d_model"], seed=720 + step, dtype="bf16")
        ref = O.decode_step(ol, xn, slots, oc)
        got = gl.decode(xn, slots, gc)
        assert relmax(got, ref) <= TOL["bf16"], step
        for i in range(5):
            assert relmax(got[i], ref[i]) <= 2 * TOL["bf16"], (step, i)
    assert pd.pd_kv_cache_len(gc, 4) == 190
    gl.close()


@pytest.mark.parametrize("B", [1, 7, 64, 130])
def test_decode_over_a_filled_fp8_cache_many_chunks(B):
    """Ragged caches filled through pd_kv_cache_set (identical codes on both sides), long enough
    that sequences are cut into several chunks and merged."""
    cfg = small()
    ol, gl = both(cfg)
    scales = (0.25, 0.125)
    rng = np.random.default_rng(100 + B)
    lens = rng.integers(0, 700, B)
    lens[0] = 699
    cap = 704
    oc, gc = O.KVCache(ol, B, cap, fp8_scales=scales), gl.cache(B, cap, fp8_scales=scales)
    for i, n in enumerate(lens):
        k, v = I.kv_fill(2, int(n), 128, seed=2000 + i, dtype="bf16")
        oc.set(i, k, v)
        if n > 0:
            pd.pd_kv_cache_set(gc, i, to_dev(k, "bf16"), to_dev(v, "bf16"))
    slots = list(range(B))
    for step in range(2):
        xn = I.hidden(B, cfg["d_model"], seed=81 + step, dtype="bf16")
        ref = O.decode_step(ol, xn, slots, oc)
        got = gl.decode(xn, slots, gc)
        assert relmax(got, ref) <= TOL["bf16"]
        assert max(relmax(got[i], ref[i]) for i in range(B)) <= 2 * TOL["bf16"]
    gl.close()


@pytest.mark.parametrize("chunk", [3, 8, 9, 100])
def test_chunked_prefill_over_the_fp8_cache(chunk):
    """Chunks of <= 8 tokens run on the decode attention kernel, longer ones on the gathered prefill
    kernel; in both every key and value, the chunk's own included, is read back from the codes."""
    cfg = small(4, 2)
    ol, gl = both(cfg)
    scales = (0.5, 0.5)
    lens = [230, 1, 77]
    oc, gc = O.KVCache(ol, 3, 256, fp8_scales=scales), gl.cache(3, 256, fp8_scales=scales)
    done = [0, 0, 0]
    step = 0
    while any(d < n for d, n in zip(done, lens)):
        take = [min(chunk, n - d) for d, n in zip(done, lens)]
        live = [s for s in range(3) if take[s] > 0]
        cu = np.concatenate([[0], np.cumsum([take[s] for s in live])]).astype(np.int32)
        x = I.hidden(int(cu[-1]), cfg["d_model"], seed=900 + step, dtype="bf16")
        ref = O.prefill_chunk(ol, x, cu, live, oc)
        got = gl.prefill_chunk(x, cu, live, gc)
        assert relmax(got, ref) <= TOL["bf16"], step
        for j, s in enumerate(live):
            assert relmax(got[cu[j]:cu[j + 1]], ref[cu[j]:cu[j + 1]]) <= 2 * TOL["bf16"], (step, s)
            done[s] += take[s]
        step += 1
        if chunk < 10 and step >= 12:
            break
    gl.close()


def test_moe_layer_decodes_over_the_fp8_cache():
    cfg = small(4, 2, n_experts=4, top_k=2)
    ol, gl = both(cfg, with_router=True)
    scales = (0.5, 0.25)
    B = 9
    oc, gc = O.KVCache(ol, B, 128, fp8_scales=scales), gl.cache(B, 128, fp8_scales=scales)
    for i in range(B):
        k, v = I.kv_fill(2, 10 + 11 * i, 128, seed=300 + i, dtype="bf16")
        oc.set(i, k, v)
        pd.pd_kv_cache_set(gc, i, to_dev(k, "bf16"), to_dev(v, "bf16"))
    xn = I.hidden(B, cfg["d_model"], seed=33, dtype="bf16")
    rl = I.router_logits(B, 4, seed=34)
    ref = O.decode_step(ol, xn, list(range(B)), oc, router_logits=rl)
    got = gl.decode(xn, list(range(B)), gc, router_logits=rl)
    assert relmax(got, ref) <= TOL["bf16"]
    gl.close()


def test_fp8_cache_argument_errors():
    cfg = small()
    ol, gl = both(cfg)
    for ks, vs in [(0.0, 1.0), (1.0, -1.0), (float("inf"), 1.0), (float("nan"), 1.0)]:
        with pytest.raises(pd.PdError) as e:
            pd.pd_kv_cache_create_fp8(gl.h, 2, 64, ks, vs)
        assert e.value.status == pd.PD_ERR_INVALID_ARG
    gl.close()
    # layers the 8-bit layout does not cover: fp32, head_dim != 128
    for cfg in (I.small_config(), I.small_config(dtype="bf16", d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ff=512)):
        ol, gl = both(cfg)
        with pytest.raises(pd.PdError) as e:
            pd.pd_kv_cache_create_fp8(gl.h, 2, 64, 1.0, 1.0)
        assert e.value.status == pd.PD_ERR_DTYPE
        gl.close()


def test_llama8b_shape_decode_over_fp8_cache_sampled_rows():
    """The 8B-shaped layer at the decode shape the bench times (8 kv heads, group 4, 2048 cached
    tokens), a batch of 64 with ragged lengths; the oracle recomputes four sampled rows."""
    cfg = I.CONFIGS["llama8b"]
    w = I.layer_weights(cfg)
    ol, gl = O.Layer(cfg, w), GpuLayer(cfg, w)
    scales = (0.5, 0.125)
    B, cap = 64, 2112
    rng = np.random.default_rng(8)
    lens = rng.integers(1500, 2100, B)
    lens[5] = 2100
    k, v = I.kv_fill(cfg["n_kv_heads"], 2100, 128, seed=41, dtype="bf16")
    kd, vd = to_dev(k, "bf16"), to_dev(v, "bf16")
    gc = gl.cache(B, cap, fp8_scales=scales)
    for i in range(B):
        pd.pd_kv_cache_set(gc, i, kd[:, :int(lens[i])].contiguous(), vd[:, :int(lens[i])].contiguous())
    xn = I.hidden(B, cfg["d_model"], seed=42, dtype="bf16")
    got = gl.decode(xn, list(range(B)), gc)
    rows = [0, 5, 31, 63]
    oc = O.KVCache(ol, len(rows), cap, fp8_scales=scales)
    for j, i in enumerate(rows):
        oc.set(j, k[:, :int(lens[i])], v[:, :int(lens[i])])
    ref = O.decode_step(ol, xn[rows], list(range(len(rows))), oc)
    for j, i in enumerate(rows):
        assert relmax(got[i], ref[j]) <= TOL["bf16"], i
    gl.close()
