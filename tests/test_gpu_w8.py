"""GPU parity of layers with 8-bit (E4M3, per-row power-of-two scale) projection weights against the
CPU oracle run on the same quantised weights (bf16 bound 2e-2)."""
import numpy as np
import pytest
import torch

import paper_2603_04716_amd as pd
import pd_inputs as I
from oracle import layer as O
from gpu_util import GpuLayer, TOL, relmax, to_dev

pytestmark = pytest.mark.gpu


def both(cfg, std=0.05, seed=None, with_router=False):
    w = I.layer_weights(cfg, seed=seed, std=std, with_router=with_router)
    return O.Layer(cfg, O.quantise_layer_weights(w)), GpuLayer(cfg, w, w8=True)


def small(hq=4, hkv=2, d=256, F=512, **kw):
    return I.small_config(dtype="bf16", d_model=d, n_q_heads=hq, n_kv_heads=hkv, head_dim=128, d_ff=F, **kw)


@pytest.mark.parametrize("B", [1, 2, 7, 16, 17, 40, 130])
def test_decode_batches_on_both_sides_of_the_skinny_kernel(B):
    """Up to 16 rows stream the 8-bit codes through the skinny kernel; above that the wide kernel does
    where K is a multiple of 512 (here the O and down projections) and the bf16 copy of the same
    quantised weights runs the tiled kernels elsewhere: one oracle for all."""
    cfg = small()
    ol, gl = both(cfg)
    rng = np.random.default_rng(B)
    lens = rng.integers(0, 200, B)
    oc, gc = O.KVCache(ol, B, 208), gl.cache(B, 208)
    for i, n in enumerate(lens):
        k, v = I.kv_fill(2, int(n), 128, seed=3000 + i, dtype="bf16")
        oc.set(i, k, v)
        if n > 0:
            pd.pd_kv_cache_set(gc, i, to_dev(k, "bf16"), to_dev(v, "bf16"))
    slots = list(range(B))
    for step in range(2):
        xn = I.hidden(B, cfg["d_model"], seed=51 + step, dtype="bf16")
        ref = O.decode_step(ol, xn, slots, oc)
        got = gl.decode(xn, slots, gc)
        assert relmax(got, ref) <= TOL["bf16"]
        assert max(relmax(got[i], ref[i]) for i in range(B)) <= 2 * TOL["bf16"]
    gl.close()


@pytest.mark.parametrize("d,F,hq,hkv", [(256, 512, 4, 2), (512, 8192, 4, 1), (8192 // 8, 256, 8, 8), (320, 576, 5, 5)])
def test_shapes_long_and_short_k_prefill_then_decode(d, F, hq, hkv):
    """K below and above the long-K variant's threshold (down projection with F = 8192), K not a
    multiple of the per-wave pair count, square and wide shapes; prefill (tiled kernels) writes the
    cache, decode (skinny kernels) reads it."""
    cfg = small(hq, hkv, d, F)
    ol, gl = both(cfg, std=0.03)
    cu = np.array([0, 70, 71, 131], np.int32)
    x = I.hidden(131, d, seed=8, dtype="bf16")
    oc, gc = O.KVCache(ol, 3, 96), gl.cache(3, 96)
    ref = O.prefill(ol, x, cu, cache=oc, slots=[0, 1, 2])
    got = gl.prefill(x, cu, cache=gc, slots=[0, 1, 2])
    assert relmax(got, ref) <= TOL["bf16"]
    for step in range(3):
        xn = I.hidden(3, d, seed=80 + step, dtype="bf16")
        ref = O.decode_step(ol, xn, [0, 1, 2], oc)
        got = gl.decode(xn, [0, 1, 2], gc)
        assert relmax(got, ref) <= TOL["bf16"], step
    gl.close()


@pytest.mark.parametrize("d,F,hq,hkv", [(512, 1024, 4, 2), (1024, 512, 8, 8), (2048, 512, 16, 4), (576, 512, 4, 1)])
@pytest.mark.parametrize("B", [17, 32, 33, 64, 65, 96, 97, 128])
def test_wide_kernel_batches_17_to_128(B, d, F, hq, hkv):
    """Every row-block count of the wide 8-bit kernel (2, 4, 6, 8 blocks of 16 rows, full and ragged),
    with all four projections on it (every K a multiple of 512), K split over workgroups for the plain,
    residual and SwiGLU epilogues (second shape; the third has K = 2048, which the 16-deep ring of the
    smaller batches splits as well) and a last workgroup with weight blocks past the end (last shape: 576 output columns of the O and down projections; its other two products have
    K = 576 and stay on the tiled kernels)."""
    cfg = small(hq, hkv, d, F)
    ol, gl = both(cfg, std=0.04, seed=B)
    rng = np.random.default_rng(1000 + B)
    lens = rng.integers(1, 90, B)
    oc, gc = O.KVCache(ol, B, 96), gl.cache(B, 96)
    for i, n in enumerate(lens):
        k, v = I.kv_fill(hkv, int(n), 128, seed=4000 + i, dtype="bf16")
        oc.set(i, k, v)
        pd.pd_kv_cache_set(gc, i, to_dev(k, "bf16"), to_dev(v, "bf16"))
    slots = list(range(B))
    xn = I.hidden(B, d, seed=52, dtype="bf16")
    ref = O.decode_step(ol, xn, slots, oc)
    got = gl.decode(xn, slots, gc)
    assert relmax(got, ref) <= TOL["bf16"]
    assert max(relmax(got[i], ref[i]) for i in range(B)) <= 2 * TOL["bf16"]
    gl.close()


@pytest.mark.parametrize("B", [1, 6, 40])
def test_moe_layer_with_8bit_expert_weights(B):
    cfg = small(4, 2, n_experts=4, top_k=2)
    ol, gl = both(cfg, with_router=True)
    oc, gc = O.KVCache(ol, B, 64), gl.cache(B, 64)
    for i in range(B):
        k, v = I.kv_fill(2, 5 + i % 50, 128, seed=700 + i, dtype="bf16")
        oc.set(i, k, v)
        pd.pd_kv_cache_set(gc, i, to_dev(k, "bf16"), to_dev(v, "bf16"))
    xn = I.hidden(B, cfg["d_model"], seed=61, dtype="bf16")
    rl = I.router_logits(B, 4, seed=62)
    ref, eref = O.decode_step(ol, xn, list(range(B)), oc, router_logits=rl, return_experts=True)
    got = gl.decode(xn, list(range(B)), gc, router_logits=rl)
    assert np.array_equal(np.sort(gl.experts(B), axis=1), np.sort(eref, axis=1))
    assert relmax(got, ref) <= TOL["bf16"]
    gl.close()


def test_w8_needs_a_matrix_core_layer():
    for cfg in (I.small_config(), small(d=200, F=512)):
        w = I.layer_weights(cfg)
        dev = {k: to_dev(v, cfg["dtype"]) for k, v in w.items()}
        with pytest.raises(pd.PdError) as e:
            pd.pd_layer_create(cfg, dev, w8=True)
        assert e.value.status == pd.PD_ERR_DTYPE


def test_llama8b_shape_w8_decode_sampled_rows_with_fp8_cache():
    """8B-shaped layer, 8-bit weights and 8-bit cache together, batch 8 (skinny kernels), 48 and 128
    (wide kernel, 4 and 8 row blocks); the oracle recomputes sampled rows."""
    cfg = I.CONFIGS["llama8b"]
    w = I.layer_weights(cfg)
    ol, gl = O.Layer(cfg, O.quantise_layer_weights(w)), GpuLayer(cfg, w, w8=True)
    scales = (0.5, 0.125)
    S = 700
    k, v = I.kv_fill(cfg["n_kv_heads"], S, 128, seed=43, dtype="bf16")
    kd, vd = to_dev(k, "bf16"), to_dev(v, "bf16")
    for B, rows in ((8, [0, 7]), (48, [3, 47]), (128, [0, 127])):
        gc = gl.cache(B, S + 8, fp8_scales=scales)
        for i in range(B):
            pd.pd_kv_cache_set(gc, i, kd[:, :S - i].contiguous(), vd[:, :S - i].contiguous())
        xn = I.hidden(B, cfg["d_model"], seed=44 + B, dtype="bf16")
        got = gl.decode(xn, list(range(B)), gc)
        oc = O.KVCache(ol, len(rows), S + 8, fp8_scales=scales)
        for j, i in enumerate(rows):
            oc.set(j, k[:, :S - i], v[:, :S - i])
        ref = O.decode_step(ol, xn[rows], list(range(len(rows))), oc)
        for j, i in enumerate(rows):
            assert relmax(got[i], ref[j]) <= TOL["bf16"], (B, i)
    gl.close()
