"""GPU parity of chunked prefill (pd_prefill_chunk through the C ABI) against the CPU oracle, call
by call on the same seeded inputs and the same chunk plan.  Bounds as for the other layer tests:
max |gpu - ref| / max |ref| <= 1e-5 (fp32), <= 2e-2 (bf16)."""
import numpy as np
import pytest
import torch

import paper_2603_04716_amd as pd
import pd_inputs as I
from oracle import layer as O
from paper_2603_04716_amd import harness as H
from gpu_util import GpuLayer, TOL, relmax, to_dev, to_np

pytestmark = pytest.mark.gpu


def run_plan(cfg, lens, plan, slots, cap, std=0.05, seed=60, with_router=False):
    """Feeds the sequences chunk by chunk to both sides; returns nothing, asserts per call."""
    w = I.layer_weights(cfg, std=std, with_router=with_router)
    ol, gl = O.Layer(cfg, w), GpuLayer(cfg, w)
    dt = cfg["dtype"]
    tol = TOL[dt]
    xs = [I.hidden(n, cfg["d_model"], seed=seed + i, dtype=dt) for i, n in enumerate(lens)]
    oc, gc = O.KVCache(ol, max(slots) + 1, cap), gl.cache(max(slots) + 1, cap)
    done = [0] * len(lens)
    for call, chunk in enumerate(plan):
        x = np.concatenate([xs[i][done[i]:done[i] + chunk[i]] for i in range(len(lens))])
        cu = np.concatenate([[0], np.cumsum(chunk)]).astype(np.int32)
        rl = I.router_logits(int(cu[-1]), cfg["n_experts"], seed=seed + 100 + call) if cfg["n_experts"] else None
        ref = O.prefill_chunk(ol, x, cu, slots, oc, router_logits=rl)
        got = gl.prefill_chunk(x, cu, slots, gc, router_logits=rl)
        assert relmax(got, ref) <= tol, call
        for i in range(len(lens)):
            a, b = cu[i], cu[i + 1]
            if b > a:
                assert relmax(got[a:b], ref[a:b]) <= 2 * tol, (call, i)
            done[i] += chunk[i]
            assert pd.pd_kv_cache_len(gc, slots[i]) == done[i] == int(oc.lens[slots[i]])
    return ol, gl, oc, gc, xs


def test_fp32_chunked_prefill_ragged_plan_and_cache_contents():
    cfg = I.small_config()
    lens, slots = [13, 1, 22], [3, 0, 1]
    plan = [[5, 1, 7], [8, 0, 4], [0, 0, 11]]
    ol, gl, oc, gc, xs = run_plan(cfg, lens, plan, slots, cap=24, std=0.08)
    # the caches hold the same rotated keys and values
    for sl, n in zip(slots, lens):
        k = torch.empty((cfg["n_kv_heads"], n, cfg["head_dim"]), device="cuda")
        v = torch.empty_like(k)
        pd.pd_kv_cache_get(gc, sl, k, v)
        torch.cuda.synchronize()
        assert relmax(to_np(k), oc.k[sl, :, :n]) <= 1e-5
        assert relmax(to_np(v), oc.v[sl, :, :n]) <= 1e-5
    # chunked == unchunked on the GPU as well (same tolerance; the two paths order sums differently)
    for i, n in enumerate(lens):
        full = gl.prefill(xs[i], np.array([0, n], np.int32))
        ref = O.prefill(ol, xs[i], np.array([0, n], np.int32))
        assert relmax(full, ref) <= 1e-5
    gl.close()


@pytest.mark.parametrize("hq,hkv", [(4, 1), (8, 2)])
def test_bf16_chunked_prefill_matrix_core_path(hq, hkv):
    """head_dim 128 in bf16: blocked cache, gathered prefix, MFMA attention with the prefix offset.
    Prefixes and chunks span several 64-key tiles and 128-query blocks with ragged tails; one
    sequence gets a one-token chunk, one an empty chunk, one starts from an empty slot."""
    cfg = I.small_config(dtype="bf16", d_model=256, n_q_heads=hq, n_kv_heads=hkv, head_dim=128, d_ff=512)
    lens = [500, 78, 321, 190]
    plan = [[130, 77, 0, 64], [241, 1, 200, 126], [129, 0, 121, 0]]
    ol, gl, oc, gc, xs = run_plan(cfg, lens, plan, [2, 0, 3, 1], cap=512)
    # decode continues from the chunk-filled caches
    slots = [2, 0, 3, 1]
    for step in range(3):
        xn = I.hidden(4, cfg["d_model"], seed=300 + step, dtype="bf16")
        ref = O.decode_step(ol, xn, slots, oc)
        got = gl.decode(xn, slots, gc)
        assert relmax(got, ref) <= TOL["bf16"], step
    gl.close()


@pytest.mark.parametrize("hq,hkv", [(4, 1), (8, 4), (6, 2)])
def test_bf16_chunked_prefill_long_prefix_splits_the_keys(hq, hkv):
    """Few query blocks behind a long prefix: the key tiles of a query block are divided over
    several workgroups and merged by a second kernel.  The second and third calls split four ways
    (2100 and 2300 keys at most); the short sequences leave some splits with one tile or none.
    Groups of 4 and 2 heads run two heads per workgroup, the group of 3 one."""
    cfg = I.small_config(dtype="bf16", d_model=256, n_q_heads=hq, n_kv_heads=hkv, head_dim=128, d_ff=256)
    lens = [2300, 1100, 150]
    plan = [[1200, 500, 0], [900, 77, 50], [200, 523, 100]]
    ol, gl, oc, gc, xs = run_plan(cfg, lens, plan, [1, 2, 0], cap=2304)
    gl.close()


def test_bf16_chunked_prefill_moe():
    cfg = I.small_config(dtype="bf16", d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=128, d_ff=256,
                         n_experts=4, top_k=2)
    ol, gl, oc, gc, xs = run_plan(cfg, [150, 90], [[70, 90], [80, 0]], [0, 1], cap=192)
    gl.close()


def test_chunk_errors_leave_state():
    cfg = I.small_config()
    w = I.layer_weights(cfg)
    gl = GpuLayer(cfg, w)
    gc = gl.cache(2, 6)
    x = I.hidden(4, cfg["d_model"], seed=1)
    gl.prefill(x, [0, 4], cache=gc, slots=[1])
    xd = to_dev(I.hidden(4, cfg["d_model"], seed=2), "f32")
    out = torch.empty_like(xd)
    with pytest.raises(pd.PdError) as e:                      # 4 + 3 > 6
        pd.pd_prefill_chunk(gl.h, xd, [0, 1, 4], [0, 1], gc, out)
    assert e.value.status == pd.PD_ERR_KV_CAPACITY
    with pytest.raises(pd.PdError) as e:                      # repeated slot
        pd.pd_prefill_chunk(gl.h, xd[:2], [0, 1, 2], [1, 1], gc, out[:2])
    assert e.value.status == pd.PD_ERR_INVALID_ARG
    with pytest.raises(pd.PdError) as e:                      # no cache
        pd.pd_prefill_chunk(gl.h, xd[:2], [0, 2], [1], None, out[:2])
    assert e.value.status == pd.PD_ERR_INVALID_ARG
    assert pd.pd_kv_cache_len(gc, 1) == 4 and pd.pd_kv_cache_len(gc, 0) == 0
    pd.pd_prefill_chunk(gl.h, xd[:2], [0, 2], [1], gc, out[:2])   # exactly full
    torch.cuda.synchronize()
    assert pd.pd_kv_cache_len(gc, 1) == 6
    gl.close()


def test_llama8b_chunk_against_cached_prefix_sampled_rows():
    """Full shape: two sequences with prefixes of 2048 and 1000 tokens (cached by pd_prefill), then a
    chunk of 2048 and of 1500 tokens.  Chunked == unchunked prefill (pinned for the oracle), so
    the reference rows are sampled rows of the oracle's prefill of the whole sequences."""
    cfg = I.CONFIGS["llama8b"]
    w = I.layer_weights(cfg)
    layer = H.Layer(cfg, w)
    pre, chk = [2048, 1000], [2048, 1500]
    xs = [I.hidden(pre[i] + chk[i], cfg["d_model"], seed=70 + i, dtype="bf16") for i in range(2)]
    cache = layer.new_cache(2, 4096)
    xp = H._dev(np.concatenate([xs[i][:pre[i]] for i in range(2)]), "bf16")
    out_p = torch.empty_like(xp)
    pd.pd_prefill(layer.h, xp, [0, pre[0], pre[0] + pre[1]], out_p, cache, [0, 1])
    xc = H._dev(np.concatenate([xs[i][pre[i]:] for i in range(2)]), "bf16")
    out_c = torch.empty_like(xc)
    pd.pd_prefill_chunk(layer.h, xc, [0, chk[0], chk[0] + chk[1]], [0, 1], cache, out_c)
    torch.cuda.synchronize()
    got = to_np(out_c)
    assert np.isfinite(got).all()
    assert pd.pd_kv_cache_len(cache, 0) == 4096 and pd.pd_kv_cache_len(cache, 1) == 2500
    ol = O.Layer(cfg, w)
    for i, rows_in_chunk in enumerate([[0, 63, 1000, 2047], [0, 129, 1499]]):
        rows = [pre[i] + r for r in rows_in_chunk]
        ref = O.prefill(ol, xs[i], np.array([0, pre[i] + chk[i]], np.int32), rows=rows)
        mine = got[[(chk[0] if i else 0) + r for r in rows_in_chunk]]
        assert relmax(mine, ref) <= TOL["bf16"], i
        for j in range(len(rows)):
            assert relmax(mine[j], ref[j]) <= 2 * TOL["bf16"], (i, rows[j])
    layer.close()


def test_llama8b_small_chunk_behind_a_long_prefix_sampled_rows():
    """Full shape, the launch the chunk sweep times: one 512-token chunk behind 3584 cached tokens
    (64 eight-wave workgroups unsplit, so the keys are split four ways).  Reference rows as in the
    test above: sampled rows of the oracle's prefill of the whole sequence."""
    cfg = I.CONFIGS["llama8b"]
    w = I.layer_weights(cfg)
    layer = H.Layer(cfg, w)
    pre, chk = 3584, 512
    xs = I.hidden(pre + chk, cfg["d_model"], seed=75, dtype="bf16")
    cache = layer.new_cache(1, 4096)
    xp = H._dev(xs[:pre], "bf16")
    pd.pd_prefill(layer.h, xp, [0, pre], torch.empty_like(xp), cache, [0])
    xc = H._dev(xs[pre:], "bf16")
    out_c = torch.empty_like(xc)
    pd.pd_prefill_chunk(layer.h, xc, [0, chk], [0], cache, out_c)
    torch.cuda.synchronize()
    got = to_np(out_c)
    assert np.isfinite(got).all()
    assert pd.pd_kv_cache_len(cache, 0) == 4096
    rows_in_chunk = [0, 31, 127, 128, 300, 511]
    ref = O.prefill(O.Layer(cfg, w), xs, np.array([0, pre + chk], np.int32), rows=[pre + r for r in rows_in_chunk])
    mine = got[rows_in_chunk]
    assert relmax(mine, ref) <= TOL["bf16"]
    for j in range(len(rows_in_chunk)):
        assert relmax(mine[j], ref[j]) <= 2 * TOL["bf16"], rows_in_chunk[j]
    layer.close()


@pytest.mark.parametrize("hq,hkv", [(4, 1), (8, 2), (2, 2), (8, 1), (16, 1)])
def test_bf16_multi_token_decode_steps(hq, hkv):
    """Chunks of at most 8 tokens over a blocked cache take the decode attention kernel with units
    of 16 / group tokens sharing one pass over the cache (group 4: 4 tokens, 1: 16, 8: 2, 16: 1):
    steps of ragged size (0..8 tokens per sequence) after a long first chunk, crossing 16-, 32- and
    64-position block boundaries of the cache."""
    cfg = I.small_config(dtype="bf16", d_model=256, n_q_heads=hq, n_kv_heads=hkv, head_dim=128, d_ff=512)
    lens = [200 + 4 + 3 + 8 + 8, 61 + 8 + 0 + 8 + 2, 130 + 1 + 8 + 8 + 7]
    plan = [[200, 61, 130], [4, 8, 1], [3, 0, 8], [8, 8, 8], [8, 2, 7]]
    ol, gl, oc, gc, xs = run_plan(cfg, lens, plan, [1, 2, 0], cap=256)
    xn = I.hidden(3, cfg["d_model"], seed=301, dtype="bf16")
    ref = O.decode_step(ol, xn, [1, 2, 0], oc)
    got = gl.decode(xn, [1, 2, 0], gc)
    assert relmax(got, ref) <= TOL["bf16"]
    gl.close()


@pytest.mark.parametrize("n_seqs,q", [(512, 1), (1024, 2), (700, 3)])
def test_bf16_multi_token_decode_of_many_sequences(n_seqs, q):
    """A multi-token decode step over hundreds of sequences (what a decode batch of several hundred
    with multi-token prediction issues): 512 slots x 1 token, 1024 slots x 2 tokens, 700 x 3.  Every
    unit of tokens needs at least one partial-result chunk, more than a one-token decode step of the
    same row count does at the 8B head layout (32 query heads over 8 kv heads)."""
    cfg = I.small_config(dtype="bf16", d_model=256, n_q_heads=32, n_kv_heads=8, head_dim=128, d_ff=512)
    w = I.layer_weights(cfg, std=0.05)
    ol, gl = O.Layer(cfg, w), GpuLayer(cfg, w)
    rng = np.random.default_rng(n_seqs)
    prefix = rng.integers(0, 90, n_seqs)
    prefix[:3] = [0, 1, 89]
    cap = 96
    oc, gc = O.KVCache(ol, n_seqs, cap), gl.cache(n_seqs, cap)
    k, v = I.kv_fill(8, 89, 128, seed=5, dtype="bf16")
    kd, vd = to_dev(k, "bf16"), to_dev(v, "bf16")
    for s_ in range(n_seqs):
        n = int(prefix[s_])
        oc.set(s_, k[:, :n], v[:, :n])
        pd.pd_kv_cache_set(gc, s_, kd[:, :n].contiguous(), vd[:, :n].contiguous())
    slots = list(rng.permutation(n_seqs).astype(int))
    cu = (np.arange(n_seqs + 1) * q).astype(np.int32)
    x = I.hidden(n_seqs * q, cfg["d_model"], seed=6, dtype="bf16")
    ref = O.prefill_chunk(ol, x, cu, slots, oc)
    got = gl.prefill_chunk(x, cu, slots, gc)
    assert relmax(got, ref) <= TOL["bf16"]
    for i in (0, 1, 2, n_seqs // 2, n_seqs - 1):
        assert relmax(got[cu[i]:cu[i + 1]], ref[cu[i]:cu[i + 1]]) <= 2 * TOL["bf16"], i
    assert all(pd.pd_kv_cache_len(gc, s_) == int(oc.lens[s_]) for s_ in (slots[0], slots[-1]))
    # and the plain decode step that follows reads what the multi-token step appended
    xn = I.hidden(n_seqs, cfg["d_model"], seed=7, dtype="bf16")
    ref = O.decode_step(ol, xn, slots, oc)
    got = gl.decode(xn, slots, gc)
    assert relmax(got, ref) <= TOL["bf16"]
    gl.close()
