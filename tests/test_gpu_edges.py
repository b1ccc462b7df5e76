"""GPU parity at the edges of the interface: the largest batch and sequence count a call takes,
work splits of the decode attention around their switch points, empty caches."""
import numpy as np
import pytest
import torch

import paper_2603_04716_amd as pd
import pd_inputs as I
from oracle import layer as O
from gpu_util import GpuLayer, TOL, relmax, to_dev

pytestmark = pytest.mark.gpu

MAX_SEQS = 4096          # sequences / batch rows one call takes


def both(cfg, std=0.05):
    w = I.layer_weights(cfg, std=std)
    return O.Layer(cfg, w), GpuLayer(cfg, w)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_decode_with_the_largest_batch_and_one_more(dtype):
    """4096 sequences in one decode step (ragged caches, some empty), then 4097 is refused."""
    if dtype == "bf16":
        cfg = I.small_config(dtype="bf16", d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=128, d_ff=512)
    else:
        cfg = I.small_config(d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ff=64)
    ol, gl = both(cfg)
    B, cap = MAX_SEQS, 24
    hkv, hd = cfg["n_kv_heads"], cfg["head_dim"]
    rng = np.random.default_rng(1)
    lens = rng.integers(0, cap - 1, B)
    lens[:4] = 0
    oc, gc = O.KVCache(ol, B, cap), gl.cache(B, cap)
    k, v = I.kv_fill(hkv, cap, hd, seed=2, dtype=dtype)
    kd, vd = to_dev(k, dtype), to_dev(v, dtype)
    for i, n in enumerate(lens):
        n = int(n)
        oc.set(i, k[:, :n], v[:, :n])
        if n > 0:
            pd.pd_kv_cache_set(gc, i, kd[:, :n].contiguous(), vd[:, :n].contiguous())
    slots = list(rng.permutation(B))
    xn = I.hidden(B, cfg["d_model"], seed=3, dtype=dtype)
    ref = O.decode_step(ol, xn, slots, oc)
    got = gl.decode(xn, slots, gc)
    assert relmax(got, ref) <= TOL[dtype]
    assert max(relmax(got[i], ref[i]) for i in range(0, B, 37)) <= 2 * TOL[dtype]
    x1 = to_dev(I.hidden(B + 1, cfg["d_model"], seed=4, dtype=dtype), dtype)
    with pytest.raises(pd.PdError) as e:
        pd.pd_decode_step(gl.h, x1, list(range(B)) + [0], gc, torch.empty_like(x1))
    assert e.value.status == pd.PD_ERR_INVALID_ARG
    gl.close()


def test_prefill_with_the_largest_sequence_count():
    """4096 sequences of 0 .. 3 tokens in one prefill call, each kept in its own cache slot."""
    cfg = I.small_config(dtype="bf16", d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=128, d_ff=512)
    ol, gl = both(cfg)
    n = MAX_SEQS
    rng = np.random.default_rng(5)
    L = rng.integers(0, 4, n)
    cu = np.concatenate([[0], np.cumsum(L)]).astype(np.int32)
    x = I.hidden(int(cu[-1]), cfg["d_model"], seed=6, dtype="bf16")
    slots = list(rng.permutation(n))
    oc, gc = O.KVCache(ol, n, 8), gl.cache(n, 8)
    ref = O.prefill(ol, x, cu, cache=oc, slots=slots)
    got = gl.prefill(x, cu, cache=gc, slots=slots)
    assert relmax(got, ref) <= TOL["bf16"]
    for s in (0, 1, 1000, n - 1):
        assert pd.pd_kv_cache_len(gc, slots[s]) == int(L[s])
    xn = I.hidden(16, cfg["d_model"], seed=7, dtype="bf16")
    pick = [slots[i] for i in range(16)]
    assert relmax(gl.decode(xn, pick, gc), O.decode_step(ol, xn, pick, oc)) <= TOL["bf16"]
    gl.close()


@pytest.mark.parametrize("B,mode", [(128, "equal"), (129, "equal"), (150, "equal"), (191, "equal"), (192, "equal"),
                                    (140, "ragged"), (200, "ragged"), (9, "one_long")])
def test_decode_attention_work_splits_around_their_switch_points(B, mode):
    """8 kv heads: 128 sequences are 1024 workers (one workgroup per CU); one more sequence makes the
    split finer; ragged lengths cap the chunk size; one long sequence among short ones is cut alone."""
    cfg = I.small_config(dtype="bf16", d_model=256, n_q_heads=8, n_kv_heads=8, head_dim=128, d_ff=256)
    ol, gl = both(cfg)
    rng = np.random.default_rng(B)
    cap = 1100
    if mode == "equal":
        lens = np.full(B, 700)
    elif mode == "ragged":
        lens = np.minimum(cap - 2, rng.lognormal(5.5, 0.8, B).astype(int))
    else:
        lens = np.full(B, 5)
        lens[3] = cap - 2
    oc, gc = O.KVCache(ol, B, cap), gl.cache(B, cap)
    k, v = I.kv_fill(8, cap, 128, seed=8, dtype="bf16")
    kd, vd = to_dev(k, "bf16"), to_dev(v, "bf16")
    for i, n in enumerate(lens):
        n = int(n)
        oc.set(i, k[:, :n], v[:, :n])
        pd.pd_kv_cache_set(gc, i, kd[:, :n].contiguous(), vd[:, :n].contiguous())
    slots = list(range(B))
    xn = I.hidden(B, cfg["d_model"], seed=9, dtype="bf16")
    ref = O.decode_step(ol, xn, slots, oc)
    got = gl.decode(xn, slots, gc)
    assert relmax(got, ref) <= TOL["bf16"]
    assert max(relmax(got[i], ref[i]) for i in range(B)) <= 2 * TOL["bf16"]
    gl.close()
