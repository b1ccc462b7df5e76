"""GPU parity on seeded random layer shapes and call sequences: for each drawn configuration
(dtype, width, heads, GQA group, head size, FFN width, dense or mixture of experts) a random
script of prefill, chunked prefill and decode calls with ragged lengths runs on both sides, and
every call's output is compared element by element.  The shapes deliberately mix those that take
the matrix-core kernels (bf16, head_dim 128, widths that are multiples of 64) with those that fall
back to the generic kernels, so the dispatch boundaries are crossed in both directions."""
import numpy as np
import pytest

import pd_inputs as I
import paper_2603_04716_amd as pd
from oracle import layer as O
from gpu_util import GpuLayer, TOL, relmax

pytestmark = pytest.mark.gpu


def draw_config(rng):
    dtype = "bf16" if rng.random() < 0.7 else "f32"
    hd = int(rng.choice([128, 128, 64, 32]))
    hkv = int(rng.choice([1, 2, 4]))
    group = int(rng.choice([1, 2, 4, 8]))
    d_model = int(rng.choice([128, 192, 256, 320]))
    d_ff = int(rng.choice([96, 128, 256, 448]))
    moe = rng.random() < 0.3
    return I.small_config(dtype=dtype, d_model=d_model, n_q_heads=hkv * group, n_kv_heads=hkv, head_dim=hd,
                          d_ff=d_ff, n_experts=4 if moe else 0, top_k=2 if moe else 0)


@pytest.mark.parametrize("seed", list(range(32)))
def test_random_shape_and_call_script(seed):
    rng = np.random.default_rng(1000 + seed)
    cfg = draw_config(rng)
    dt, tol = cfg["dtype"], TOL[cfg["dtype"]]
    w = I.layer_weights(cfg, std=0.06, with_router=False)
    ol, gl = O.Layer(cfg, w), GpuLayer(cfg, w)
    n_seq = int(rng.integers(1, 5))
    cap = 160
    oc, gc = O.KVCache(ol, n_seq, cap), gl.cache(n_seq, cap)
    slots = [int(s) for s in rng.permutation(n_seq)]
    held = [0] * n_seq
    E = cfg["n_experts"]

    def logits(rows, s):
        return I.router_logits(rows, E, seed=s) if E else None

    # first call: a prefill that fills the slots
    lens = [int(rng.integers(1, 70)) for _ in range(n_seq)]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    x = I.hidden(int(cu[-1]), cfg["d_model"], seed=2000 + seed, dtype=dt)
    rl = logits(int(cu[-1]), 3000 + seed)
    ref = O.prefill(ol, x, cu, router_logits=rl, cache=oc, slots=slots)
    got = gl.prefill(x, cu, cache=gc, slots=slots, router_logits=rl)
    assert relmax(got, ref) <= tol, ("prefill", cfg)
    held = list(lens)
    for step in range(6):
        kind = rng.choice(["decode", "chunk", "short"])
        if kind == "decode":
            xn = I.hidden(n_seq, cfg["d_model"], seed=4000 + 10 * seed + step, dtype=dt)
            rl = logits(n_seq, 5000 + 10 * seed + step)
            ref = O.decode_step(ol, xn, slots, oc, router_logits=rl)
            got = gl.decode(xn, slots, gc, router_logits=rl)
            held = [h + 1 for h in held]
        else:
            hi = 9 if kind == "short" else 40
            add = [int(rng.integers(0, hi)) for _ in range(n_seq)]
            add = [min(a, cap - h - 8) for a, h in zip(add, held)]
            if sum(add) == 0:
                add[0] = 1
            cu = np.concatenate([[0], np.cumsum(add)]).astype(np.int32)
            xn = I.hidden(int(cu[-1]), cfg["d_model"], seed=6000 + 10 * seed + step, dtype=dt)
            rl = logits(int(cu[-1]), 7000 + 10 * seed + step)
            ref = O.prefill_chunk(ol, xn, cu, slots, oc, router_logits=rl)
            got = gl.prefill_chunk(xn, cu, slots, gc, router_logits=rl)
            held = [h + a for h, a in zip(held, add)]
        assert relmax(got, ref) <= tol, (kind, step, cfg)
        for i, sl in enumerate(slots):
            assert pd.pd_kv_cache_len(gc, sl) == held[i] == int(oc.lens[sl])
    gl.close()
