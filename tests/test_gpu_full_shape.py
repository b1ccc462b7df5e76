"""GPU parity at the benchmark's full shapes, in the launch configuration bench.py times.
The oracle cannot evaluate 8192 x 8B-shaped rows in seconds, so it produces sampled output rows
(keys and values of all earlier tokens of the sampled sequences are still computed in full) and
those rows are compared element by element.  Bound: max|gpu - ref| / max|ref| <= 2e-2 (bf16)."""
import numpy as np
import pytest
import torch

import paper_2603_04716_amd as pd
import pd_inputs as I
from oracle import layer as O
from paper_2603_04716_amd import harness as H
from gpu_util import TOL, relmax, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def llama():
    cfg = I.CONFIGS["llama8b"]
    w = I.layer_weights(cfg)
    layer = H.Layer(cfg, w)
    yield cfg, w, layer
    layer.close()


def tile_rows(T, l_in, seed, tile=256):
    """One seeded row inside every `tile`-row band of the call (the row tiles of the large GEMM kernels
    and two query blocks of the attention kernel each), plus the first and the last row of every
    sequence: a mapping error confined to one band of the tile grid, or to one sequence, shows."""
    rng = np.random.default_rng(seed)
    rows = {int(t0 + rng.integers(0, min(tile, T - t0))) for t0 in range(0, T, tile)}
    for s0 in range(0, T, l_in):
        rows |= {s0, min(s0 + l_in, T) - 1}
    return sorted(rows)


@pytest.mark.parametrize("l_in", [2048, 4096, 1024])
def test_llama8b_prefill_8192_tokens_sampled_rows(llama, l_in):
    cfg, w, layer = llama
    T = 8192
    n_seq = T // l_in
    x = I.hidden(T, cfg["d_model"], seed=10, dtype="bf16")
    cu = I.uniform_cu_seqlens(n_seq, l_in)
    xd = H._dev(x, "bf16")
    out = torch.empty_like(xd)
    pd.pd_prefill(layer.h, xd, cu, out)
    torch.cuda.synchronize()
    got = to_np(out)
    assert np.isfinite(got).all()
    rows = tile_rows(T, l_in, seed=l_in)                # every 256-row tile, every sequence's ends
    ref = O.prefill(O.Layer(cfg, w), x, cu, rows=rows)
    assert relmax(got[rows], ref) <= TOL["bf16"]
    for i, r in enumerate(rows):
        assert relmax(got[r], ref[i]) <= 2 * TOL["bf16"], r
    # properties that hold at any size: sequences with identical inputs give identical outputs
    x2 = x.copy()
    x2[l_in:2 * l_in] = x[:l_in]
    pd.pd_prefill(layer.h, H._dev(x2, "bf16"), cu, out)
    torch.cuda.synchronize()
    got2 = to_np(out)
    assert np.array_equal(got2[l_in:2 * l_in], got2[:l_in])
    assert np.array_equal(got2[:l_in], got[:l_in])


@pytest.mark.parametrize("B", [256, 8])
def test_llama8b_decode_kv2048_sampled_rows_graph_replay(llama, B):
    cfg, w, layer = llama
    S = 2048
    hkv, hd = cfg["n_kv_heads"], cfg["head_dim"]
    cache = layer.new_cache(B, S + 8)
    sets = [I.kv_fill(hkv, S, hd, seed=40 + j, dtype="bf16") for j in range(4)]
    dev_sets = [(H._dev(k, "bf16"), H._dev(v, "bf16")) for k, v in sets]
    for s in range(B):
        pd.pd_kv_cache_set(cache, s, *dev_sets[s % 4])
    x = I.hidden(B, cfg["d_model"], seed=41, dtype="bf16")
    run = layer.make_decode_step(cache, H._dev(x, "bf16"), [S] * B, use_graph=True)
    run()
    run()                                    # replays must rewind and reproduce
    torch.cuda.synchronize()
    got = to_np(run.out)
    assert np.isfinite(got).all()
    # one seeded row in every band of 32 rows (two 16-row matrix-core blocks each) and both ends
    rng = np.random.default_rng(B)
    sample = sorted({0, B - 1} | {int(b0 + rng.integers(0, min(32, B - b0))) for b0 in range(0, B, 32)})
    ol = O.Layer(cfg, w)
    oc = O.KVCache(ol, len(sample), S + 8)
    for i, b in enumerate(sample):
        oc.set(i, *sets[b % 4])
    ref = O.decode_step(ol, x[sample], list(range(len(sample))), oc)
    assert relmax(got[sample], ref) <= TOL["bf16"]
    for i, b in enumerate(sample):
        assert relmax(got[b], ref[i]) <= 2 * TOL["bf16"], b
    # the appended key/value of a sampled slot equal the oracle's
    n = S + 1
    k = torch.empty((hkv, n, hd), dtype=torch.bfloat16, device="cuda")
    v = torch.empty_like(k)
    pd.pd_kv_cache_get(cache, sample[-1], k, v)
    torch.cuda.synchronize()
    assert relmax(to_np(k)[:, S], oc.k[len(sample) - 1, :, S]) <= TOL["bf16"]
    assert relmax(to_np(v)[:, S], oc.v[len(sample) - 1, :, S]) <= TOL["bf16"]
    layer.free_cache(cache)


def test_llama8b_decode_ragged_long_context_sampled_rows(llama):
    """Ragged KV lengths (log-normal prompt + partial generation, capacity 8192) at batch 32."""
    cfg, w, layer = llama
    B, cap = 32, 8192
    hkv, hd = cfg["n_kv_heads"], cfg["head_dim"]
    lens = I.ragged_kv_lengths(B, cap - 1, seed=2)
    lens[5] = cap - 1                                   # one sequence at full capacity
    cache = layer.new_cache(B, cap)
    k, v = I.kv_fill(hkv, cap - 1, hd, seed=50, dtype="bf16")
    kd, vd = H._dev(k, "bf16"), H._dev(v, "bf16")
    layer.fill_cache(cache, lens, kd, vd)
    x = I.hidden(B, cfg["d_model"], seed=51, dtype="bf16")
    run = layer.make_decode_step(cache, H._dev(x, "bf16"), lens, use_graph=True)
    run()
    torch.cuda.synchronize()
    got = to_np(run.out)
    sample = [0, 5, int(np.argmin(lens))]
    ol = O.Layer(cfg, w)
    oc = O.KVCache(ol, len(sample), cap)
    for i, b in enumerate(sample):
        oc.set(i, k[:, :lens[b]], v[:, :lens[b]])
    ref = O.decode_step(ol, x[sample], list(range(len(sample))), oc)
    for i, b in enumerate(sample):
        assert relmax(got[b], ref[i]) <= TOL["bf16"], (b, int(lens[b]))
    layer.free_cache(cache)


@pytest.mark.parametrize("ragged", [False, True])
def test_llama8b_decode_kv16384_128_slots_sampled_rows(llama, ragged):
    """The long-context configuration at its largest size: 128 slots of capacity 16384, so the cache
    planes of the upper slots lie beyond 4 GiB (128 x 8 x 16384 x 128 x 2 B = 4.3 GB each for keys
    and values).  Uniform lengths (every slot full but for the new token) and one ragged batch
    (log-normal prompt + partial generation, with a full slot and the shortest slot sampled)."""
    cfg, w, layer = llama
    B, cap = 128, 16384
    hkv, hd = cfg["n_kv_heads"], cfg["head_dim"]
    if ragged:
        lens = I.ragged_kv_lengths(B, cap - 1, seed=3)
        lens[127] = cap - 1
        lens[1] = 17
    else:
        lens = np.full(B, cap - 1, np.int32)
    cache = layer.new_cache(B, cap)
    sets = [I.kv_fill(hkv, cap - 1, hd, seed=70 + j, dtype="bf16") for j in range(2)]
    dev_sets = [(H._dev(k, "bf16"), H._dev(v, "bf16")) for k, v in sets]
    for s in range(B):
        kd, vd = dev_sets[s % 2]
        pd.pd_kv_cache_set(cache, s, kd[:, :int(lens[s])].contiguous(), vd[:, :int(lens[s])].contiguous())
    x = I.hidden(B, cfg["d_model"], seed=71, dtype="bf16")
    run = layer.make_decode_step(cache, H._dev(x, "bf16"), lens, use_graph=True)
    run()
    run()
    torch.cuda.synchronize()
    got = to_np(run.out)
    assert np.isfinite(got).all()
    sample = sorted({0, 1, 62, 63, 64, 126, 127, int(np.argmax(lens)), int(np.argmin(lens))})
    ol = O.Layer(cfg, w)
    oc = O.KVCache(ol, len(sample), cap)
    for i, b in enumerate(sample):
        k, v = sets[b % 2]
        oc.set(i, k[:, :lens[b]], v[:, :lens[b]])
    ref = O.decode_step(ol, x[sample], list(range(len(sample))), oc)
    for i, b in enumerate(sample):
        assert relmax(got[b], ref[i]) <= TOL["bf16"], (b, int(lens[b]))
    # the appended key / value of the last slot (plane offset beyond 4 GiB) equal the oracle's
    n = int(lens[127]) + 1
    k = torch.empty((hkv, n, hd), dtype=torch.bfloat16, device="cuda")
    v = torch.empty_like(k)
    pd.pd_kv_cache_get(cache, 127, k, v)
    torch.cuda.synchronize()
    j = sample.index(127)
    assert relmax(to_np(k)[:, n - 1], oc.k[j, :, n - 1]) <= TOL["bf16"]
    assert relmax(to_np(v)[:, n - 1], oc.v[j, :, n - 1]) <= TOL["bf16"]
    assert np.array_equal(to_np(k)[:, :n - 1], sets[127 % 2][0][:, :n - 1])
    layer.free_cache(cache)


def test_moe_8_experts_full_shape_sampled_rows():
    cfg = I.CONFIGS["moe"]
    w = I.layer_weights(cfg)
    layer = H.Layer(cfg, w)
    T, l_in = 8192, 2048
    x = I.hidden(T, cfg["d_model"], seed=60, dtype="bf16")
    r = I.router_logits(T, cfg["n_experts"], seed=61)
    cu = I.uniform_cu_seqlens(T // l_in, l_in)
    xd, rd = H._dev(x, "bf16"), torch.from_numpy(r).cuda()
    out = torch.empty_like(xd)
    pd.pd_prefill(layer.h, xd, cu, out, router_logits=rd)
    torch.cuda.synchronize()
    got = to_np(out)
    e = torch.empty((T, 2), dtype=torch.int32, device="cuda")
    pd.pd_last_expert_choice(layer.h, T, e)
    torch.cuda.synchronize()
    rows = tile_rows(T, l_in, seed=5, tile=512)         # 16 bands + the ends of the four sequences
    ol = O.Layer(cfg, w)
    ref, eref = O.prefill(ol, x, cu, router_logits=r, rows=rows, return_experts=True)
    assert np.array_equal(e.cpu().numpy()[rows], eref)
    # every token's experts: the two largest logits (no ties in continuous draws)
    assert np.array_equal(np.sort(e.cpu().numpy(), 1), np.sort(np.argsort(-r, 1, kind="stable")[:, :2], 1))
    assert relmax(got[rows], ref) <= TOL["bf16"]
    for i, r_ in enumerate(rows):
        assert relmax(got[r_], ref[i]) <= 2 * TOL["bf16"], r_
    # decode step over a filled cache, batch 16
    B, S = 16, 512
    cache = layer.new_cache(B, S + 8)
    k, v = I.kv_fill(cfg["n_kv_heads"], S, cfg["head_dim"], seed=62, dtype="bf16")
    layer.fill_cache(cache, [S] * B, H._dev(k, "bf16"), H._dev(v, "bf16"))
    xn = I.hidden(B, cfg["d_model"], seed=63, dtype="bf16")
    rn = I.router_logits(B, cfg["n_experts"], seed=64)
    run = layer.make_decode_step(cache, H._dev(xn, "bf16"), [S] * B, router_logits=torch.from_numpy(rn).cuda(),
                                 use_graph=True)
    run()
    torch.cuda.synchronize()
    sample = [0, 9]
    oc = O.KVCache(ol, 2, S + 8)
    for i in range(2):
        oc.set(i, k, v)
    refd = O.decode_step(ol, xn[sample], [0, 1], oc, router_logits=rn[sample])
    assert relmax(to_np(run.out)[sample], refd) <= TOL["bf16"]
    layer.close()


def test_llama8b_8bit_layer_at_the_bench_shapes_sampled_rows():
    """The 8-bit section of bench.py: 8-bit weights and (above 256 rows) activations, prefill of 4 x 2048
    tokens, then a decode step of batch 448 over an 8-bit cache at KV 2048 through a replayed graph;
    the oracle recomputes sampled rows, told that these calls quantise.  Bounds: those of the 8-bit-activation
    layer (6e-2 of the largest output)."""
    tol = 6e-2
    cfg = I.CONFIGS["llama8b"]
    w = I.layer_weights(cfg)
    layer = H.Layer(cfg, w, a8=True)
    ol = O.Layer(cfg, O.quantise_layer_weights(w))
    T, l_in = 8192, 2048
    x = I.hidden(T, cfg["d_model"], seed=10, dtype="bf16")
    cu = I.uniform_cu_seqlens(T // l_in, l_in)
    xd = H._dev(x, "bf16")
    out = torch.empty_like(xd)
    pd.pd_prefill(layer.h, xd, cu, out)
    torch.cuda.synchronize()
    got = to_np(out)
    assert np.isfinite(got).all()
    rows = tile_rows(T, l_in, seed=6, tile=512)
    ref = O.prefill(ol, x, cu, rows=rows, act8=True)    # 8192 rows: the library's call quantises
    for i, r in enumerate(rows):
        assert relmax(got[r], ref[i]) <= tol, r
    # decode: batch 448 (8-bit activations too), 8-bit cache
    B, S = 448, 2048
    scales = (0.5, 0.125)
    hkv, hd = cfg["n_kv_heads"], cfg["head_dim"]
    cache = layer.new_cache(B, S + 8, fp8_scales=scales)
    sets = [I.kv_fill(hkv, S, hd, seed=40 + j, dtype="bf16") for j in range(4)]
    dev_sets = [(H._dev(k, "bf16"), H._dev(v, "bf16")) for k, v in sets]
    for s in range(B):
        pd.pd_kv_cache_set(cache, s, *dev_sets[s % 4])
    xb = I.hidden(B, cfg["d_model"], seed=41, dtype="bf16")
    run = layer.make_decode_step(cache, H._dev(xb, "bf16"), [S] * B, use_graph=True)
    run()
    run()
    torch.cuda.synchronize()
    gotd = to_np(run.out)
    rows = sorted({0, 255, 256, 447} | {int(r_) for r_ in np.random.default_rng(7).integers(0, B, 12)})
    # a call of 448 rows quantises in the library; rows are independent of each other, so the oracle
    # evaluates the sampled rows alone and is told that the call quantises
    ocp = O.KVCache(ol, len(rows), S + 8, fp8_scales=scales)
    for j, r_ in enumerate(rows):
        ocp.set(j, *sets[r_ % 4])
    refd = O.decode_step(ol, xb[rows], list(range(len(rows))), ocp, act8=True)
    for j, r in enumerate(rows):
        assert relmax(gotd[r], refd[j]) <= tol, r
    layer.close()
