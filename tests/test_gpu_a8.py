"""GPU parity of 8-bit activations (pd_layer_create_w8a8, pd_quantize_rows_e4m3, pd_gemm_e4m3): the row
quantiser is compared byte for byte with the oracle's, the product on given codes to the bf16 rounding
of its output, and the layer against the oracle, each oracle call being told whether the library's
call quantises (the library's rule: calls of more than 256 rows).  In the layer the two sides do
not quantise the same numbers: what they quantise (attention output, normalised hidden state, SwiGLU
output) already differs by the bf16 bound, a code has 3 mantissa bits, so a few per cent of the
activations land one code apart; TOL_A8 is the bound derived for that."""
import numpy as np
import pytest
import torch

import paper_2603_04716_amd as pd
import pd_inputs as I
from oracle import layer as O
from gpu_util import GpuLayer, TOL, relmax, to_dev

pytestmark = pytest.mark.gpu

# activations differing by up to 2^-8 relative against a code spacing of 2^-3 .. 2^-4: a fraction
# p ~ 2^-8 / 2^-3.5 * 2 ~ 0.09 of them gets the neighbouring code (an error of one spacing, ~0.09 of the
# element), i.e. sqrt(p) * 0.09 ~ 0.027 of a projection's output, through two projections in a row
# (attention output -> h -> FFN) and relative to the largest output: 6e-2.
TOL_A8 = 6e-2
# The library's rule (pd.h, pd_layer_create_w8a8): a call of more than this many rows quantises the
# inputs of its projections.  The oracle knows no such rule; every oracle call below is told whether
# its call quantises.
A8_ROWS = 256


def small(hq=4, hkv=2, d=256, F=512, **kw):
    return I.small_config(dtype="bf16", d_model=d, n_q_heads=hq, n_kv_heads=hkv, head_dim=128, d_ff=F, **kw)


def gpu_quantise(x_bf16_as_f32):
    xd = to_dev(x_bf16_as_f32, "bf16")
    codes = torch.empty(xd.shape, dtype=torch.uint8, device="cuda")
    scales = torch.empty(xd.shape[0], dtype=torch.float32, device="cuda")
    pd.pd_quantize_rows_e4m3(xd, codes, scales)
    torch.cuda.synchronize()
    return codes.cpu().numpy(), scales.cpu().numpy()


def test_row_quantiser_every_bf16_value_bit_exact():
    """All 65280 finite bf16 bit patterns as one long row per scale setter: the codes are decided by
    the hardware conversion after an exact scaling, the oracle's by its own encoder."""
    bits = np.arange(65536, dtype=np.uint32)
    finite = (bits & 0x7f80) != 0x7f80
    vals = (bits[finite] << 16).astype(np.uint32).view(np.float32)
    n = (len(vals) + 7) // 8 * 8
    row = np.zeros(n, np.float32)
    row[:len(vals)] = vals
    # the row maximum is the largest finite bf16: scale 2^119; then rows whose maximum is capped so
    # that the small values are not all flushed: keep |v| <= c and zero the rest
    rows = [row]
    for c in (448.0, 1.0, 3.0e-3, 2.0 ** -100):
        rows.append(np.where(np.abs(row) <= c, row, 0.0).astype(np.float32))
    x = np.stack(rows)
    codes, scales = gpu_quantise(x)
    xq, s_ref, c_ref = O.act_quantise_rows(x)
    assert np.array_equal(scales, s_ref)
    assert np.array_equal(codes, c_ref)


def test_row_quantiser_random_rows_ties_and_boundaries():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((300, 1024)) * np.exp(rng.uniform(-10, 6, (300, 1)))).astype(np.float32)
    x = torch.from_numpy(x).to(torch.bfloat16).float().numpy()
    x[0] = 0.0                                        # zero row
    x[1, :] = 0.0
    x[1, 7] = 448.0                                   # exactly the largest code, scale 1
    x[2, :] = 0.0
    x[2, 3] = 480.0                                   # above 448: next scale, 240 is exact
    x[3, :64] = np.arange(64) * 2.0 ** -10            # subnormal codes and ties (scale 1 by the next line)
    x[3, 64] = 300.0
    x[4, :16] = np.array([17, 19, 21, 23, 25, 27, 29, 31, 34, 38, 42, 46, 50, 54, 58, 62]) * 1.0   # ties at 4 bits
    x[4, 16] = 448.0
    x[5, 0] = np.inf                                  # infinity: scale 1, saturates
    codes, scales = gpu_quantise(x)
    xq, s_ref, c_ref = O.act_quantise_rows(x)
    assert np.array_equal(scales, s_ref)
    assert np.array_equal(codes, c_ref)
    assert scales[0] == 1 and scales[1] == 1 and scales[2] == 2 and scales[5] == 1 and codes[5, 0] == 0x7E


def test_quantiser_argument_errors():
    x = torch.zeros(4, 12, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(pd.PdError) as e:
        pd.pd_quantize_rows_e4m3(x, torch.empty(4, 12, dtype=torch.uint8, device="cuda"),
                                 torch.empty(4, dtype=torch.float32, device="cuda"))
    assert e.value.status == pd.PD_ERR_INVALID_ARG


@pytest.mark.parametrize("M,N,K", [(1, 16, 128), (257, 512, 256), (300, 528, 1152), (300, 512, 8192), (448, 4096, 14336),
                                   (1100, 1024, 4096), (2048, 6144, 4096)])
def test_gemm_e4m3_same_codes_on_both_sides(M, N, K):
    """The matrix-core product on given codes and scales against the oracle on the same bytes: only
    the fp32 summation order and the one rounding to bf16 differ (2^-8 of the largest output).  Sizes
    on both sides of 512 rows (decode-style narrow tiles with K split over workgroups below, large
    tiles above), one row, ragged row and column tiles."""
    rng = np.random.default_rng(M + N)
    a = rng.integers(0, 256, (M, K), dtype=np.uint8)
    b = rng.integers(0, 256, (N, K), dtype=np.uint8)
    a[(a & 0x7f) == 0x7f] = 0x30
    b[(b & 0x7f) == 0x7f] = 0xB1
    a[rng.random((M, K)) < 0.5] &= 0xBF               # thin out the large exponents: a bell-like spread
    b[rng.random((N, K)) < 0.5] &= 0xBF
    sa = (2.0 ** rng.integers(-8, 2, M)).astype(np.float32)
    sb = (2.0 ** rng.integers(-10, -2, N)).astype(np.float32)
    out = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    pd.pd_gemm_e4m3(torch.from_numpy(a).cuda(), torch.from_numpy(sa).cuda(), torch.from_numpy(b).cuda(),
                    torch.from_numpy(sb).cuda(), out)
    got = out.float().cpu().numpy()
    if M * N <= 400000:
        ref = O.gemm_e4m3(a, sa, b, sb)
        assert relmax(got, ref) <= 2.0 ** -8
        # row by row as well: a wrong scale on a small row would hide behind the largest one
        assert max(relmax(got[m], ref[m]) for m in range(M)) <= 2.0 ** -7
    else:
        rows = rng.choice(M, 24, replace=False)
        ref = O.gemm_e4m3(a[rows], sa[rows], b, sb)
        assert max(relmax(got[r], ref[j]) for j, r in enumerate(rows)) <= 2.0 ** -7


def test_gemm_e4m3_argument_errors():
    z8 = lambda *s: torch.zeros(*s, dtype=torch.uint8, device="cuda")
    zf = lambda n: torch.ones(n, dtype=torch.float32, device="cuda")
    for M, N, K in ((4, 24, 128), (4, 32, 192), (4, 32, 64)):
        with pytest.raises(pd.PdError) as e:
            pd.pd_gemm_e4m3(z8(M, K), zf(M), z8(N, K), zf(N), torch.empty(M, N, dtype=torch.bfloat16, device="cuda"))
        assert e.value.status == pd.PD_ERR_SHAPE


def both(cfg, std=0.05, seed=None):
    w = I.layer_weights(cfg, seed=seed, std=std)
    return O.Layer(cfg, O.quantise_layer_weights(w)), GpuLayer(cfg, w, a8=True)


@pytest.mark.parametrize("T,cu", [(257, [0, 257]), (300, [0, 130, 131, 300]), (700, [0, 5, 400, 700]), (1100, [0, 1100])])
@pytest.mark.parametrize("d,F,hq,hkv", [(256, 512, 4, 2), (512, 1152, 4, 1)])
def test_prefill_with_8bit_activations(T, cu, d, F, hq, hkv):
    """More than 256 rows: every projection multiplies codes by codes (plain, residual and SwiGLU
    epilogues, K split over workgroups at these sizes, ragged last row tile); the cache it writes
    is then read by a decode step, which has few rows and keeps bf16 activations."""
    cfg = small(hq, hkv, d, F)
    ol, gl = both(cfg, std=0.04, seed=T)
    cu = np.array(cu, np.int32)
    n = len(cu) - 1
    x = I.hidden(T, d, seed=8, dtype="bf16")
    oc, gc = O.KVCache(ol, n, 1104), gl.cache(n, 1104)
    ref = O.prefill(ol, x, cu, cache=oc, slots=list(range(n)), act8=T > A8_ROWS)
    got = gl.prefill(x, cu, cache=gc, slots=list(range(n)))
    assert relmax(got, ref) <= TOL_A8
    rms = float(np.sqrt(np.mean((got - ref) ** 2)) / np.sqrt(np.mean(ref ** 2)))
    assert rms <= TOL_A8 / 3
    xn = I.hidden(n, d, seed=81, dtype="bf16")
    ref = O.decode_step(ol, xn, list(range(n)), oc, act8=n > A8_ROWS)
    got = gl.decode(xn, list(range(n)), gc)
    assert relmax(got, ref) <= TOL["bf16"]         # keys and values come from a projection of exact inputs
    gl.close()


def test_decode_step_of_more_than_256_rows_quantises_too():
    """The rule counts the rows of the call, whichever entry point: a decode batch of 300."""
    cfg = small()
    ol, gl = both(cfg, std=0.04, seed=3)
    B = 300
    rng = np.random.default_rng(9)
    lens = rng.integers(1, 40, B)
    oc, gc = O.KVCache(ol, B, 48), gl.cache(B, 48)
    for i, n in enumerate(lens):
        k, v = I.kv_fill(2, int(n), 128, seed=6000 + i, dtype="bf16")
        oc.set(i, k, v)
        pd.pd_kv_cache_set(gc, i, to_dev(k, "bf16"), to_dev(v, "bf16"))
    xn = I.hidden(B, cfg["d_model"], seed=53, dtype="bf16")
    ref = O.decode_step(ol, xn, list(range(B)), oc, act8=B > A8_ROWS)
    got = gl.decode(xn, list(range(B)), gc)
    assert relmax(got, ref) <= TOL_A8
    gl.close()


@pytest.mark.parametrize("fp8_cache", [False, True])
def test_chunked_prefill_counts_the_rows_of_each_call(fp8_cache):
    """A 40-token first chunk (bf16 activations), then one of 300 tokens against that prefix (8-bit
    activations), then a decode step; with the bf16 and with the 8-bit cache."""
    cfg = small()
    ol, gl = both(cfg, std=0.04, seed=11)
    scales = (0.5, 0.125) if fp8_cache else None
    oc, gc = O.KVCache(ol, 2, 352, fp8_scales=scales), gl.cache(2, 352, fp8_scales=scales)
    d = cfg["d_model"]
    for step, (n0, n1) in enumerate(((25, 15), (180, 120))):
        cu = np.array([0, n0, n0 + n1], np.int32)
        x = I.hidden(n0 + n1, d, seed=70 + step, dtype="bf16")
        ref = O.prefill_chunk(ol, x, cu, [0, 1], oc, act8=n0 + n1 > A8_ROWS)
        got = gl.prefill_chunk(x, cu, [0, 1], gc)
        assert relmax(got, ref) <= (TOL["bf16"] if step == 0 else TOL_A8), step
    xn = I.hidden(2, d, seed=75, dtype="bf16")
    ref = O.decode_step(ol, xn, [0, 1], oc, act8=2 > A8_ROWS)
    got = gl.decode(xn, [0, 1], gc)
    assert relmax(got, ref) <= TOL_A8       # the cached keys and values of the second chunk carry its code differences
    gl.close()


def test_calls_of_up_to_256_rows_are_those_of_the_8bit_weight_layer():
    cfg = small()
    w = I.layer_weights(cfg, std=0.05)
    ga, gw = GpuLayer(cfg, w, a8=True), GpuLayer(cfg, w, w8=True)
    cu = np.array([0, 100, 256], np.int32)
    x = I.hidden(256, cfg["d_model"], seed=3, dtype="bf16")
    assert np.array_equal(ga.prefill(x, cu), gw.prefill(x, cu))
    cu = np.array([0, 100, 257], np.int32)
    x = I.hidden(257, cfg["d_model"], seed=3, dtype="bf16")
    assert not np.array_equal(ga.prefill(x, cu), gw.prefill(x, cu))
    ga.close()
    gw.close()


@pytest.mark.parametrize("T,given_logits", [(300, True), (700, False)])
def test_moe_prefill_with_8bit_activations(T, given_logits):
    """Grouped products on codes: the gathered operand is quantised once per token where it lies, its
    scale follows the gather, every expert has its own weight scales; expert choices are compared
    as integers."""
    cfg = small(4, 2, 256, 384, n_experts=4, top_k=2)
    w = I.layer_weights(cfg, std=0.04, with_router=True, seed=T)
    ol, gl = O.Layer(cfg, O.quantise_layer_weights(w)), GpuLayer(cfg, w, a8=True)
    cu = np.array([0, 120, T], np.int32)
    x = I.hidden(T, cfg["d_model"], seed=18, dtype="bf16")
    rl = I.router_logits(T, 4, seed=19) if given_logits else None
    ref, eref = O.prefill(ol, x, cu, router_logits=rl, return_experts=True, act8=T > A8_ROWS)
    got = gl.prefill(x, cu, router_logits=rl)
    if given_logits:
        assert np.array_equal(np.sort(gl.experts(T), axis=1), np.sort(eref, axis=1))
        assert relmax(got, ref) <= TOL_A8
    else:
        # own router logits come from different roundings: compare the tokens that chose the same experts
        same = np.all(np.sort(gl.experts(T), axis=1) == np.sort(eref, axis=1), axis=1)
        assert same.mean() > 0.97
        assert relmax(got[same], ref[same]) <= TOL_A8
    gl.close()


def test_moe_with_8bit_activations_and_empty_experts():
    """All tokens on experts 1 and 2 (the others get no rows), one expert with fewer rows than a row tile."""
    cfg = small(4, 2, 256, 384, n_experts=4, top_k=2)
    w = I.layer_weights(cfg, std=0.04, with_router=True, seed=5)
    ol, gl = O.Layer(cfg, O.quantise_layer_weights(w)), GpuLayer(cfg, w, a8=True)
    T = 400
    cu = np.array([0, T], np.int32)
    x = I.hidden(T, cfg["d_model"], seed=28, dtype="bf16")
    rl = np.full((T, 4), -20.0, np.float32)
    rl[:, 1], rl[:, 2] = 3.0, 2.0
    rl[:7, 3] = 5.0                                 # seven tokens also pick expert 3 (instead of 2)
    ref, eref = O.prefill(ol, x, cu, router_logits=rl, return_experts=True, act8=T > A8_ROWS)
    got = gl.prefill(x, cu, router_logits=rl)
    assert np.array_equal(gl.experts(T), eref)
    assert relmax(got, ref) <= TOL_A8
    gl.close()


def test_w8a8_needs_dimensions_in_multiples_of_128():
    for cfg in (small(d=320, F=512), small(F=576)):
        w = I.layer_weights(cfg, with_router=cfg.get("n_experts", 0) > 0)
        dev = {k: to_dev(v, cfg["dtype"]) for k, v in w.items()}
        with pytest.raises(pd.PdError) as e:
            pd.pd_layer_create(cfg, dev, w8=True, a8=True)
        assert e.value.status == pd.PD_ERR_DTYPE


def test_llama8b_shape_prefill_sampled_rows():
    """8B-shaped layer, 2 x 1024 tokens; the oracle recomputes sampled rows of the same call."""
    cfg = I.CONFIGS["llama8b"]
    w = I.layer_weights(cfg)
    ol, gl = O.Layer(cfg, O.quantise_layer_weights(w)), GpuLayer(cfg, w, a8=True)
    T = 2048
    cu = np.array([0, 1024, 2048], np.int32)
    x = I.hidden(T, cfg["d_model"], seed=10, dtype="bf16")
    got = gl.prefill(x, cu)
    rows = np.array([0, 511, 1023, 1024, 2047], np.int32)
    ref = O.prefill(ol, x, cu, rows=rows, act8=T > A8_ROWS)
    for j, r in enumerate(rows):
        assert relmax(got[r], ref[j]) <= TOL_A8, r
    gl.close()
