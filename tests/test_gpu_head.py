"""GPU parity of the stack ends (embedding, final RMSNorm + vocabulary projection) against the CPU
oracle: embedding bit for bit, logits within the layer bounds (1e-5 fp32, 2e-2 bf16)."""
import numpy as np
import pytest
import torch

import paper_2603_04716_amd as pd
import pd_inputs as I
from oracle import layer as O
from gpu_util import TOL, relmax, to_dev, to_np

pytestmark = pytest.mark.gpu


def make_head(d, V, dtype, seed, std=0.05, max_rows=256, with_embed=True):
    hw = I.head_weights(d, V, seed=seed, dtype=dtype, std=std)
    dev = {k: to_dev(v, dtype) for k, v in hw.items()}
    h = pd.pd_head_create(d, V, 1e-6, dtype, dev["g_final"], dev["w_lm"], dev["w_embed"] if with_embed else None, max_rows)
    return hw, h


@pytest.mark.parametrize("dtype,d,V", [("f32", 96, 333), ("f32", 256, 1000), ("bf16", 100, 301),
                                       ("bf16", 256, 1040), ("bf16", 512, 4112)])
@pytest.mark.parametrize("T", [1, 5, 16, 17, 70, 200])
def test_lm_head_rows_and_shapes(dtype, d, V, T):
    """Generic kernels (fp32, odd shapes) and the matrix-core kernels (bf16, d a multiple of 64, V of
    16): skinny form up to 16 rows, tiled forms above, ragged last column tile."""
    hw, h = make_head(d, V, dtype, seed=d + V)
    x = I.hidden(T, d, seed=T, dtype=dtype)
    ref = O.lm_head(x, hw["g_final"], hw["w_lm"])
    logits = torch.empty((T, V), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")
    pd.pd_lm_head(h, to_dev(x, dtype), logits)
    torch.cuda.synchronize()
    got = to_np(logits)
    assert relmax(got, ref) <= TOL[dtype]
    assert max(relmax(got[t], ref[t]) for t in range(T)) <= 2 * TOL[dtype]
    pd.pd_head_destroy(h)


@pytest.mark.parametrize("d,V", [(256, 1040), (512, 4112)])
@pytest.mark.parametrize("T", [1, 16, 17, 64, 100, 128, 130])
def test_lm_head_with_8bit_weights(d, V, T):
    """pd_head_create_w8: the oracle is the head on the row-quantised vocabulary matrix; the codes are
    streamed up to 128 rows (skinny kernel to 16 rows, the wide one above where d is a multiple of
    512), the bf16 copy of the same weights serves the rest.  The embedding is not quantised."""
    hw = I.head_weights(d, V, seed=d + V + 1, dtype="bf16", std=0.05)
    dev = {k: to_dev(v, "bf16") for k, v in hw.items()}
    h = pd.pd_head_create(d, V, 1e-6, "bf16", dev["g_final"], dev["w_lm"], dev["w_embed"], 256, w8=True)
    x = I.hidden(T, d, seed=T + 3, dtype="bf16")
    ref = O.lm_head(x, hw["g_final"], O.quantise_rows(hw["w_lm"])[0])
    logits = torch.empty((T, V), dtype=torch.bfloat16, device="cuda")
    pd.pd_lm_head(h, to_dev(x, "bf16"), logits)
    torch.cuda.synchronize()
    got = to_np(logits)
    assert relmax(got, ref) <= TOL["bf16"]
    assert max(relmax(got[t], ref[t]) for t in range(T)) <= 2 * TOL["bf16"]
    ids = torch.tensor([0, V - 1, 7], dtype=torch.int32, device="cuda")
    out = torch.empty((3, d), dtype=torch.bfloat16, device="cuda")
    pd.pd_embed(h, ids, out)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(out), hw["w_embed"][[0, V - 1, 7]])
    pd.pd_head_destroy(h)


def test_8bit_head_needs_bf16_matrix_core_shapes():
    for dtype, d, V in (("f32", 256, 1024), ("bf16", 100, 320), ("bf16", 256, 1001)):
        hw = I.head_weights(d, V, seed=1, dtype=dtype)
        dev = {k: to_dev(v, dtype) for k, v in hw.items()}
        with pytest.raises(pd.PdError) as e:
            pd.pd_head_create(d, V, 1e-6, dtype, dev["g_final"], dev["w_lm"], None, 16, w8=True)
        assert e.value.status == pd.PD_ERR_DTYPE


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_embedding_bit_exact_and_out_of_range_ids_give_zero_rows(dtype):
    d, V = 192, 777
    hw, h = make_head(d, V, dtype, seed=9)
    ids = np.array([0, 776, 5, 5, 400, -1, 777, 123], np.int32)
    out = torch.full((len(ids), d), 7.0, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")
    pd.pd_embed(h, torch.from_numpy(ids).cuda(), out)
    torch.cuda.synchronize()
    got = to_np(out)
    ok = (ids >= 0) & (ids < V)
    assert np.array_equal(got[ok], O.embed(hw["w_embed"], ids[ok]))
    assert np.all(got[~ok] == 0.0)
    pd.pd_head_destroy(h)


def test_head_argument_errors():
    hw, h = make_head(64, 128, "bf16", seed=1, max_rows=8, with_embed=False)
    x = to_dev(I.hidden(9, 64, seed=2, dtype="bf16"), "bf16")
    logits = torch.zeros((9, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(pd.PdError) as e:
        pd.pd_lm_head(h, x, logits)                       # more rows than reserved
    assert e.value.status == pd.PD_ERR_INVALID_ARG
    with pytest.raises(pd.PdError) as e:
        pd.pd_embed(h, torch.zeros(3, dtype=torch.int32, device="cuda"), x[:3].contiguous())   # no table
    assert e.value.status == pd.PD_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert float(logits.abs().sum()) == 0.0
    pd.pd_lm_head(h, x[:0].contiguous(), logits[:0].contiguous())    # zero rows: nothing happens
    pd.pd_head_destroy(h)
    g = to_dev(hw["g_final"], "bf16")
    w = to_dev(hw["w_lm"], "bf16")
    for args, status in [((0, 128), pd.PD_ERR_SHAPE), ((64, -3), pd.PD_ERR_SHAPE)]:
        with pytest.raises(pd.PdError) as e:
            pd.pd_head_create(args[0], args[1], 1e-6, "bf16", g, w)
        assert e.value.status == status


def test_llama8b_vocabulary_head_full_rows():
    """d = 4096, 128256 vocabulary entries (the 8B model family's), batches on the skinny and on the
    tiled kernels; the oracle computes every logit of four rows."""
    d, V = 4096, 128256
    hw, h = make_head(d, V, "bf16", seed=77, std=0.02, max_rows=256, with_embed=False)
    for T in (8, 200):
        x = I.hidden(T, d, seed=500 + T, dtype="bf16")
        logits = torch.empty((T, V), dtype=torch.bfloat16, device="cuda")
        pd.pd_lm_head(h, to_dev(x, "bf16"), logits)
        torch.cuda.synchronize()
        rows = [0, T // 2, T - 1]
        ref = O.lm_head(x[rows], hw["g_final"], hw["w_lm"])
        got = to_np(logits[rows])
        for j in range(len(rows)):
            assert relmax(got[j], ref[j]) <= TOL["bf16"], (T, rows[j])
    pd.pd_head_destroy(h)
