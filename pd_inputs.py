"""Seeded synthetic inputs shared by the oracle-side and GPU-side tests and the bench.

Holds no arithmetic of the method: only random draws, the benchmark's shape
presets, and bf16 <-> fp32 value conversion of *inputs*.  Every array is made
on the host with numpy's PCG64 (`default_rng(seed)`); the same arrays are
handed to both sides.
"""
import numpy as np

# Shape presets.  "tiny" is the fp32 parity configuration, "llama8b" the bf16
# dense layer the throughput metric is quoted on, "moe" the 8-expert top-2 layer.
CONFIGS = {
    "tiny": dict(d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ff=1024, n_experts=0,
                 top_k=0, rms_eps=1e-6, rope_base=10000.0, dtype="f32", n_layers=2, seed=0),
    "llama8b": dict(d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, d_ff=14336,
                    n_experts=0, top_k=0, rms_eps=1e-6, rope_base=10000.0, dtype="bf16",
                    n_layers=32, seed=1),
    "moe": dict(d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, d_ff=14336, n_experts=8,
                top_k=2, rms_eps=1e-6, rope_base=10000.0, dtype="bf16", n_layers=32, seed=4),
}


def small_config(**over):
    """A reduced layer for parity tests; keyword overrides replace fields."""
    c = dict(d_model=128, n_q_heads=4, n_kv_heads=2, head_dim=32, d_ff=256, n_experts=0, top_k=0,
             rms_eps=1e-6, rope_base=10000.0, dtype="f32", n_layers=1, seed=7)
    c.update(over)
    return c


# ---- bf16 value conversion -----------------------------------------------------------------------

def f32_to_bf16_bits(a):
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b):
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


def round_to_bf16(a):
    """fp32 array whose values are exactly representable in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))


def _storage(a, dtype):
    a = a.astype(np.float32)
    return round_to_bf16(a) if dtype == "bf16" else a


# ---- draws ---------------------------------------------------------------------------------------

def layer_weights(cfg, seed=None, std=0.02, with_router=False):
    """fp32 arrays (bf16-representable when cfg['dtype']=='bf16'): W ~ N(0, std^2), gains = 1.

    Gains are ones: drawing an RMSNorm gain from N(0, 0.02^2) would scale the signal to ~0.
    """
    rng = np.random.default_rng(cfg["seed"] if seed is None else seed)
    d, hq, hkv, hd, f = (cfg["d_model"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"],
                         cfg["d_ff"])
    e = cfg.get("n_experts", 0)
    dt = cfg["dtype"]

    def normal(*shape):
        return _storage(rng.standard_normal(shape, dtype=np.float32) * np.float32(std), dt)

    w = {
        "g_attn": np.ones(d, np.float32),
        "w_q": normal(hq * hd, d),
        "w_k": normal(hkv * hd, d),
        "w_v": normal(hkv * hd, d),
        "w_o": normal(d, hq * hd),
        "g_ffn": np.ones(d, np.float32),
    }
    if e > 0:
        w["w_gate"] = normal(e, f, d)
        w["w_up"] = normal(e, f, d)
        w["w_down"] = normal(e, d, f)
        if with_router:
            w["w_router"] = normal(e, d)
    else:
        w["w_gate"] = normal(f, d)
        w["w_up"] = normal(f, d)
        w["w_down"] = normal(d, f)
    return w


def head_weights(d_model, vocab, seed, dtype="f32", std=0.02):
    """Final-norm gain (around 1), LM-head matrix [vocab, d_model] and embedding table (tied to the
    LM head, as in the 8B model family's smaller members) of a seeded stack end."""
    rng = np.random.default_rng(seed)
    g = _storage(1.0 + 0.1 * rng.standard_normal(d_model, dtype=np.float32), dtype)
    w = _storage(std * rng.standard_normal((vocab, d_model), dtype=np.float32), dtype)
    return {"g_final": g, "w_lm": w, "w_embed": w}


def hidden(n_rows, d, seed, dtype="f32"):
    """Hidden-state rows ~ N(0,1)."""
    rng = np.random.default_rng(seed)
    return _storage(rng.standard_normal((n_rows, d), dtype=np.float32), dtype)


def kv_fill(n_kv_heads, length, head_dim, seed, dtype="bf16"):
    """Benchmark cache contents: k, v ~ N(0,1), each [Hkv, length, hd]."""
    rng = np.random.default_rng(seed)
    k = _storage(rng.standard_normal((n_kv_heads, length, head_dim), dtype=np.float32), dtype)
    v = _storage(rng.standard_normal((n_kv_heads, length, head_dim), dtype=np.float32), dtype)
    return k, v


def router_logits(n_rows, n_experts, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((n_rows, n_experts), dtype=np.float32)


def uniform_cu_seqlens(n_seqs, length):
    return (np.arange(n_seqs + 1, dtype=np.int64) * length).astype(np.int32)


def lognormal_mean(mean, sigma, size, rng):
    """Log-normal draws whose distribution MEAN is `mean` (mu_log = ln mean - sigma^2/2)."""
    return rng.lognormal(np.log(mean) - 0.5 * sigma * sigma, sigma, size)


def ragged_kv_lengths(batch, capacity, seed, mean_in=3000.0, mean_out=500.0, sigma=0.6):
    """Per-sequence KV lengths of a decode batch caught mid-generation.

    L_in ~ LogNormal(mean 3000, sigma 0.6), L_out ~ LogNormal(mean 500, sigma 0.6),
    kv_len = L_in + floor(u * L_out), u ~ U[0,1), clipped to [1, capacity].
    """
    rng = np.random.default_rng(seed)
    l_in = lognormal_mean(mean_in, sigma, batch, rng)
    l_out = lognormal_mean(mean_out, sigma, batch, rng)
    u = rng.random(batch)
    kv = np.floor(l_in) + np.floor(u * l_out)
    return np.clip(kv, 1, capacity).astype(np.int32)


def request_lengths(n, seed, mean=2048.0, lo=64, hi=16384):
    """Prompt lengths ~ Exponential(mean), rounded and clipped to [lo, hi]."""
    rng = np.random.default_rng(seed)
    return np.clip(np.rint(rng.exponential(mean, n)), lo, hi).astype(np.int32)


def poisson_arrivals(n, rate, seed):
    """Arrival times of a Poisson process of the given rate (cumulative Exp(1/rate) gaps)."""
    rng = np.random.default_rng(seed)
    return np.cumsum(rng.exponential(1.0 / rate, n))
