/*
 * CPU oracle for one pre-norm decoder layer (prefill, chunked prefill against a cached
 * prefix, and single-token decode).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is compared against.  It shares no code, header, table or
 * helper with the HIP path and must never be called from the product path.
 *
 * The paper treats the inference engine as a black box whose prefill
 * throughput and TPOT-versus-batch curve are measured (sections "Acquire
 * prefill throughput under TTFT constraints" and "Acquire decode throughput
 * under TPOT constraints"); it defines no layer.  The layer evaluated here is
 * therefore the textbook Llama-style block at the benchmark's shapes:
 *
 *     y   = rmsnorm(x, g_attn)
 *     q,k,v = y Wq^T, y Wk^T, y Wv^T          (no bias)
 *     q,k = rope(q,k, position inside own sequence)     (rotate-half pairing)
 *     o   = causal grouped-query attention, scale 1/sqrt(head_dim)
 *     h   = x + o Wo^T
 *     y2  = rmsnorm(h, g_ffn)
 *     out = h + (silu(y2 Wg^T) * (y2 Wu^T)) Wd^T        (dense)
 *     out = h + sum_{e in top-k} w_e FFN_e(y2)           (mixture of experts)
 *
 * Tensors are stored as fp32; every dot product, mean square, softmax sum and
 * rotation angle is accumulated / evaluated in double, so results do not
 * depend on summation order at the tolerances used by the tests.
 *
 * Every function is pinned by tests/test_oracle_layer.py against an
 * independent float64 composition of library primitives, brute-force
 * attention, the decode == prefill-of-extended-sequence identity, the chunked ==
 * unchunked prefill identity and textbook invariants.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t d_model, n_q_heads, n_kv_heads, head_dim, d_ff;
    int32_t n_experts; /* 0 = dense FFN */
    int32_t top_k;
    int32_t act8;      /* != 0: this call quantises the input rows of its projections (see act_quantise_row) */
    double rms_eps, rope_base;
} orc_config;

typedef struct {
    const float *g_attn;   /* [d] */
    const float *w_q;      /* [Hq*hd, d] */
    const float *w_k;      /* [Hkv*hd, d] */
    const float *w_v;      /* [Hkv*hd, d] */
    const float *w_o;      /* [d, Hq*hd] */
    const float *g_ffn;    /* [d] */
    const float *w_gate;   /* [F, d]  (MoE: [E, F, d]) */
    const float *w_up;     /* [F, d]  (MoE: [E, F, d]) */
    const float *w_down;   /* [d, F]  (MoE: [E, d, F]) */
    const float *w_router; /* [E, d] or NULL */
} orc_weights;

/* y[i] = x[i] / sqrt(mean_j x[j]^2 + eps) * g[i]   (one row) */
/*
 * OCP 8-bit floating point, E4M3 ("fn" variant: no infinities, one NaN code per sign): 1 sign
 * bit, 4 exponent bits (bias 7), 3 mantissa bits; normal values 2^(e-7) (1 + m/8) for e >= 1,
 * subnormals m * 2^-9 for e = 0, largest finite value 448 (code 0x7E).  Encoding rounds to the
 * nearest representable value, ties to the even mantissa, and saturates at +-448 (the usual rule
 * for a quantised KV cache; NaN maps to the NaN code).
 */
double orc_fp8_e4m3_decode(uint8_t code)
{
    int sign = code >> 7, e = (code >> 3) & 15, m = code & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m, -9);
    else v = ldexp(1.0 + m / 8.0, e - 7);
    return sign ? -v : v;
}

uint8_t orc_fp8_e4m3_encode(double x)
{
    if (isnan(x)) return 0x7F;
    uint8_t sign = signbit(x) ? 0x80 : 0;
    double a = fabs(x);
    if (a >= 448.0) return sign | 0x7E;
    /* spacing of representable values around a: 2^-9 below 2^-6, else 2^(floor(log2 a) - 3) */
    int ex;
    frexp(a, &ex);                       /* a = f * 2^ex, f in [0.5, 1)  ->  floor(log2 a) = ex - 1 */
    int e_unb = ex - 1;
    if (e_unb < -6) e_unb = -6;
    double step = ldexp(1.0, e_unb - 3);
    double q = nearbyint(a / step);      /* default rounding mode: to nearest, ties to even */
    double r = q * step;                 /* may carry into the next binade, still representable */
    if (r >= 448.0) return sign | 0x7E;
    if (r < ldexp(1.0, -6)) return sign | (uint8_t)q;          /* subnormal: q = mantissa (0..7), or 8 = 2^-6 */
    int er;
    double fr = frexp(r, &er);           /* r = fr * 2^er */
    int e = er - 1 + 7;
    int m = (int)nearbyint((fr * 2.0 - 1.0) * 8.0);
    return sign | (uint8_t)(e << 3) | (uint8_t)m;
}

/* value a cache position holds for input x: x itself, or scale * fp8(x / scale) */
static float cache_value(float x, int fp8, double scale)
{
    if (!fp8) return x;
    return (float)(scale * orc_fp8_e4m3_decode(orc_fp8_e4m3_encode((double)x / scale)));
}

static void cache_store(float *dst, const float *src, int n, int fp8, double scale)
{
    for (int i = 0; i < n; ++i) dst[i] = cache_value(src[i], fp8, scale);
}

/* exposed for the cache-fill helper of the tests */
void orc_cache_quantise(float *x, size_t n, double scale)
{
    for (size_t i = 0; i < n; ++i) x[i] = cache_value(x[i], 1, scale);
}

/*
 * 8-bit weights: every row of a [n_rows, K] matrix is replaced by s * fp8(w / s) with the row's own
 * scale s, the smallest power of two with max|w_row| / s <= 448 (1 for a row of zeros).  The layer
 * then runs unchanged on the replaced weights.
 */
static double row_scale(const float *w, int K)
{
    double m = 0.0;
    for (int k = 0; k < K; ++k)
        if (fabs((double)w[k]) > m) m = fabs((double)w[k]);
    double s = 1.0;
    if (m > 0.0 && isfinite(m)) {
        int e;
        double f = frexp(m / 448.0, &e);          /* m / 448 = f * 2^e, f in [0.5, 1) */
        s = ldexp(1.0, f == 0.5 ? e - 1 : e);     /* smallest power of two >= m / 448 */
    }
    return s;
}

void orc_quantise_rows(float *W, int n_rows, int K, float *scales)
{
    for (int n = 0; n < n_rows; ++n) {
        float *w = W + (size_t)n * K;
        double s = row_scale(w, K);
        for (int k = 0; k < K; ++k) w[k] = cache_value(w[k], 1, s);
        if (scales) scales[n] = (float)s;
    }
}

/*
 * 8-bit activations: a call whose configuration has act8 set gives every projection (q/k/v, output,
 * gate/up, down) its input row replaced by s * fp8(v / s), s as for a weight row.  Whether a call
 * quantises is the caller's statement, call by call; nothing here decides it.  The tensor being
 * quantised is a bf16 tensor (bf16 is the storage precision of the activations of an 8-bit layer),
 * so the row is first rounded to bf16 (nearest even) and the codes are those of the stored values.
 */
static float round_bf16(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return x; /* NaN */
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&x, &u, 4);
    return x;
}

/* rows of v replaced in place; scales [n_rows] and codes [n_rows, n] (the E4M3 bytes) are optional outputs */
void orc_act_quantise_rows(float *v, int n_rows, int n, float *scales, uint8_t *codes)
{
    for (int r = 0; r < n_rows; ++r) {
        float *row = v + (size_t)r * n;
        for (int i = 0; i < n; ++i) row[i] = round_bf16(row[i]);
        double s = row_scale(row, n);
        for (int i = 0; i < n; ++i) {
            uint8_t c = orc_fp8_e4m3_encode((double)row[i] / s);
            if (codes) codes[(size_t)r * n + i] = c;
            row[i] = (float)(s * orc_fp8_e4m3_decode(c));
        }
        if (scales) scales[r] = (float)s;
    }
}

static void act_quantise_row(float *v, int n) { orc_act_quantise_rows(v, 1, n, NULL, NULL); }

void orc_rmsnorm_row(const float *x, const float *g, int d, double eps, float *y)
{
    double ss = 0.0;
    for (int j = 0; j < d; ++j) ss += (double)x[j] * (double)x[j];
    double inv = 1.0 / sqrt(ss / (double)d + eps);
    for (int j = 0; j < d; ++j) y[j] = (float)((double)x[j] * inv * (double)g[j]);
}

void orc_rmsnorm(const float *x, const float *g, int T, int d, double eps, float *y)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) orc_rmsnorm_row(x + (size_t)t * d, g, d, eps, y + (size_t)t * d);
}

/* y[o] = sum_i x[i] W[o][i]   (one row; W is [n_out, n_in] row-major) */
void orc_linear_row(const float *x, const float *W, int n_in, int n_out, float *y)
{
    for (int o = 0; o < n_out; ++o) {
        const float *w = W + (size_t)o * n_in;
        double acc = 0.0;
#pragma omp simd reduction(+ : acc)
        for (int i = 0; i < n_in; ++i) acc += (double)x[i] * (double)w[i];
        y[o] = (float)acc;
    }
}

/*
 * Ends of the decoder stack (the layers sit between them):
 *   embedding  hidden[t, :] = E[id[t], :]                                  (-1 if an id is outside 0 .. V-1)
 *   LM head    logits[t, :] = RMSNorm(hidden[t, :]; g, eps) . W^T          (W [V, d], no bias)
 */
int orc_embed(const float *E, const int32_t *ids, int T, int d, int V, float *hidden)
{
    for (int t = 0; t < T; ++t)
        if (ids[t] < 0 || ids[t] >= V) return -1;
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < d; ++j) hidden[(size_t)t * d + j] = E[(size_t)ids[t] * d + j];
    return 0;
}

void orc_lm_head(const float *hidden, const float *g, const float *W, int T, int d, int V, double eps,
                 float *logits)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int t = 0; t < T; ++t) {
        float *y = (float *)malloc(sizeof(float) * (size_t)d);
        orc_rmsnorm_row(hidden + (size_t)t * d, g, d, eps, y);
        orc_linear_row(y, W, d, V, logits + (size_t)t * V);
        free(y);
    }
}

void orc_linear(const float *x, const float *W, int T, int n_in, int n_out, float *y)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        orc_linear_row(x + (size_t)t * n_in, W, n_in, n_out, y + (size_t)t * n_out);
}

/*
 * Rotary embedding of one token's heads x[H][hd] at absolute position pos.
 * Rotate-half pairing: channel i (< hd/2) is paired with channel i + hd/2,
 * angle = pos * base^(-2i/hd).
 */
void orc_rope_row(float *x, int H, int hd, int pos, double base)
{
    int half = hd / 2;
    for (int h = 0; h < H; ++h) {
        float *v = x + (size_t)h * hd;
        for (int i = 0; i < half; ++i) {
            double theta = pow(base, -2.0 * (double)i / (double)hd);
            double ang = (double)pos * theta;
            double c = cos(ang), s = sin(ang);
            double a = v[i], b = v[i + half];
            v[i] = (float)(a * c - b * s);
            v[i + half] = (float)(b * c + a * s);
        }
    }
}

/*
 * One query token attending over n_keys keys (softmax with max subtraction).
 * q is [Hq][hd]; key s / kv-head g lives at K + s*stride_s + g*stride_h.
 * Query head h reads kv-head h / (Hq/Hkv).  o is [Hq][hd].
 */
void orc_attend_row(const float *q, const float *K, const float *V, size_t stride_s,
                    size_t stride_h, int n_keys, int Hq, int Hkv, int hd, float *o)
{
    int group = Hq / Hkv;
    double scale = 1.0 / sqrt((double)hd);
    double *p = (double *)malloc(sizeof(double) * (size_t)n_keys);
    for (int h = 0; h < Hq; ++h) {
        int g = h / group;
        const float *qh = q + (size_t)h * hd;
        double mx = -INFINITY;
        for (int s = 0; s < n_keys; ++s) {
            const float *ks = K + (size_t)s * stride_s + (size_t)g * stride_h;
            double acc = 0.0;
            for (int i = 0; i < hd; ++i) acc += (double)qh[i] * (double)ks[i];
            p[s] = acc * scale;
            if (p[s] > mx) mx = p[s];
        }
        double denom = 0.0;
        for (int s = 0; s < n_keys; ++s) {
            p[s] = exp(p[s] - mx);
            denom += p[s];
        }
        for (int i = 0; i < hd; ++i) {
            double acc = 0.0;
            for (int s = 0; s < n_keys; ++s)
                acc += p[s] * (double)V[(size_t)s * stride_s + (size_t)g * stride_h + i];
            o[(size_t)h * hd + i] = (float)(acc / denom);
        }
    }
    free(p);
}

static double silu(double z) { return z / (1.0 + exp(-z)); }

/* out[d] += scale * Wd (silu(Wg y) * (Wu y)) for one token and one FFN. */
static void ffn_row_accumulate(const float *y, const float *Wg, const float *Wu, const float *Wd,
                               int d, int F, double scale, double *out_acc, float *act, int q8)
{
    for (int f = 0; f < F; ++f) {
        const float *wg = Wg + (size_t)f * d, *wu = Wu + (size_t)f * d;
        double a = 0.0, b = 0.0;
#pragma omp simd reduction(+ : a, b)
        for (int i = 0; i < d; ++i) {
            a += (double)y[i] * (double)wg[i];
            b += (double)y[i] * (double)wu[i];
        }
        act[f] = (float)(silu(a) * b);
    }
    if (q8) act_quantise_row(act, F);
    for (int o = 0; o < d; ++o) {
        const float *wd = Wd + (size_t)o * F;
        double acc = 0.0;
#pragma omp simd reduction(+ : acc)
        for (int f = 0; f < F; ++f) acc += (double)act[f] * (double)wd[f];
        out_acc[o] += scale * acc;
    }
}

/*
 * Router for one token: p = softmax(logits over all E experts); pick the top_k
 * largest p (ties: lower expert index first); weights renormalised to sum 1.
 */
void orc_route_row(const float *logits, int E, int top_k, int32_t *idx, double *wgt)
{
    double mx = -INFINITY, denom = 0.0;
    double *p = (double *)malloc(sizeof(double) * (size_t)E);
    for (int e = 0; e < E; ++e)
        if ((double)logits[e] > mx) mx = (double)logits[e];
    for (int e = 0; e < E; ++e) {
        p[e] = exp((double)logits[e] - mx);
        denom += p[e];
    }
    for (int e = 0; e < E; ++e) p[e] /= denom;
    double sum = 0.0;
    for (int k = 0; k < top_k; ++k) {
        int best = -1;
        for (int e = 0; e < E; ++e) {
            int taken = 0;
            for (int j = 0; j < k; ++j)
                if (idx[j] == e) taken = 1;
            if (taken) continue;
            if (best < 0 || p[e] > p[best]) best = e; /* strict '>' keeps the lower index on ties */
        }
        idx[k] = best;
        wgt[k] = p[best];
        sum += p[best];
    }
    for (int k = 0; k < top_k; ++k) wgt[k] /= sum;
    free(p);
}

/* Second half of the layer for one token: out = h + FFN(rmsnorm(h)). */
static void ffn_block_row(const orc_config *c, const orc_weights *w, const float *h,
                          const float *router_logits_row, float *out, int32_t *expert_idx_out, int q8)
{
    int d = c->d_model, F = c->d_ff;
    float *y2 = (float *)malloc(sizeof(float) * (size_t)d);
    float *act = (float *)malloc(sizeof(float) * (size_t)F);
    double *acc = (double *)calloc((size_t)d, sizeof(double));
    orc_rmsnorm_row(h, w->g_ffn, d, c->rms_eps, y2);
    if (c->n_experts <= 0) {
        if (q8) act_quantise_row(y2, d);
        ffn_row_accumulate(y2, w->w_gate, w->w_up, w->w_down, d, F, 1.0, acc, act, q8);
    } else {
        int E = c->n_experts, K = c->top_k;
        float *logits = (float *)malloc(sizeof(float) * (size_t)E);
        int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
        double *wgt = (double *)malloc(sizeof(double) * (size_t)K);
        if (router_logits_row) {
            memcpy(logits, router_logits_row, sizeof(float) * (size_t)E);
        } else {
            orc_linear_row(y2, w->w_router, d, E, logits);
        }
        orc_route_row(logits, E, K, idx, wgt);
        if (q8) act_quantise_row(y2, d);   /* after routing: the router reads the unquantised row */
        for (int k = 0; k < K; ++k) {
            size_t e = (size_t)idx[k];
            ffn_row_accumulate(y2, w->w_gate + e * (size_t)F * d, w->w_up + e * (size_t)F * d,
                               w->w_down + e * (size_t)d * F, d, F, wgt[k], acc, act, q8);
            if (expert_idx_out) expert_idx_out[k] = idx[k];
        }
        free(logits);
        free(idx);
        free(wgt);
    }
    for (int o = 0; o < d; ++o) out[o] = (float)((double)h[o] + acc[o]);
    free(y2);
    free(act);
    free(acc);
}

/*
 * Prefill of a packed batch of sequences.
 *
 *   x            [T, d] hidden-state rows; sequence s owns rows cu_seqlens[s] .. cu_seqlens[s+1]-1
 *   router_logits [T, E] or NULL (then w_router is used when the layer is MoE)
 *   rows / n_rows  if rows != NULL only those token rows are produced: out is
 *                [n_rows, d] in the order of rows[].  Keys and values are still
 *                computed for every earlier token of the same sequence, so the
 *                sampled rows equal the rows of a full evaluation.
 *   slots        NULL, or n_seqs cache slots: rotated k and v of sequence s are
 *                stored in k_cache/v_cache [n_slots][Hkv][max_len][hd] and
 *                lens[slot] = length.  (Requires rows == NULL.)
 *   expert_idx   NULL or [n_out_rows, top_k] chosen experts (MoE)
 * Returns 0, or -1 on an invalid argument.
 */
int orc_prefill(const orc_config *c, const orc_weights *w, const float *x, int T, int n_seqs,
                const int32_t *cu_seqlens, const float *router_logits, const int32_t *rows,
                int n_rows, const int32_t *slots, float *k_cache, float *v_cache, int32_t *lens,
                int max_len, float *out, int32_t *expert_idx, int kv_fp8, double k_scale,
                double v_scale)
{
    int d = c->d_model, Hq = c->n_q_heads, Hkv = c->n_kv_heads, hd = c->head_dim;
    const int q8 = c->act8 != 0;   /* 8-bit activations in this call */
    if (Hkv <= 0 || Hq % Hkv != 0 || hd % 2 != 0) return -1;
    if (cu_seqlens[0] != 0 || cu_seqlens[n_seqs] != T) return -1;
    if (slots && rows) return -1;
    size_t dq = (size_t)Hq * hd, dkv = (size_t)Hkv * hd;

    int32_t *seq_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    char *need_out = (char *)calloc((size_t)(T > 0 ? T : 1), 1);
    char *need_kv = (char *)calloc((size_t)(T > 0 ? T : 1), 1);
    int32_t *out_slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    for (int s = 0; s < n_seqs; ++s) {
        if (cu_seqlens[s + 1] < cu_seqlens[s]) return -1;
        for (int t = cu_seqlens[s]; t < cu_seqlens[s + 1]; ++t) seq_of[t] = s;
    }
    if (rows) {
        for (int r = 0; r < n_rows; ++r) {
            if (rows[r] < 0 || rows[r] >= T) return -1;
            need_out[rows[r]] = 1;
        }
    } else {
        for (int t = 0; t < T; ++t) need_out[t] = 1;
    }
    /* a token's k,v are needed if it or any later token of its sequence is produced */
    for (int s = 0; s < n_seqs; ++s) {
        int later = 0;
        for (int t = cu_seqlens[s + 1] - 1; t >= cu_seqlens[s]; --t) {
            if (need_out[t]) later = 1;
            need_kv[t] = (char)later;
        }
    }

    float *kbuf = (float *)calloc((size_t)(T > 0 ? T : 1) * dkv, sizeof(float));
    float *vbuf = (float *)calloc((size_t)(T > 0 ? T : 1) * dkv, sizeof(float));

    /* pass 1: normalise, project and rotate keys / values */
#pragma omp parallel for schedule(dynamic, 4)
    for (int t = 0; t < T; ++t) {
        if (!need_kv[t]) continue;
        float *y = (float *)malloc(sizeof(float) * (size_t)d);
        orc_rmsnorm_row(x + (size_t)t * d, w->g_attn, d, c->rms_eps, y);
        if (q8) act_quantise_row(y, d);
        orc_linear_row(y, w->w_k, d, (int)dkv, kbuf + (size_t)t * dkv);
        orc_linear_row(y, w->w_v, d, (int)dkv, vbuf + (size_t)t * dkv);
        orc_rope_row(kbuf + (size_t)t * dkv, Hkv, hd, t - cu_seqlens[seq_of[t]], c->rope_base);
        free(y);
    }
    if (slots) {
        for (int s = 0; s < n_seqs; ++s) {
            int L = cu_seqlens[s + 1] - cu_seqlens[s];
            if (L > max_len) return -1;
            size_t base = (size_t)slots[s] * Hkv * (size_t)max_len * hd;
            for (int p = 0; p < L; ++p)
                for (int g = 0; g < Hkv; ++g) {
                    size_t dst = base + ((size_t)g * max_len + p) * hd;
                    size_t src = (size_t)(cu_seqlens[s] + p) * dkv + (size_t)g * hd;
                    cache_store(k_cache + dst, kbuf + src, hd, kv_fp8, k_scale);
                    cache_store(v_cache + dst, vbuf + src, hd, kv_fp8, v_scale);
                }
            lens[slots[s]] = L;
        }
    }
    if (rows) {
        for (int r = 0; r < n_rows; ++r) out_slot[rows[r]] = r;
    } else {
        for (int t = 0; t < T; ++t) out_slot[t] = t;
    }

    /* pass 2: queries, attention, output projection, FFN for produced rows */
#pragma omp parallel for schedule(dynamic, 1)
    for (int t = 0; t < T; ++t) {
        if (!need_out[t]) continue;
        int s0 = cu_seqlens[seq_of[t]];
        float *y = (float *)malloc(sizeof(float) * (size_t)d);
        float *q = (float *)malloc(sizeof(float) * dq);
        float *o = (float *)malloc(sizeof(float) * dq);
        float *h = (float *)malloc(sizeof(float) * (size_t)d);
        orc_rmsnorm_row(x + (size_t)t * d, w->g_attn, d, c->rms_eps, y);
        if (q8) act_quantise_row(y, d);
        orc_linear_row(y, w->w_q, d, (int)dq, q);
        orc_rope_row(q, Hq, hd, t - s0, c->rope_base);
        orc_attend_row(q, kbuf + (size_t)s0 * dkv, vbuf + (size_t)s0 * dkv, dkv, (size_t)hd,
                       t - s0 + 1, Hq, Hkv, hd, o);
        if (q8) act_quantise_row(o, (int)dq);
        orc_linear_row(o, w->w_o, (int)dq, d, h);
        for (int i = 0; i < d; ++i) h[i] = (float)((double)x[(size_t)t * d + i] + (double)h[i]);
        size_t r = (size_t)out_slot[t];
        ffn_block_row(c, w, h, router_logits ? router_logits + (size_t)t * c->n_experts : NULL,
                      out + r * d, expert_idx ? expert_idx + r * (size_t)c->top_k : NULL, q8);
        free(y);
        free(q);
        free(o);
        free(h);
    }
    free(seq_of);
    free(need_out);
    free(need_kv);
    free(out_slot);
    free(kbuf);
    free(vbuf);
    return 0;
}

/*
 * One decode step for B sequences.  Row b is the newest token of the sequence
 * held in cache slot slots[b]; its position is p = lens[slot].  Its rotated key
 * and its value are appended at p first, then it attends over positions 0..p
 * (itself included), and lens[slot] becomes p + 1.
 * Caches are [n_slots][Hkv][max_len][hd] fp32.  Returns 0, -1 bad argument,
 * -2 cache capacity exceeded (nothing is modified in that case).
 */
int orc_decode_step(const orc_config *c, const orc_weights *w, const float *x, int B,
                    const int32_t *slots, float *k_cache, float *v_cache, int32_t *lens,
                    int max_len, const float *router_logits, float *out, int32_t *expert_idx,
                    int kv_fp8, double k_scale, double v_scale)
{
    int d = c->d_model, Hq = c->n_q_heads, Hkv = c->n_kv_heads, hd = c->head_dim;
    const int q8 = c->act8 != 0;   /* 8-bit activations in this call */
    if (Hkv <= 0 || Hq % Hkv != 0 || hd % 2 != 0) return -1;
    size_t dq = (size_t)Hq * hd, dkv = (size_t)Hkv * hd;
    for (int b = 0; b < B; ++b)
        if (lens[slots[b]] + 1 > max_len) return -2;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int slot = slots[b], p = lens[slot];
        float *y = (float *)malloc(sizeof(float) * (size_t)d);
        float *q = (float *)malloc(sizeof(float) * dq);
        float *k = (float *)malloc(sizeof(float) * dkv);
        float *v = (float *)malloc(sizeof(float) * dkv);
        float *o = (float *)malloc(sizeof(float) * dq);
        float *h = (float *)malloc(sizeof(float) * (size_t)d);
        orc_rmsnorm_row(x + (size_t)b * d, w->g_attn, d, c->rms_eps, y);
        if (q8) act_quantise_row(y, d);
        orc_linear_row(y, w->w_q, d, (int)dq, q);
        orc_linear_row(y, w->w_k, d, (int)dkv, k);
        orc_linear_row(y, w->w_v, d, (int)dkv, v);
        orc_rope_row(q, Hq, hd, p, c->rope_base);
        orc_rope_row(k, Hkv, hd, p, c->rope_base);
        size_t base = (size_t)slot * Hkv * (size_t)max_len * hd;
        for (int g = 0; g < Hkv; ++g) {
            cache_store(k_cache + base + ((size_t)g * max_len + p) * hd, k + (size_t)g * hd, hd, kv_fp8, k_scale);
            cache_store(v_cache + base + ((size_t)g * max_len + p) * hd, v + (size_t)g * hd, hd, kv_fp8, v_scale);
        }
        orc_attend_row(q, k_cache + base, v_cache + base, (size_t)hd, (size_t)max_len * hd, p + 1,
                       Hq, Hkv, hd, o);
        if (q8) act_quantise_row(o, (int)dq);
        orc_linear_row(o, w->w_o, (int)dq, d, h);
        for (int i = 0; i < d; ++i) h[i] = (float)((double)x[(size_t)b * d + i] + (double)h[i]);
        ffn_block_row(c, w, h, router_logits ? router_logits + (size_t)b * c->n_experts : NULL,
                      out + (size_t)b * d, expert_idx ? expert_idx + (size_t)b * c->top_k : NULL, q8);
        free(y);
        free(q);
        free(k);
        free(v);
        free(o);
        free(h);
    }
    for (int b = 0; b < B; ++b) lens[slots[b]] += 1;
    return 0;
}

/*
 * Chunked prefill: a packed batch of chunks, each continuing the sequence held in
 * a cache slot (the paper's "Evaluation" discusses the prefill chunk size; a chunk
 * is a run of new prompt tokens processed against the prefix already cached).
 * Sequence s owns rows cu_seqlens[s] .. cu_seqlens[s+1]-1; with P = lens[slots[s]]
 * cached tokens, its i-th row is the token at position P + i: its rotated key and
 * its value are stored at that position, and it attends over positions 0 .. P + i
 * (the whole prefix, the earlier rows of the chunk, itself).  Afterwards
 * lens[slot] = P + L.  P = 0 is an ordinary prefill; L = 1 is a decode step.
 * Slots must be distinct.  Returns 0, -1 bad argument, -2 cache capacity exceeded
 * (nothing is modified in that case).
 *
 * kv_fp8 != 0 (here, in orc_prefill and in orc_decode_step): the cache holds keys and values as
 * 8-bit E4M3 numbers with the static scales k_scale / v_scale, i.e. a stored element reads back
 * as scale * fp8(x / scale).  Whatever attention reads from the cache is the quantised value;
 * orc_prefill's own attention works on the fresh keys and values and only its stores quantise.
 */
int orc_prefill_chunk(const orc_config *c, const orc_weights *w, const float *x, int T, int n_seqs,
                      const int32_t *cu_seqlens, const float *router_logits, const int32_t *slots,
                      float *k_cache, float *v_cache, int32_t *lens, int max_len, float *out,
                      int32_t *expert_idx, int kv_fp8, double k_scale, double v_scale)
{
    int d = c->d_model, Hq = c->n_q_heads, Hkv = c->n_kv_heads, hd = c->head_dim;
    const int q8 = c->act8 != 0;   /* 8-bit activations in this call */
    if (Hkv <= 0 || Hq % Hkv != 0 || hd % 2 != 0) return -1;
    if (!slots || cu_seqlens[0] != 0 || cu_seqlens[n_seqs] != T) return -1;
    size_t dq = (size_t)Hq * hd, dkv = (size_t)Hkv * hd;
    for (int s = 0; s < n_seqs; ++s) {
        if (cu_seqlens[s + 1] < cu_seqlens[s]) return -1;
        for (int r = 0; r < s; ++r)
            if (slots[r] == slots[s]) return -1;
    }
    for (int s = 0; s < n_seqs; ++s)
        if (lens[slots[s]] + (cu_seqlens[s + 1] - cu_seqlens[s]) > max_len) return -2;

    int32_t *seq_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    for (int s = 0; s < n_seqs; ++s)
        for (int t = cu_seqlens[s]; t < cu_seqlens[s + 1]; ++t) seq_of[t] = s;

    /* pass 1: keys and values of the new tokens go into the cache behind the prefix */
#pragma omp parallel for schedule(dynamic, 4)
    for (int t = 0; t < T; ++t) {
        int s = seq_of[t], slot = slots[s];
        int pos = lens[slot] + (t - cu_seqlens[s]);
        float *y = (float *)malloc(sizeof(float) * (size_t)d);
        float *k = (float *)malloc(sizeof(float) * dkv);
        float *v = (float *)malloc(sizeof(float) * dkv);
        orc_rmsnorm_row(x + (size_t)t * d, w->g_attn, d, c->rms_eps, y);
        if (q8) act_quantise_row(y, d);
        orc_linear_row(y, w->w_k, d, (int)dkv, k);
        orc_linear_row(y, w->w_v, d, (int)dkv, v);
        orc_rope_row(k, Hkv, hd, pos, c->rope_base);
        size_t base = (size_t)slot * Hkv * (size_t)max_len * hd;
        for (int g = 0; g < Hkv; ++g) {
            cache_store(k_cache + base + ((size_t)g * max_len + pos) * hd, k + (size_t)g * hd, hd, kv_fp8, k_scale);
            cache_store(v_cache + base + ((size_t)g * max_len + pos) * hd, v + (size_t)g * hd, hd, kv_fp8, v_scale);
        }
        free(y);
        free(k);
        free(v);
    }

    /* pass 2: each new token attends over cache positions 0 .. its own */
#pragma omp parallel for schedule(dynamic, 1)
    for (int t = 0; t < T; ++t) {
        int s = seq_of[t], slot = slots[s];
        int pos = lens[slot] + (t - cu_seqlens[s]);
        float *y = (float *)malloc(sizeof(float) * (size_t)d);
        float *q = (float *)malloc(sizeof(float) * dq);
        float *o = (float *)malloc(sizeof(float) * dq);
        float *h = (float *)malloc(sizeof(float) * (size_t)d);
        orc_rmsnorm_row(x + (size_t)t * d, w->g_attn, d, c->rms_eps, y);
        if (q8) act_quantise_row(y, d);
        orc_linear_row(y, w->w_q, d, (int)dq, q);
        orc_rope_row(q, Hq, hd, pos, c->rope_base);
        size_t base = (size_t)slot * Hkv * (size_t)max_len * hd;
        orc_attend_row(q, k_cache + base, v_cache + base, (size_t)hd, (size_t)max_len * hd, pos + 1,
                       Hq, Hkv, hd, o);
        if (q8) act_quantise_row(o, (int)dq);
        orc_linear_row(o, w->w_o, (int)dq, d, h);
        for (int i = 0; i < d; ++i) h[i] = (float)((double)x[(size_t)t * d + i] + (double)h[i]);
        ffn_block_row(c, w, h, router_logits ? router_logits + (size_t)t * c->n_experts : NULL,
                      out + (size_t)t * d, expert_idx ? expert_idx + (size_t)t * c->top_k : NULL, q8);
        free(y);
        free(q);
        free(o);
        free(h);
    }
    for (int s = 0; s < n_seqs; ++s) lens[slots[s]] += cu_seqlens[s + 1] - cu_seqlens[s];
    free(seq_of);
    return 0;
}

/* Stand-alone pieces exposed so that tests can pin each one separately. */
void orc_rope(float *x, int T, int H, int hd, const int32_t *pos, double base)
{
    for (int t = 0; t < T; ++t) orc_rope_row(x + (size_t)t * H * hd, H, hd, pos[t], base);
}

/* Causal attention over one packed batch; q [T,Hq,hd], k,v [T,Hkv,hd], o [T,Hq,hd]. */
void orc_attention(const float *q, const float *k, const float *v, int n_seqs,
                   const int32_t *cu_seqlens, int Hq, int Hkv, int hd, float *o)
{
    size_t dq = (size_t)Hq * hd, dkv = (size_t)Hkv * hd;
    for (int s = 0; s < n_seqs; ++s) {
        int s0 = cu_seqlens[s], s1 = cu_seqlens[s + 1];
#pragma omp parallel for schedule(dynamic, 1)
        for (int t = s0; t < s1; ++t)
            orc_attend_row(q + (size_t)t * dq, k + (size_t)s0 * dkv, v + (size_t)s0 * dkv, dkv,
                           (size_t)hd, t - s0 + 1, Hq, Hkv, hd, o + (size_t)t * dq);
    }
}

/* out = h + FFN(rmsnorm(h)) for T rows (dense or MoE). */
void orc_ffn_block(const orc_config *c, const orc_weights *w, const float *h, int T,
                   const float *router_logits, float *out, int32_t *expert_idx)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int t = 0; t < T; ++t)
        ffn_block_row(c, w, h + (size_t)t * c->d_model,
                      router_logits ? router_logits + (size_t)t * c->n_experts : NULL,
                      out + (size_t)t * c->d_model,
                      expert_idx ? expert_idx + (size_t)t * c->top_k : NULL,
                      c->act8 != 0);
}
