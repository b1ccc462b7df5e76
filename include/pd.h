/*
 * pd.h - C ABI of the prefill/decode layer-forward library and of the P/D allocation model.
 *
 * The paper sizes a prefill/decode-disaggregated deployment from two measured curves of one
 * serving instance (maximum prefill throughput at a given input length; TPOT versus decode batch)
 * and closed forms (Eqs. (5)-(7), (13)).  This library provides the measured side on one GPU -
 * one decoder layer's forward pass, for prefill and for a batched single-token decode step over a
 * KV cache - and the closed forms themselves.
 *
 * Conventions
 *   - Plain C, no exceptions cross the boundary; every call returns a pd_status.
 *   - "device" pointers are HIP device memory on the current device; "host" pointers are ordinary
 *     host memory.  The caller owns every tensor it passes and keeps it alive until the stream has
 *     executed the call's work.  The library owns only its opaque handles (and the repacked copies
 *     of the weights they hold).  *_destroy(NULL) is a no-op.
 *   - pd_prefill / pd_decode_step only enqueue work on the given stream (a hipStream_t passed as
 *     void*, NULL = default stream) and do not synchronise; small host arrays (cu_seqlens, slots)
 *     are consumed during the call.  A layer's scratch workspace is shared by all calls on that
 *     layer: calls on one layer must be ordered on one stream.  The workspace grows on demand
 *     (device allocation, which may synchronise); pd_layer_reserve sizes it ahead of time.
 *   - Tensors are row-major; "hidden" rows are hidden-state vectors, not token ids.  Element type
 *     is the layer's dtype (fp32 or bf16) unless stated otherwise.
 *   - On error nothing is enqueued, no output is written and no state changes; pd_last_error()
 *     returns a thread-local description of the last failure.
 *   - Throughputs are tokens per second, times are seconds, lengths are (mean) token counts.
 */
#ifndef PD_H
#define PD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PD_OK = 0,
    PD_ERR_INVALID_ARG = 1,
    PD_ERR_SHAPE = 2,
    PD_ERR_DTYPE = 3,
    PD_ERR_OOM = 4,
    PD_ERR_DEVICE = 5,
    PD_ERR_KV_CAPACITY = 6,
    PD_ERR_TTFT_INFEASIBLE = 7,
    PD_ERR_TPOT_INFEASIBLE = 8
} pd_status;

typedef enum { PD_F32 = 0, PD_BF16 = 1 } pd_dtype;

/*
 * One pre-norm decoder layer (the unit whose forward time the method benchmarks; the paper's
 * Introduction characterises prefill as compute-bound and decode as memory-bandwidth-bound):
 *   y = rmsnorm(x, g_attn); q,k,v = y Wq^T, y Wk^T, y Wv^T; rotary embedding of q,k (rotate-half
 *   pairing, angle = position * rope_base^(-2i/head_dim)); causal grouped-query attention with
 *   scale 1/sqrt(head_dim) (query head h reads kv head h / (n_q_heads/n_kv_heads));
 *   h = x + o Wo^T; y2 = rmsnorm(h, g_ffn); out = h + (silu(y2 Wg^T) * (y2 Wu^T)) Wd^T,
 *   or, when n_experts > 0, out = h + sum over the top_k experts of w_e FFN_e(y2) with
 *   p = softmax(router logits over all experts), ties to the lower index, w = p_top / sum p_top.
 * rmsnorm(x, g)_i = x_i / sqrt(mean_j x_j^2 + rms_eps) * g_i.
 */
typedef struct {
    int32_t d_model, n_q_heads, n_kv_heads, head_dim, d_ff;
    int32_t n_experts; /* 0 = dense FFN */
    int32_t top_k;     /* used when n_experts > 0 */
    float rms_eps, rope_base;
    int32_t dtype;     /* pd_dtype */
} pd_layer_config;

/* Device pointers, each [out_features, in_features] row-major in the layer's dtype. */
typedef struct {
    const void *g_attn;   /* [d] */
    const void *w_q;      /* [n_q_heads*head_dim, d] */
    const void *w_k;      /* [n_kv_heads*head_dim, d] */
    const void *w_v;      /* [n_kv_heads*head_dim, d] */
    const void *w_o;      /* [d, n_q_heads*head_dim] */
    const void *g_ffn;    /* [d] */
    const void *w_gate;   /* [F, d]   (MoE: [E, F, d]) */
    const void *w_up;     /* [F, d]   (MoE: [E, F, d]) */
    const void *w_down;   /* [d, F]   (MoE: [E, d, F]) */
    const void *w_router; /* [E, d] or NULL (then router logits must be passed per call) */
} pd_layer_weights;

typedef struct pd_layer pd_layer;       /* opaque */
typedef struct pd_kv_cache pd_kv_cache; /* opaque */

/*
 * Creates a layer on the current device.  The weights are copied (and repacked) into memory the
 * layer owns; the caller's buffers may be released once the call returns (the call synchronises).
 * Errors: PD_ERR_INVALID_ARG (NULL), PD_ERR_SHAPE (non-positive sizes, odd head_dim, n_q_heads not
 * a multiple of n_kv_heads, top_k > n_experts, top_k > 8, n_experts > 64, head_dim > 256),
 * PD_ERR_DTYPE, PD_ERR_OOM, PD_ERR_DEVICE.
 */
pd_status pd_layer_create(const pd_layer_config *cfg, const pd_layer_weights *w, pd_layer **out);
/*
 * The same layer with 8-bit weights: every projection matrix (W_q, W_k, W_v, W_o, gate, up, down;
 * not the norm gains, not the router) is held as OCP E4M3 codes with one scale per output row,
 * the smallest power of two s with max|w_row| / s <= 448 (1 for a row of zeros); the layer then
 * computes with w' = s * value(code) everywhere (activations stay bf16).  Decode is bound by
 * reading the weights (Introduction: decode is bound by memory bandwidth), so dense calls of up
 * to 128 rows stream the codes (half the bytes) and widen them in registers; larger calls use a
 * bf16 copy of w' and give the same results
 * as a layer created from w' with pd_layer_create.  All other calls take such a layer unchanged.
 * Errors: as pd_layer_create, plus PD_ERR_DTYPE if the layer is not bf16 with d_model, d_ff and the
 * head dimensions multiples of 64.
 */
pd_status pd_layer_create_w8(const pd_layer_config *cfg, const pd_layer_weights *w, pd_layer **out);

/*
 * 8-bit weights as above and, where the layer is bound by the matrix cores (Introduction: prefill
 * is compute-bound), 8-bit activations too: in every call of more than 256 rows (T of a prefill call, B of a decode
 * call) each of the four projections first quantises its bf16 input rows (the normalised hidden
 * state, the attention output, the SwiGLU output) like pd_quantize_rows_e4m3 and multiplies codes
 * by codes in E4M3 on the matrix cores with fp32 accumulation; the sums are multiplied by the two
 * scales.  In a mixture-of-experts layer the normalised row is quantised once per token (the router
 * reads it unquantised) and the SwiGLU row once per (token, expert) pair.  Calls of up to 256 rows
 * behave as in a pd_layer_create_w8 layer.
 * Errors: as pd_layer_create_w8, plus PD_ERR_DTYPE when d_model, d_ff or n_q_heads * head_dim is not
 * a multiple of 128.
 */
pd_status pd_layer_create_w8a8(const pd_layer_config *cfg, const pd_layer_weights *w, pd_layer **out);
void pd_layer_destroy(pd_layer *layer);

/*
 * Row-wise 8-bit quantisation as used for activations by a pd_layer_create_w8a8 layer:
 * x [n_rows, n_cols] bf16 (device, row-major, n_cols a multiple of 8) -> codes [n_rows, n_cols]
 * bytes (device) and scales [n_rows] fp32 (device); scale = the smallest power of two s with
 * max|x_row| / s <= 448 (1 for a row of zeros or one holding an infinity), code = OCP E4M3 of
 * x / s, rounded to nearest even, saturating at +-448.  Asynchronous on stream.
 * Errors: PD_ERR_INVALID_ARG (NULL pointer, negative n_rows, n_cols not a positive multiple of 8).
 */
pd_status pd_quantize_rows_e4m3(const void *x, int32_t n_rows, int32_t n_cols, void *codes,
                                float *scales, void *stream);

/*
 * The product a pd_layer_create_w8a8 layer computes in its projections, on its own:
 *   c[m, n] = a_scales[m] * b_scales[n] * sum_k value(a_codes[m, k]) * value(b_codes[n, k])
 * a_codes [M, K] and b_codes [N, K] are row-major OCP E4M3 bytes (device), the scales fp32 (device),
 * c [M, N] bf16 (device); products and sums in fp32 on the matrix cores, one rounding to bf16.
 * A synchronous helper for tests and tools, unlike every other call that takes a stream: it
 * allocates temporary device memory, returns after the work on stream has finished, and must not
 * be called while the stream is being captured into a graph.
 * Errors: PD_ERR_INVALID_ARG (NULL pointer), PD_ERR_SHAPE (M < 1, N not a multiple of 16, K not a
 * multiple of 128, an operand of 4 GiB or more), PD_ERR_DEVICE.
 */
pd_status pd_gemm_e4m3(const void *a_codes, const float *a_scales, const void *b_codes,
                       const float *b_scales, int32_t M, int32_t N, int32_t K, void *c, void *stream);

/*
 * Pre-sizes the layer's workspace for calls of up to max_tokens rows (prefill T or decode B).
 * A call with more rows than reserved so far (and a prefill whose attention scratch has to grow)
 * synchronises the device, frees the old workspace and allocates a larger one: a HIP graph
 * captured over this layer before that holds the freed addresses and must not be replayed again.
 * Reserve for the largest call first, then capture.
 */
pd_status pd_layer_reserve(pd_layer *layer, int32_t max_tokens);

/*
 * A KV cache of max_seqs slots, each holding up to max_len positions of rotated keys and values
 * for every kv head, in the layer's dtype.  The memory layout is private to the library.
 */
pd_status pd_kv_cache_create(const pd_layer *layer, int32_t max_seqs, int32_t max_len,
                             pd_kv_cache **out);
/*
 * The same cache stored as 8-bit floating point (OCP E4M3: 4 exponent bits with bias 7, 3 mantissa
 * bits, no infinities, largest finite value 448) with one static scale for keys and one for
 * values: an element x is held as the code nearest to x / scale (ties to the even mantissa,
 * saturating at +-448) and read as scale * value(code).  Decode is bound by reading the cache
 * (the memory-bandwidth-bound decode stage of the Introduction), so halving its bytes halves that
 * part of a step.
 * Everything attention reads from such a cache (pd_decode_step, pd_prefill_chunk, pd_kv_cache_get)
 * is the quantised value; pd_prefill's own attention works on the fresh keys and values and only
 * its stores quantise.  pd_kv_cache_set / _get still take and return tensors in the layer's dtype.
 * All other cache calls behave as for pd_kv_cache_create.
 * Errors: PD_ERR_INVALID_ARG (NULL, non-positive sizes, scales not positive and finite),
 * PD_ERR_DTYPE (layer is not bf16 with head_dim 128, at most 16 query heads per kv head and
 * dimensions that are multiples of 64), PD_ERR_OOM, PD_ERR_DEVICE.
 */
pd_status pd_kv_cache_create_fp8(const pd_layer *layer, int32_t max_seqs, int32_t max_len,
                                 double k_scale, double v_scale, pd_kv_cache **out);
void pd_kv_cache_destroy(pd_kv_cache *cache);

/*
 * Benchmark fill: copies len positions of (already rotated) keys and values, each a device tensor
 * [n_kv_heads, len, head_dim], into a slot and sets its length.  Enqueued on `stream`.
 * Errors: PD_ERR_INVALID_ARG (bad slot, NULL), PD_ERR_KV_CAPACITY (len > max_len).
 */
pd_status pd_kv_cache_set(pd_kv_cache *cache, int32_t slot, int32_t len, const void *k,
                          const void *v, void *stream);
/* Sets a slot's length without touching its contents (0 <= len <= max_len); used to rewind a
 * cache between timed repetitions of the same decode step.  Enqueued on `stream`. */
pd_status pd_kv_cache_set_len(pd_kv_cache *cache, int32_t slot, int32_t len, void *stream);
/* The same for n (slot, len) pairs at once (host arrays). */
pd_status pd_kv_cache_set_lens(pd_kv_cache *cache, int32_t n, const int32_t *slots,
                               const int32_t *lens, void *stream);
/* Reads a slot's length (host-side mirror; no device access). */
pd_status pd_kv_cache_len(const pd_kv_cache *cache, int32_t slot, int32_t *len);
/* Debug/test read-back of one slot's first len positions into device tensors [n_kv_heads, len, head_dim]. */
pd_status pd_kv_cache_get(const pd_kv_cache *cache, int32_t slot, int32_t len, void *k, void *v,
                          void *stream);

/*
 * Prefill: the layer forward over a packed batch of n_seqs sequences (T = cu_seqlens[n_seqs]
 * rows; sequence s owns rows cu_seqlens[s] .. cu_seqlens[s+1]-1 and its positions start at 0).
 * This is the operation whose saturated throughput is the paper's maximum prefill throughput
 * (section "Acquire prefill throughput under TTFT constraints").
 */
typedef struct {
    const void *hidden;          /* device [T, d] */
    int32_t n_seqs;              /* 1 .. 4096 */
    const int32_t *cu_seqlens;   /* host [n_seqs + 1], non-decreasing, cu_seqlens[0] = 0 */
    const int32_t *slots;        /* host [n_seqs] distinct cache slots, or NULL = keep no KV */
    const void *router_logits;   /* device fp32 [T, n_experts], or NULL (MoE: use w_router) */
} pd_tokens;

/*
 * Writes out_hidden (device [T, d]).  With a cache and slots, stores each sequence's rotated keys
 * and values into its slot and sets the slot's length to the sequence length.
 * Errors: PD_ERR_INVALID_ARG, PD_ERR_SHAPE (bad cu_seqlens), PD_ERR_KV_CAPACITY (a sequence longer
 * than max_len), PD_ERR_OOM / PD_ERR_DEVICE (workspace growth, launch failure).
 */
pd_status pd_prefill(pd_layer *layer, const pd_tokens *tokens, pd_kv_cache *cache /* nullable */,
                     void *out_hidden, void *stream);

/*
 * Chunked prefill: the same forward over a packed batch of chunks, each continuing the sequence
 * that a cache slot already holds (the paper's evaluation varies the prefill chunk size; a chunk is
 * a run of new prompt tokens processed against the cached prefix).  With P = the current length
 * of slots[s], row i of sequence s is the token at position P + i: its rotated key and its value
 * are appended at that position and it attends over positions 0 .. P + i.  Afterwards the slot's
 * length is P + L_s.  An empty slot makes this an ordinary prefill that keeps its KV; a chunk of
 * one token is a decode step.  cache and tokens->slots are required; a sequence may be empty.
 * Errors as pd_prefill; PD_ERR_KV_CAPACITY if P + L_s exceeds max_len for any sequence (checked
 * before anything is enqueued, nothing changes).
 */
pd_status pd_prefill_chunk(pd_layer *layer, const pd_tokens *tokens, pd_kv_cache *cache,
                           void *out_hidden, void *stream);

/*
 * One decode step (section "Acquire decode throughput under TPOT constraints": TPOT is measured as
 * a function of the decode batch).  Row b is the newest token of the sequence in slots[b], at
 * position p = len(slot).  Its rotated key and its value are appended at p, the row attends over
 * positions 0..p, and the slot's length becomes p + 1.
 */
typedef struct {
    const void *hidden;          /* device [B, d] */
    int32_t batch;               /* B, 1 .. 4096 */
    const int32_t *slots;        /* host [B], distinct */
    const void *router_logits;   /* device fp32 [B, n_experts], or NULL */
} pd_batch;

/* Errors as pd_prefill; PD_ERR_KV_CAPACITY if any listed slot is full (checked before anything is
 * enqueued).
 * Under graph capture: the launch grids (how the cached keys are divided over workers, whether a merge
 * launch is needed) are chosen from the slot lengths at the time of the call, and the library's host
 * record of those lengths advances at the call, not at a replay.  A captured step is therefore
 * replayed only with the lengths it was captured at: set them back with pd_kv_cache_set_lens before
 * each replay. */
pd_status pd_decode_step(pd_layer *layer, const pd_batch *batch, pd_kv_cache *cache,
                         void *out_hidden, void *stream);

/*
 * pd_decode_step for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The same step with the same kernels, but
 * every intermediate buffer (normalised rows, projections, attention partial results, split-K
 * partial sums, routing tables) lies in one 64 MiB array of static device memory that every GPU
 * the library runs on holds until the process ends, instead of the layer's own workspace.  The call
 * makes no hipMalloc / hipFree (nor any allocating library call) and needs no pd_layer_reserve;
 * the layer's workspace, if it has one, is left as it was.
 * Limits: the step's scratch need grows with the batch and the layer's widths; a call that needs
 * more than the 64 MiB returns PD_ERR_SHAPE and enqueues nothing (the 8B-shaped dense bf16 layer
 * fits up to batch 256).  The layer's device must be the current device.  No per-kernel events are
 * recorded.  Every call on one GPU shares that GPU's array: nothing in it has to start at zero
 * (each region is written before it is read within a step), but two such calls that overlap in
 * time on one GPU (different streams or threads) race, and so does a call that overlaps a replay of
 * a graph captured from one.
 * Arguments, state changes and all other errors as pd_decode_step.
 */
pd_status pd_decode_step_noalloc(pd_layer *layer, const pd_batch *batch, pd_kv_cache *cache,
                                 void *out_hidden, void *stream);

/* MoE only: device-to-device copy of the experts chosen by the last call on this layer, int32
 * [rows, top_k], into `expert_idx` (device).  Enqueued on `stream`. */
pd_status pd_last_expert_choice(const pd_layer *layer, int32_t rows, void *expert_idx, void *stream);

/*
 * Optional per-kernel timing, for roofline accounting of the individual steps of the layer.
 * While enabled, pd_prefill / pd_decode_step bracket every step they enqueue with events on the
 * caller's stream.  pd_profile_read waits for the last call's events and returns up to
 * max_entries (name, milliseconds) pairs in launch order; names are static strings owned by the
 * library ("qkv_proj", "gate_up_swiglu", "decode_attention", ...).
 */
pd_status pd_profile_enable(pd_layer *layer, int32_t on);
pd_status pd_profile_read(pd_layer *layer, int32_t max_entries, const char **names, float *ms,
                          int32_t *n);

/*
 * Plain device-to-device copy of `bytes` bytes (a multiple of 16; both pointers 16-byte aligned,
 * non-overlapping) as one grid-stride kernel on `stream`.  A measurement aid, not a step of the
 * layer: a kernel with exactly known HBM traffic (bytes read + bytes written) against which
 * hardware traffic counters and the streaming ceiling of the device are calibrated.
 * Errors: PD_ERR_INVALID_ARG for NULL / misaligned / bytes <= 0.
 */
pd_status pd_stream_copy(void *dst, const void *src, int64_t bytes, void *stream);

/*
 * The other measurement aid: the matrix pipe alone on given operand values.  n_workgroups workgroups
 * of 8 waves load their operands once - lane t of a workgroup takes a_vals[32 t .. 32 t + 31] (four
 * A fragments) and b_vals[16 t .. 16 t + 15] (two B fragments), bf16 device arrays of 16384 and 8192
 * elements, 16-byte aligned - and then issue iters x 8 v_mfma_f32_32x32x16_bf16 per wave with no
 * memory traffic: 2 * 32 * 32 * 16 * 8 * iters * 8 * n_workgroups flops.  The time of this launch is
 * the ceiling that operand values of that distribution allow the prefill GEMMs (Introduction:
 * prefill is compute-bound), whatever feeds the matrix pipe.  sink: device fp32 [n_workgroups * 512],
 * written once at the end.  Asynchronous on stream.
 * Errors: PD_ERR_INVALID_ARG (NULL / misaligned pointer, n_workgroups outside 1 .. 65536, iters < 1).
 */
pd_status pd_mfma_probe(const void *a_vals, const void *b_vals, int32_t n_workgroups, int32_t iters,
                        float *sink, void *stream);

/*
 * The two ends of the decoder stack around the layers (the paper's measured throughputs are those
 * of whole served models; Section "Acquire ... throughput" times them end to end): the token
 * embedding in front and, behind the last layer, the final RMSNorm and the vocabulary projection.
 *   pd_embed:    hidden[t, :] = w_embed[token_ids[t], :]
 *   pd_lm_head:  logits[t, :] = RMSNorm(hidden[t, :]; g_final, rms_eps) . w_lm^T      (no bias)
 * pd_head_create copies (and for bf16 repacks) g_final [d_model], w_lm [vocab, d_model] and, when
 * given, w_embed [vocab, d_model] (device pointers, row-major, `dtype` elements; w_embed may be
 * NULL if pd_embed is not used, and may equal w_lm for tied weights) into memory the handle owns,
 * plus a workspace for max_rows normalised rows, so the two calls allocate nothing and only
 * enqueue on `stream`.  token_ids is a DEVICE array of T int32; an id outside 0 .. vocab-1 yields
 * a row of zeros (checked in the kernel; ids never index outside the table).  hidden and logits
 * are device tensors [T, d_model] and [T, vocab] in `dtype`; T = 0 is a no-op.
 * Errors: PD_ERR_INVALID_ARG (NULL, T < 0, T > max_rows for pd_lm_head, pd_embed without
 * w_embed), PD_ERR_SHAPE (non-positive sizes), PD_ERR_DTYPE, PD_ERR_OOM, PD_ERR_DEVICE.
 */
typedef struct pd_head pd_head; /* opaque */
pd_status pd_head_create(int32_t d_model, int32_t vocab, float rms_eps, pd_dtype dtype,
                         const void *g_final, const void *w_embed, const void *w_lm,
                         int32_t max_rows, pd_head **out);

/*
 * The same head with the vocabulary projection held as 8-bit weights exactly like a layer's
 * projections in pd_layer_create_w8 (E4M3 codes, one power-of-two scale per vocabulary row;
 * pd_lm_head streams the codes for calls of up to 128 rows and uses a bf16 copy of the quantised
 * weights above that); the embedding table is kept as given.
 * Errors: as pd_head_create, plus PD_ERR_DTYPE unless dtype is bf16, d_model a multiple of 64 and
 * vocab a multiple of 16.
 */
pd_status pd_head_create_w8(int32_t d_model, int32_t vocab, float rms_eps, pd_dtype dtype,
                         const void *g_final, const void *w_embed, const void *w_lm,
                         int32_t max_rows, pd_head **out);
void pd_head_destroy(pd_head *head);
pd_status pd_embed(pd_head *head, const int32_t *token_ids, int32_t T, void *hidden, void *stream);
pd_status pd_lm_head(pd_head *head, const void *hidden, int32_t T, void *logits, void *stream);

/*
 * Allocation model (host only; needs no GPU).
 *   T_s        = ttft_slo - t_overhead                                         Eq. (12)
 *   TP_prefill = prefill_max_tps - l_in / T_s                                  Eq. (13)
 *   b*         = largest measured batch with TPOT <= tpot_slo (duplicates of a batch keep their
 *                smallest TPOT), TP_decode = b* / TPOT(b*)
 *   N_prefill  = (tp_total l_in)  / ((l_in + l_out) TP_prefill)                Eq. (5)
 *   N_decode   = (tp_total l_out) / ((l_in + l_out) TP_decode)                 Eq. (6)
 *   R          = (l_in TP_decode) / (l_out TP_prefill)                         Eq. (7)
 * evaluated in IEEE double in exactly this order and parenthesisation.
 * Integer counts: rounding 0 = max(1, floor(N + 0.5)) (reproduces the paper's worked example),
 * rounding 1 = max(1, ceil(N)).
 */
typedef struct {
    double prefill_max_tps;       /* measured maximum prefill tokens/s of one instance at this l_in */
    int32_t n_decode;             /* points on the measured TPOT-versus-batch curve */
    const int32_t *decode_batch;  /* host [n_decode], > 0, any order */
    const double *decode_tpot_s;  /* host [n_decode], > 0 */
    double t_overhead_s;          /* Eq. (8) overhead term, >= 0 */
    int32_t rounding;             /* 0 nearest (half up), 1 ceiling */
} pd_measured_curves;

typedef struct {
    double tp_prefill_eff, tp_decode_eff;
    int32_t decode_batch;
    double decode_tpot_s;
    double n_prefill_real, n_decode_real, ratio_pd;
    int32_t n_prefill, n_decode;
    int32_t curve_non_monotone;   /* 1 if TPOT does not increase with batch somewhere (warning only) */
} pd_allocation;

/*
 * Errors: PD_ERR_INVALID_ARG (NULL, non-finite or non-positive input, empty or malformed curve),
 * PD_ERR_TTFT_INFEASIBLE (T_s <= 0 or Eq. (13) <= 0), PD_ERR_TPOT_INFEASIBLE (no point meets the
 * target).  *out is untouched on error.
 */
pd_status pd_allocate(double tp_total_tps, double l_in, double l_out, double ttft_slo_s,
                      double tpot_slo_s, const pd_measured_curves *curves, pd_allocation *out);

/*
 * Eqs. (5), (6) for any number of independently deployed pipeline stages (host only; the paper's
 * conclusion names encode / prefill / decode disaggregation as the generalisation).  Requests
 * arrive at tp_total_tps / (l_in + l_out) per second (Eq. (1)); stage k does work_per_request[k]
 * units per request at stage_tps[k] units per second per instance (already SLO-constrained, e.g.
 * Eq. (13) for prefill), and every stage takes the same time (Eq. (4)):
 *   n_real[k] = (tp_total_tps * work_per_request[k]) / ((l_in + l_out) * stage_tps[k]),
 * n_instances[k] rounded as in pd_allocate.  With the stages (l_in, TP_prefill), (l_out, TP_decode)
 * this is exactly pd_allocate's pair of counts.  All arrays are host [n_stages].
 * Errors: PD_ERR_INVALID_ARG; outputs untouched on error.
 */
pd_status pd_allocate_stages(int32_t n_stages, double tp_total_tps, double l_in, double l_out,
                             const double *work_per_request, const double *stage_tps, int32_t rounding,
                             double *n_real, int32_t *n_instances);

/*
 * Queue check helpers (host only).  pd_fifo_replay serves n requests in arrival order on one
 * server in virtual time, D_i = max(A_i, D_{i-1}) + S_i, and writes each request's sojourn time
 * D_i - A_i (the queueing + computation part of TTFT, Eq. (8)).  pd_mm1_sojourn is Eq. (12),
 * 1 / (mu - lambda) with mu = prefill_max_tps / l_in (Eq. (9)); PD_ERR_TTFT_INFEASIBLE when
 * lambda >= mu.
 */
pd_status pd_fifo_replay(int32_t n, const double *arrival_s, const double *service_s,
                         double *sojourn_s);
pd_status pd_mm1_sojourn(double prefill_max_tps, double l_in, double lambda_rps, double *t_s);

/*
 * Queue-model variants (host only).
 * pd_fifo_replay_batched: one server that, whenever it becomes free, takes the first
 * min(max_batch, waiting) requests of the FIFO queue and serves them together in
 * batch_service_s[b-1] seconds (host [max_batch]; equal-length requests); every request of a batch
 * completes at the batch's end; an idle server starts as soon as one request is present.  This is
 * the regime the paper describes for a chunked prefill size much larger than the request length
 * (section "Acquire prefill throughput under TTFT constraints").  Writes each request's sojourn
 * time in arrival order.  max_batch = 1 is pd_fifo_replay with a constant service time.
 * pd_prefill_throughput_dp: Eq. (13) with prefill-side data parallelism, each of dp_groups groups
 * its own M/M/1 queue with 1/dp_groups of the maximum throughput and of the arrivals (the remark
 * under Eq. (8)): dp_groups * (prefill_max_tps / dp_groups - l_in / (ttft_slo_s - t_overhead_s)).
 * pd_mg1_sojourn: the Pollaczek-Khinchine mean sojourn time E[S] + lambda E[S^2] / (2 (1 - rho)),
 * context beside Eq. (12) for service times that are not exponential (not part of the paper).
 * Errors: PD_ERR_INVALID_ARG; PD_ERR_TTFT_INFEASIBLE where no stable queue / positive throughput
 * exists.  Outputs untouched on error.
 */
pd_status pd_fifo_replay_batched(int32_t n, const double *arrival_s, int32_t max_batch,
                                 const double *batch_service_s, double *sojourn_s);
pd_status pd_prefill_throughput_dp(double prefill_max_tps, double l_in, double ttft_slo_s,
                                   double t_overhead_s, int32_t dp_groups, double *tp_prefill);
pd_status pd_mg1_sojourn(double lambda_rps, double mean_service_s, double mean_service_sq_s2,
                         double *t_s);

/*
 * The overhead term of Eq. (8) as a model instead of a given scalar (host only).  The paper names
 * its parts: the request's input / output transmission between the user and the server, and the
 * transmission of the KV cache from the prefill to the decode instance.  Here
 *   t_overhead = fixed_s + l_in * n_layers * 2 * n_kv_heads * head_dim * bytes_per_elem / link_bytes_per_s
 * (the keys and values of all l_in prompt tokens of every layer cross one link of the given rate;
 * fixed_s holds everything that does not grow with the prompt: user-side transmission, connection
 * set-up).  bytes_per_elem is 2 for a bf16 cache, 1 for the 8-bit one; l_in may be fractional
 * (a mean).  The result is what pd_measured_curves.t_overhead_s takes.
 * Errors: PD_ERR_INVALID_ARG (NULL, negative or non-finite values, non-positive sizes or rate);
 * output untouched on error.
 */
pd_status pd_kv_transfer_overhead(double l_in, int32_t n_layers, int32_t n_kv_heads, int32_t head_dim,
                                  double bytes_per_elem, double link_bytes_per_s, double fixed_s,
                                  double *t_overhead_s);

const char *pd_status_string(pd_status s);
const char *pd_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PD_H */
