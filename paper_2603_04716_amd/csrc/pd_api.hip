// C-ABI entry points that touch the device: layer and KV-cache handles, pd_prefill and
// pd_decode_step.  Each call validates on the host, then enqueues the layer's kernels on the
// caller's stream in the order of the layer definition in pd.h.
#include <math.h>
#include <cmath>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <vector>

#include "pd_internal.h"

using namespace pd;

struct pd_layer {
    pd_layer_config cfg;
    int device;
    size_t esz;
    int Nq, Nkv, Nqkv;
    bool use_mfma;       // bf16 layer whose shapes fit the MFMA kernels
    bool packed;         // weights stored in the matrix-core block layout (gate/up as one interleaved pack)
    void *g_attn, *g_ffn, *w_qkv, *w_o, *w_gate, *w_up, *w_down, *w_router;
    // 8-bit weights: E4M3 codes of the four packed matrices (for the skinny kernel) and one
    // power-of-two scale per packed row; the bf16 packs above then hold scale * value(code)
    bool w8;
    void *q_qkv, *q_o, *q_gate, *q_down;
    float *s_qkv, *s_o, *s_gate, *s_down;
    // 8-bit activations on top of 8-bit weights: projections called with more than 256 rows quantise
    // their input rows and multiply codes by codes; t_* are the weight codes in the tiled kernel's pack
    bool a8;
    void *t_qkv, *t_o, *t_gate, *t_down;
    uint8_t *a8_codes;        // [ws_tokens * top_k][max K] activation codes (inside ws)
    float *a8_scales;         // [ws_tokens * top_k]
    mutable const void *a8_src;   // the buffer whose (unwritten) rows a8_codes already encode: set by a fused
                                  // norm + quantisation, consumed by the projection that follows
    double *inv_freq;
    float2 *rope_table;       // (cos, sin) for positions < kRopeTableLen
    int32_t *d_cu, *d_slots, *d_pad_cu, *d_prefix;  // [4097] each
    int32_t *units;           // [4][ws_tokens]: slot, first position, first row, token count of multi-token units
    void *vt;                 // transposed-V scratch for the MFMA attention, vt_cap bytes
    size_t vt_cap;
    float *dec_part;          // partial outputs of the decode attention chunks (inside ws)
    int chunk_slack_workers;  // the partial-output part holds batch + this many workers' chunks (see decode_chunk_bound)
    float *splitk;            // split-K partials of the decode-sized GEMMs (inside ws)
    size_t splitk_elems;
    // workspace, sized for ws_tokens rows
    int ws_tokens;
    char *ws;
    void *y, *qkv, *o, *h, *act, *eo;
    int32_t *tok_seq, *tok_pos, *tok_slot, *eidx, *sorted_token, *pair_pos, *offsets, *chunk_cu, *chunk_seq, *block_hist;
    float *logits, *ew;
    int last_rows;
    int call_rows;            // rows of the call in progress (T of a prefill, B of a decode step)
    // optional per-kernel timing of the last call
    bool prof_on;
    std::vector<hipEvent_t> prof_ev;          // pairs (start, stop)
    std::vector<const char *> prof_names;     // one per recorded pair
};

struct pd_kv_cache {
    int dtype, Hkv, hd, max_seqs, max_len;
    int blocked;       // bf16 / head_dim 128: blocked layout for the matrix-core decode attention
    int plane_len;     // positions per (slot, kv head) plane: max_len, or padded to 64 when blocked
    int fp8;           // elements are 8-bit E4M3 codes of x / scale (blocked 8-bit layout)
    double k_scale, v_scale;
    void *k, *v;
    int32_t *d_len;
    std::vector<int32_t> h_len;
};

static const int kMaxSeqs = 4096;
// a layer with 8-bit activations quantises the input of a projection when the call has more rows than this
static const int kA8Rows = 256;
// Work split of the decode attention: a sequence of n keys is cut into ceil(n / chunk_keys) equal
// chunks, one wavefront-sized worker per (chunk, kv head).  Two measured effects set chunk_keys
// (8B shape, 2048 .. 16384 keys, batch 4 .. 256, both cache formats):
//  - a lone worker streams about 13 GB/s, so some 500 workers saturate the memory system; beyond
//    that the time is the bytes moved and more, smaller chunks only add start-up and merge work.
//    Best for equal lengths: about kDecodeWorkers workers, one chunk per sequence from there on.
//  - all workers start together, so with ragged lengths the short ones finish first and the few
//    long ones left run latency-bound: a tail.  Chunks of at most mean^2 / max keys (the mean
//    length shrunk by how far the longest sequence sticks out; equal lengths: no limit) keep
//    enough equal workers running to the end: 10 - 30 % faster from batch 64 up on log-normal
//    lengths with mean 3 k and maximum 8 k.
// max_chunks: what the partial-output workspace holds; the chunk size is raised until the step fits
// (one chunk per sequence always does).
static const int kDecodeWorkers = 768;
// Workers (chunk x kv head) beyond one per sequence that the partial-output buffer of a layer's own
// workspace leaves room for, and what the static scratch of pd_decode_step_noalloc leaves room for
// (the work split asks for at most about 1536 workers beyond one chunk per sequence).
static const int kChunkSlackWorkers = 8192, kChunkSlackWorkersStatic = 2048;

static int pick_chunk_keys(const std::vector<int32_t> &keys, int n_kv_heads, size_t max_chunks)
{
    long long total = 0;
    int max_k = 1;
    for (int32_t k : keys) {
        total += k;
        max_k = std::max(max_k, (int)k);
    }
    const double mean = keys.empty() ? 1.0 : (double)total / (double)keys.size();
    const long long by_workers = (total * n_kv_heads + kDecodeWorkers - 1) / kDecodeWorkers;
    const long long by_tail = (long long)(mean * mean / (double)max_k) + 1;
    long long ck = (std::min(by_workers, by_tail) + 63) / 64 * 64;
    if (ck < 64) ck = 64;
    const long long whole = ((long long)max_k + 63) / 64 * 64;
    if (ck > whole) ck = whole;
    auto chunks = [&](long long c) {
        size_t n = 0;
        for (int32_t k : keys) n += (size_t)((k + c - 1) / c);
        return n;
    };
    // A launch holds one 4-wave workgroup per CU up to 1024 workers.  A little above that a few CUs
    // carry two workgroups, which then run about 1.5 times as long and everything waits for them
    // (measured at 8192 keys: 6.0 us per sequence at 1024 workers, 7.6 at 1040, back to 5.9 from
    // 1536 on, where the dispatcher has enough workgroups to even the load out).  Cut finer to get
    // out of that range.
    {
        const long long w = (long long)chunks(ck) * n_kv_heads;
        if (w > 1024 && w < 1536 && ck > 64) {
            long long finer = ck * w / 1536 / 64 * 64;
            if (finer < 64) finer = 64;
            while (finer > 64 && (long long)chunks(finer) * n_kv_heads < 1536) finer -= 64;
            ck = finer;
        }
    }
    while (ck < whole && chunks(ck) > max_chunks) ck = std::min(whole, 2 * ck);
    return (int)ck;
}

static const int kShortChunk = 8;   // chunks up to this many tokens use the decode attention kernel per row
static const int kRopeTableLen = 32768;   // positions with precomputed rotary factors

#define HIP_TRY(expr, status)                                                        \
    do {                                                                             \
        hipError_t e__ = (expr);                                                     \
        if (e__ != hipSuccess) {                                                     \
            set_error("%s failed: %s", #expr, hipGetErrorString(e__));               \
            return (e__ == hipErrorOutOfMemory) ? PD_ERR_OOM : (status);             \
        }                                                                            \
    } while (0)

static void prof_begin(pd_layer *L, const char *name, hipStream_t s)
{
    if (!L->prof_on) return;
    const size_t i = L->prof_names.size();
    while (L->prof_ev.size() < 2 * (i + 1)) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return;
        L->prof_ev.push_back(e);
    }
    L->prof_names.push_back(name);
    (void)hipEventRecord(L->prof_ev[2 * i], s);
}
static void prof_end(pd_layer *L, hipStream_t s)
{
    if (!L->prof_on || L->prof_names.empty()) return;
    (void)hipEventRecord(L->prof_ev[2 * L->prof_names.size() - 1], s);
}
#define STEP(name, expr)                 \
    do {                                 \
        prof_begin(L, name, s);          \
        HIP_TRY(expr, PD_ERR_DEVICE);    \
        prof_end(L, s);                  \
    } while (0)

static size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

// Packs a [n_rows, K] bf16 weight matrix into the block layout of wpack_off (one 16-byte chunk per
// thread).  With `up` != nullptr the packed rows are the 32-row interleave gate[j..j+31],
// up[j..j+31], ... of two [n_rows/2, K] matrices.
__global__ void pack_weight_kernel(uint4 *dst, const uint4 *src, const uint4 *up, int n_rows, int K)
{
    const size_t n_chunks = (size_t)n_rows * (K >> 3);
    const int row_vec = K >> 3;
    for (size_t c = (size_t)blockIdx.x * blockDim.x + threadIdx.x; c < n_chunks;
         c += (size_t)gridDim.x * blockDim.x) {
        const size_t block = c >> 6;
        const int kg = (int)(c >> 4) & 3, r = (int)c & 15;
        const int rb = (int)(block / (K >> 5)), kb = (int)(block % (K >> 5));
        const int n = rb * 16 + r, k8 = kb * 4 + kg;          // packed row, 8-element k chunk
        const uint4 *from = src;
        int row = n;
        if (up) {
            const int q = n >> 6, w = n & 63;
            row = q * 32 + (w & 31);
            if (w >= 32) from = up;
        }
        dst[c] = from[(size_t)row * row_vec + k8];
    }
}

// Per packed row n of a [n_rows, K] bf16 matrix (row mapping as in pack_weight_kernel): the smallest
// power of two s with max_k |w[n, k]| / s <= 448, the largest E4M3 value (1 for a row of zeros).
// One wavefront per row.
__global__ __launch_bounds__(256) void w8_row_scale_kernel(float *scale, const uint16_t *src, const uint16_t *up,
                                                           int n_rows, int K)
{
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (n >= n_rows) return;
    const uint16_t *from = src;
    int row = n;
    if (up) {
        const int q = n >> 6, w = n & 63;
        row = q * 32 + (w & 31);
        if (w >= 32) from = up;
    }
    const uint16_t *p = from + (size_t)row * K;
    float m = 0.f;
    for (int k = lane; k < K; k += 64) m = fmaxf(m, fabsf(bfbits2f(p[k])));
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if (lane == 0) {
        float s = 1.f;
        if (m > 0.f && m < INFINITY) {
            int e;
            const double f = frexp((double)m / 448.0, &e);    // m / 448 = f * 2^e, f in [0.5, 1)
            s = (float)ldexp(1.0, f == 0.5 ? e - 1 : e);
        }
        scale[n] = s;
    }
}

// Quantises and packs in one pass: per 8-element chunk of packed row n, the E4M3 codes of w / scale[n]
// into the 8-bit layout and scale[n] * value(code) as bf16 into the block layout of wpack_off.
__global__ void pack_weight_w8_kernel(uint4 *dst, uint8_t *dst8, const uint4 *src, const uint4 *up,
                                      const float *scale, int n_rows, int K)
{
    const size_t n_chunks = (size_t)n_rows * (K >> 3);
    const int row_vec = K >> 3;
    for (size_t c = (size_t)blockIdx.x * blockDim.x + threadIdx.x; c < n_chunks;
         c += (size_t)gridDim.x * blockDim.x) {
        const size_t block = c >> 6;
        const int kg = (int)(c >> 4) & 3, r = (int)c & 15;
        const int rb = (int)(block / (K >> 5)), kb = (int)(block % (K >> 5));
        const int n = rb * 16 + r, k8 = kb * 4 + kg;
        const uint4 *from = src;
        int row = n;
        if (up) {
            const int q = n >> 6, w = n & 63;
            row = q * 32 + (w & 31);
            if (w >= 32) from = up;
        }
        const uint4 v = from[(size_t)row * row_vec + k8];
        const uint32_t w32[4] = {v.x, v.y, v.z, v.w};
        const double s = (double)scale[n];
        uint32_t code[8], outw[4];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t bits = (w32[j >> 1] >> (16 * (j & 1))) & 0xffffu;
            code[j] = e4m3_encode((double)bfbits2f(bits) / s);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
            outw[j] = pack2bf((float)(s * (double)e4m3_decode(code[2 * j])),
                              (float)(s * (double)e4m3_decode(code[2 * j + 1])));
        dst[c] = make_uint4(outw[0], outw[1], outw[2], outw[3]);
        uint2 q8;
        q8.x = code[0] | (code[1] << 8) | (code[2] << 16) | (code[3] << 24);
        q8.y = code[4] | (code[5] << 8) | (code[6] << 16) | (code[7] << 24);
        *(uint2 *)(dst8 + w8pack_off(n, k8 * 8, K)) = q8;
    }
}

static void free_layer(pd_layer *L)
{
    if (!L) return;
    void *ptrs[] = {L->q_qkv, L->q_o, L->q_gate, L->q_down, L->s_qkv, L->s_o, L->s_gate, L->s_down,
                    L->t_qkv, L->t_o, L->t_gate, L->t_down,
                    L->g_attn, L->g_ffn, L->w_qkv, L->w_o, L->w_gate, L->w_up, L->w_down,
                    L->w_router, L->inv_freq, L->rope_table, L->d_cu, L->d_slots, L->d_pad_cu, L->d_prefix, L->vt, L->ws};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    for (hipEvent_t e : L->prof_ev) (void)hipEventDestroy(e);
    delete L;
}

static pd_status layer_create(const pd_layer_config *cfg, const pd_layer_weights *w, bool w8, bool a8,
                              pd_layer **out);

extern "C" pd_status pd_layer_create(const pd_layer_config *cfg, const pd_layer_weights *w,
                                     pd_layer **out)
{
    return layer_create(cfg, w, false, false, out);
}

extern "C" pd_status pd_layer_create_w8(const pd_layer_config *cfg, const pd_layer_weights *w,
                                        pd_layer **out)
{
    return layer_create(cfg, w, true, false, out);
}

extern "C" pd_status pd_layer_create_w8a8(const pd_layer_config *cfg, const pd_layer_weights *w,
                                          pd_layer **out)
{
    return layer_create(cfg, w, true, true, out);
}

static pd_status layer_create(const pd_layer_config *cfg, const pd_layer_weights *w, bool w8, bool a8,
                              pd_layer **out)
{
    if (!cfg || !w || !out) {
        set_error("pd_layer_create: NULL argument");
        return PD_ERR_INVALID_ARG;
    }
    if (cfg->dtype != PD_F32 && cfg->dtype != PD_BF16) {
        set_error("pd_layer_create: dtype %d is neither fp32 nor bf16", cfg->dtype);
        return PD_ERR_DTYPE;
    }
    const int d = cfg->d_model, Hq = cfg->n_q_heads, Hkv = cfg->n_kv_heads, hd = cfg->head_dim,
              F = cfg->d_ff, E = cfg->n_experts;
    if (d <= 0 || Hq <= 0 || Hkv <= 0 || hd <= 0 || F <= 0 || E < 0 || (hd & 1) || hd > 256 ||
        Hq % Hkv != 0 || E > 64 || (E > 0 && (cfg->top_k <= 0 || cfg->top_k > E || cfg->top_k > 8)) ||
        !(cfg->rms_eps >= 0.f) || !(cfg->rope_base > 0.f)) {
        set_error("pd_layer_create: unsupported shape (d=%d Hq=%d Hkv=%d hd=%d F=%d E=%d top_k=%d)", d,
                  Hq, Hkv, hd, F, E, cfg->top_k);
        return PD_ERR_SHAPE;
    }
    if (!w->g_attn || !w->w_q || !w->w_k || !w->w_v || !w->w_o || !w->g_ffn || !w->w_gate ||
        !w->w_up || !w->w_down) {
        set_error("pd_layer_create: a weight pointer is NULL");
        return PD_ERR_INVALID_ARG;
    }
    pd_layer *L = new pd_layer();   // value-initialised: every pointer and counter starts at zero
    L->cfg = *cfg;
    L->esz = cfg->dtype == PD_F32 ? 4 : 2;
    L->Nq = Hq * hd;
    L->Nkv = Hkv * hd;
    L->Nqkv = L->Nq + 2 * L->Nkv;
    L->use_mfma = cfg->dtype == PD_BF16 && d % 64 == 0 && F % 64 == 0 && L->Nq % 64 == 0 &&
                  L->Nkv % 64 == 0;
    L->packed = L->use_mfma;
    L->w8 = w8;
    L->a8 = a8;
    L->chunk_slack_workers = kChunkSlackWorkers;
    if (w8 && !L->use_mfma) {
        set_error("pd_layer_create_w8: needs a bf16 layer whose dimensions are multiples of 64");
        delete L;
        return PD_ERR_DTYPE;
    }
    if (a8 && (d % 128 != 0 || F % 128 != 0 || L->Nq % 128 != 0)) {
        set_error("pd_layer_create_w8a8: needs a layer whose dimensions are multiples of 128");
        delete L;
        return PD_ERR_DTYPE;
    }
    const size_t esz = L->esz;
    const int G = E > 0 ? E : 1;
    pd_status st = PD_OK;
    auto fail = [&](pd_status s) {
        free_layer(L);
        return s;
    };
#define CREATE_TRY(expr)                                                               \
    do {                                                                               \
        hipError_t e__ = (expr);                                                       \
        if (e__ != hipSuccess) {                                                       \
            set_error("pd_layer_create: %s failed: %s", #expr, hipGetErrorString(e__)); \
            return fail(e__ == hipErrorOutOfMemory ? PD_ERR_OOM : PD_ERR_DEVICE);      \
        }                                                                              \
    } while (0)
    CREATE_TRY(hipGetDevice(&L->device));
    CREATE_TRY(hipMalloc(&L->g_attn, d * esz));
    CREATE_TRY(hipMalloc(&L->g_ffn, d * esz));
    CREATE_TRY(hipMalloc(&L->w_qkv, (size_t)L->Nqkv * d * esz));
    CREATE_TRY(hipMalloc(&L->w_o, (size_t)d * L->Nq * esz));
    CREATE_TRY(hipMalloc(&L->w_down, (size_t)G * d * F * esz));
    CREATE_TRY(hipMalloc(&L->inv_freq, sizeof(double) * (hd / 2)));
    CREATE_TRY(hipMalloc(&L->d_cu, sizeof(int32_t) * (kMaxSeqs + 1)));
    CREATE_TRY(hipMalloc(&L->d_slots, sizeof(int32_t) * (kMaxSeqs + 1)));
    CREATE_TRY(hipMalloc(&L->d_pad_cu, sizeof(int32_t) * (kMaxSeqs + 1)));
    CREATE_TRY(hipMalloc(&L->d_prefix, sizeof(int32_t) * (kMaxSeqs + 1)));
    CREATE_TRY(hipMemcpy(L->g_attn, w->g_attn, d * esz, hipMemcpyDeviceToDevice));
    CREATE_TRY(hipMemcpy(L->g_ffn, w->g_ffn, d * esz, hipMemcpyDeviceToDevice));
    if (L->packed) {
        // packs one [n_rows, K] matrix (gate/up interleaved when up != nullptr); for 8-bit weights
        // also its row scales and codes, the bf16 pack then holding the dequantised values
        auto pack = [&](void *dst, const void *src, const void *up, int n_rows, int K, void *dst8,
                        float *scale) -> hipError_t {
            if (w8) {
                w8_row_scale_kernel<<<(n_rows + 3) / 4, 256>>>(scale, (const uint16_t *)src, (const uint16_t *)up, n_rows, K);
                hipError_t e = hipGetLastError();
                if (e != hipSuccess) return e;
                pack_weight_w8_kernel<<<2048, 256>>>((uint4 *)dst, (uint8_t *)dst8, (const uint4 *)src,
                                                     (const uint4 *)up, scale, n_rows, K);
            } else {
                pack_weight_kernel<<<2048, 256>>>((uint4 *)dst, (const uint4 *)src, (const uint4 *)up, n_rows, K);
            }
            return hipGetLastError();
        };
        if (w8) {
            CREATE_TRY(hipMalloc(&L->q_qkv, (size_t)L->Nqkv * d));
            CREATE_TRY(hipMalloc(&L->q_o, (size_t)d * L->Nq));
            CREATE_TRY(hipMalloc(&L->q_gate, (size_t)G * 2 * F * d));
            CREATE_TRY(hipMalloc(&L->q_down, (size_t)G * d * F));
            CREATE_TRY(hipMalloc((void **)&L->s_qkv, sizeof(float) * L->Nqkv));
            CREATE_TRY(hipMalloc((void **)&L->s_o, sizeof(float) * d));
            CREATE_TRY(hipMalloc((void **)&L->s_gate, sizeof(float) * (size_t)G * 2 * F));
            CREATE_TRY(hipMalloc((void **)&L->s_down, sizeof(float) * (size_t)G * d));
        }
        // stack q|k|v plainly in a temporary, then pack every matrix into the block layout
        void *tmp = nullptr;
        CREATE_TRY(hipMalloc(&tmp, (size_t)L->Nqkv * d * esz));
        hipError_t e1 = hipMemcpy(tmp, w->w_q, (size_t)L->Nq * d * esz, hipMemcpyDeviceToDevice);
        if (e1 == hipSuccess)
            e1 = hipMemcpy((char *)tmp + (size_t)L->Nq * d * esz, w->w_k, (size_t)L->Nkv * d * esz, hipMemcpyDeviceToDevice);
        if (e1 == hipSuccess)
            e1 = hipMemcpy((char *)tmp + (size_t)(L->Nq + L->Nkv) * d * esz, w->w_v, (size_t)L->Nkv * d * esz, hipMemcpyDeviceToDevice);
        if (e1 == hipSuccess) e1 = pack(L->w_qkv, tmp, nullptr, L->Nqkv, d, L->q_qkv, L->s_qkv);
        if (e1 == hipSuccess) e1 = hipDeviceSynchronize();
        (void)hipFree(tmp);
        CREATE_TRY(e1);
        CREATE_TRY(pack(L->w_o, w->w_o, nullptr, d, L->Nq, L->q_o, L->s_o));
        CREATE_TRY(hipMalloc(&L->w_gate, (size_t)G * 2 * F * d * esz));
        for (int g = 0; g < G; ++g) {
            CREATE_TRY(pack((char *)L->w_gate + (size_t)g * 2 * F * d * esz,
                            (const char *)w->w_gate + (size_t)g * F * d * esz,
                            (const char *)w->w_up + (size_t)g * F * d * esz, 2 * F, d,
                            w8 ? (char *)L->q_gate + (size_t)g * 2 * F * d : nullptr,
                            w8 ? L->s_gate + (size_t)g * 2 * F : nullptr));
            CREATE_TRY(pack((char *)L->w_down + (size_t)g * d * F * esz,
                            (const char *)w->w_down + (size_t)g * d * F * esz, nullptr, d, F,
                            w8 ? (char *)L->q_down + (size_t)g * d * F : nullptr,
                            w8 ? L->s_down + (size_t)g * d : nullptr));
        }
        if (a8) {
            CREATE_TRY(hipMalloc(&L->t_qkv, (size_t)L->Nqkv * d));
            CREATE_TRY(hipMalloc(&L->t_o, (size_t)d * L->Nq));
            CREATE_TRY(hipMalloc(&L->t_gate, (size_t)G * 2 * F * d));
            CREATE_TRY(hipMalloc(&L->t_down, (size_t)G * d * F));
            CREATE_TRY(launch_repack_w8_tiles(L->q_qkv, L->t_qkv, L->Nqkv, d, nullptr));
            CREATE_TRY(launch_repack_w8_tiles(L->q_o, L->t_o, d, L->Nq, nullptr));
            for (int g = 0; g < G; ++g) {
                CREATE_TRY(launch_repack_w8_tiles((const char *)L->q_gate + (size_t)g * 2 * F * d,
                                                  (char *)L->t_gate + (size_t)g * 2 * F * d, 2 * F, d, nullptr));
                CREATE_TRY(launch_repack_w8_tiles((const char *)L->q_down + (size_t)g * d * F,
                                                  (char *)L->t_down + (size_t)g * d * F, d, F, nullptr));
            }
        }
    } else {
        CREATE_TRY(hipMemcpy(L->w_qkv, w->w_q, (size_t)L->Nq * d * esz, hipMemcpyDeviceToDevice));
        CREATE_TRY(hipMemcpy((char *)L->w_qkv + (size_t)L->Nq * d * esz, w->w_k,
                             (size_t)L->Nkv * d * esz, hipMemcpyDeviceToDevice));
        CREATE_TRY(hipMemcpy((char *)L->w_qkv + (size_t)(L->Nq + L->Nkv) * d * esz, w->w_v,
                             (size_t)L->Nkv * d * esz, hipMemcpyDeviceToDevice));
        CREATE_TRY(hipMemcpy(L->w_o, w->w_o, (size_t)d * L->Nq * esz, hipMemcpyDeviceToDevice));
        CREATE_TRY(hipMemcpy(L->w_down, w->w_down, (size_t)G * d * F * esz, hipMemcpyDeviceToDevice));
        CREATE_TRY(hipMalloc(&L->w_gate, (size_t)G * F * d * esz));
        CREATE_TRY(hipMalloc(&L->w_up, (size_t)G * F * d * esz));
        CREATE_TRY(hipMemcpy(L->w_gate, w->w_gate, (size_t)G * F * d * esz, hipMemcpyDeviceToDevice));
        CREATE_TRY(hipMemcpy(L->w_up, w->w_up, (size_t)G * F * d * esz, hipMemcpyDeviceToDevice));
    }
    if (E > 0 && w->w_router) {
        CREATE_TRY(hipMalloc(&L->w_router, (size_t)E * d * esz));
        CREATE_TRY(hipMemcpy(L->w_router, w->w_router, (size_t)E * d * esz, hipMemcpyDeviceToDevice));
    }
    {
        std::vector<double> f(hd / 2);
        for (int i = 0; i < hd / 2; ++i)
            f[i] = pow((double)cfg->rope_base, -2.0 * (double)i / (double)hd);
        CREATE_TRY(hipMemcpy(L->inv_freq, f.data(), sizeof(double) * f.size(), hipMemcpyHostToDevice));
    }
    CREATE_TRY(hipMalloc((void **)&L->rope_table, sizeof(float2) * (size_t)kRopeTableLen * (hd / 2)));
    CREATE_TRY(launch_rope_table(L->rope_table, kRopeTableLen, hd / 2, L->inv_freq, nullptr));
    CREATE_TRY(hipDeviceSynchronize());
#undef CREATE_TRY
    (void)st;
    *out = L;
    return PD_OK;
}

extern "C" void pd_layer_destroy(pd_layer *layer)
{
    if (!layer) return;
    (void)hipDeviceSynchronize();
    free_layer(layer);
}

// Chunks of one decode attention launch whose partial outputs the workspace holds (the chunk size
// is chosen so that a step fits), so a decode step never allocates.
static size_t decode_chunk_bound(const pd_layer *L, int batch)
{
    return (size_t)(L->chunk_slack_workers / L->cfg.n_kv_heads + 1) + (size_t)batch;
}

extern "C" pd_status pd_quantize_rows_e4m3(const void *x, int32_t n_rows, int32_t n_cols, void *codes,
                                           float *scales, void *stream)
{
    if (!x || !codes || !scales || n_rows < 0 || n_cols <= 0 || n_cols % 8 != 0) {
        set_error("pd_quantize_rows_e4m3: NULL argument, negative row count or a column count that is not a multiple of 8");
        return PD_ERR_INVALID_ARG;
    }
    HIP_TRY(launch_quant_rows_e4m3(x, n_cols, n_rows, n_cols, codes, scales, (hipStream_t)stream), PD_ERR_DEVICE);
    return PD_OK;
}

extern "C" pd_status pd_gemm_e4m3(const void *a_codes, const float *a_scales, const void *b_codes,
                                  const float *b_scales, int32_t M, int32_t N, int32_t K, void *c, void *stream)
{
    if (!a_codes || !a_scales || !b_codes || !b_scales || !c) {
        set_error("pd_gemm_e4m3: NULL argument");
        return PD_ERR_INVALID_ARG;
    }
    if (M < 1 || N < 16 || N % 16 != 0 || K < 128 || K % 128 != 0 || (int64_t)N * K >= (1ll << 32) ||
        (int64_t)M * K >= (1ll << 32)) {
        set_error("pd_gemm_e4m3: needs M >= 1, N a multiple of 16, K a multiple of 128 and operands below 4 GiB (M=%d N=%d K=%d)",
                  M, N, K);
        return PD_ERR_SHAPE;
    }
    hipStream_t s = (hipStream_t)stream;
    void *tiles = nullptr;
    float *ws = nullptr;
    const size_t ws_elems = (size_t)8 * 256 * N + (size_t)M * N;   // a few splits of mid-sized problems
    HIP_TRY(hipMalloc(&tiles, (size_t)N * K), PD_ERR_DEVICE);
    hipError_t e = hipMalloc((void **)&ws, ws_elems * sizeof(float));
    if (e == hipSuccess) e = launch_pack_rows_e4m3_tiles(b_codes, tiles, N, K, s);
    if (e == hipSuccess) {
        GemmArgs g;
        memset(&g, 0, sizeof(g));
        g.A = a_codes; g.B = tiles; g.C = c; g.M = M; g.N = N; g.K = K / 2; g.lda = K / 2; g.ldb = K / 2; g.ldc = N;
        g.epilogue = EPI_NONE; g.packed = 1; g.n_groups = 1; g.a_scale = a_scales; g.b_scale = b_scales;
        g.splitk_ws = ws; g.splitk_ws_elems = ws_elems;
        e = gemm_mfma_f8_supported(g) ? launch_gemm_mfma_f8(g, s) : hipErrorInvalidValue;
    }
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    (void)hipFree(tiles);
    (void)hipFree(ws);
    HIP_TRY(e, PD_ERR_DEVICE);
    return PD_OK;
}

// Offsets of the parts of a workspace for calls of up to max_tokens rows, and its size.
struct WsLayout {
    size_t y, qkv, o, h, act, eo, seq, pos, slot, eidx, sorted, pp, off, bh, log, ew, ccu, cseq, units, part, sk, a8c, a8s;
    size_t sk_elems;
    size_t total;
};

// sk_rows: rows the split-K scratch is sized for (a launcher whose partials would not fit takes fewer splits)
static WsLayout ws_layout(const pd_layer *L, int max_tokens, size_t sk_rows = 256, size_t sk_per_row = 0)
{
    const size_t T = (size_t)max_tokens, esz = L->esz;
    const int d = L->cfg.d_model, F = L->cfg.d_ff, E = L->cfg.n_experts;
    const size_t K = E > 0 ? (size_t)L->cfg.top_k : 1;
    WsLayout w;
    size_t off = 0;
    auto carve = [&](size_t bytes) {
        size_t o = off;
        off += align256(bytes);
        return o;
    };
    w.y = carve(T * d * esz); w.qkv = carve(T * L->Nqkv * esz); w.o = carve(T * L->Nq * esz);
    w.h = carve(T * d * esz); w.act = carve(T * K * F * esz);
    w.eo = carve(E > 0 ? T * K * d * esz : 0); w.seq = carve(T * 4); w.pos = carve(T * 4);
    w.slot = carve(T * 4); w.eidx = carve(T * K * 4); w.sorted = carve(T * K * 4);
    w.pp = carve(T * K * 4); w.off = carve(65 * 4 + 4); w.bh = carve(E > 0 ? (T * K / 256 + 1) * (size_t)E * 4 : 0);
    w.log = carve(T * (E > 0 ? E : 1) * 4);
    w.ew = carve(T * K * 4); w.ccu = carve((T + 1) * 4); w.cseq = carve(decode_chunk_bound(L, max_tokens) * 4);
    w.units = carve(4 * T * 4);
    w.part = carve(decode_chunk_bound(L, max_tokens) * L->cfg.n_q_heads * 130 * sizeof(float));
    // split-K scratch: splits * columns never exceeds 640 tiles * 128 columns + one row of tiles (a
    // launcher that would need more takes fewer splits)
    size_t maxn = (size_t)L->Nqkv;
    if ((size_t)2 * F > maxn) maxn = (size_t)2 * F;
    if ((size_t)d > maxn) maxn = (size_t)d;
    if (sk_per_row == 0) sk_per_row = 640 * 128 + 2 * maxn;
    w.sk_elems = L->use_mfma ? sk_rows * sk_per_row : 0;
    w.sk = carve(w.sk_elems * sizeof(float));
    size_t maxk = (size_t)d > (size_t)L->Nq ? (size_t)d : (size_t)L->Nq;
    if ((size_t)F > maxk) maxk = (size_t)F;
    w.a8c = carve(L->a8 ? T * K * maxk : 0);
    w.a8s = carve(L->a8 ? T * K * sizeof(float) : 0);
    w.total = off;
    return w;
}

// Points the layer's workspace members into base (a buffer of w.total bytes laid out for max_tokens rows).
static void ws_bind(pd_layer *L, char *nw, const WsLayout &w, int max_tokens)
{
    const int E = L->cfg.n_experts;
    L->ws_tokens = max_tokens;
    L->y = nw + w.y;
    L->qkv = nw + w.qkv;
    L->o = nw + w.o;
    L->h = nw + w.h;
    L->act = nw + w.act;
    L->eo = nw + w.eo;
    L->tok_seq = (int32_t *)(nw + w.seq);
    L->tok_pos = (int32_t *)(nw + w.pos);
    L->tok_slot = (int32_t *)(nw + w.slot);
    L->eidx = (int32_t *)(nw + w.eidx);
    L->sorted_token = (int32_t *)(nw + w.sorted);
    L->pair_pos = (int32_t *)(nw + w.pp);
    L->block_hist = E > 0 ? (int32_t *)(nw + w.bh) : nullptr;
    L->offsets = (int32_t *)(nw + w.off);
    L->logits = (float *)(nw + w.log);
    L->ew = (float *)(nw + w.ew);
    L->chunk_cu = (int32_t *)(nw + w.ccu);
    L->chunk_seq = (int32_t *)(nw + w.cseq);
    L->units = (int32_t *)(nw + w.units);
    L->dec_part = (float *)(nw + w.part);
    L->splitk = w.sk_elems ? (float *)(nw + w.sk) : nullptr;
    L->splitk_elems = w.sk_elems;
    L->a8_codes = L->a8 ? (uint8_t *)(nw + w.a8c) : nullptr;
    L->a8_scales = L->a8 ? (float *)(nw + w.a8s) : nullptr;
}

extern "C" pd_status pd_layer_reserve(pd_layer *L, int32_t max_tokens)
{
    if (!L || max_tokens < 0) {
        set_error("pd_layer_reserve: bad argument");
        return PD_ERR_INVALID_ARG;
    }
    if (max_tokens <= L->ws_tokens) return PD_OK;
    const WsLayout w = ws_layout(L, max_tokens);
    HIP_TRY(hipDeviceSynchronize(), PD_ERR_DEVICE);
    char *nw = nullptr;
    hipError_t e = hipMalloc((void **)&nw, w.total);
    if (e != hipSuccess) {
        set_error("pd_layer_reserve: cannot allocate %zu bytes of workspace: %s", w.total, hipGetErrorString(e));
        return PD_ERR_OOM;
    }
    if (L->ws) (void)hipFree(L->ws);
    L->ws = nw;
    ws_bind(L, nw, w, max_tokens);
    return PD_OK;
}

// ---- KV cache ------------------------------------------------------------------------------------

static pd_status cache_create(const pd_layer *L, int32_t max_seqs, int32_t max_len, int fp8, double k_scale,
                              double v_scale, pd_kv_cache **out)
{
    if (!L || !out || max_seqs <= 0 || max_len <= 0) {
        set_error("pd_kv_cache_create: bad argument");
        return PD_ERR_INVALID_ARG;
    }
    const bool can_block = L->cfg.dtype == PD_BF16 && L->cfg.head_dim == 128 &&
                           L->cfg.n_q_heads / L->cfg.n_kv_heads <= 16;
    if (fp8) {
        if (!(k_scale > 0.0) || !(v_scale > 0.0) || !std::isfinite(k_scale) || !std::isfinite(v_scale)) {
            set_error("pd_kv_cache_create_fp8: scales must be positive and finite");
            return PD_ERR_INVALID_ARG;
        }
        if (!can_block || !L->use_mfma) {
            set_error("pd_kv_cache_create_fp8: needs a bf16 layer with head_dim 128, at most 16 query heads per "
                      "kv head and the matrix-core plan");
            return PD_ERR_DTYPE;
        }
    }
    pd_kv_cache *c = new pd_kv_cache();
    c->dtype = L->cfg.dtype;
    c->Hkv = L->cfg.n_kv_heads;
    c->hd = L->cfg.head_dim;
    c->max_seqs = max_seqs;
    c->max_len = max_len;
    c->blocked = can_block ? 1 : 0;
    c->plane_len = c->blocked ? (max_len + 63) / 64 * 64 : max_len;
    c->fp8 = fp8;
    c->k_scale = fp8 ? k_scale : 1.0;
    c->v_scale = fp8 ? v_scale : 1.0;
    c->k = c->v = nullptr;
    c->d_len = nullptr;
    size_t bytes = (size_t)max_seqs * c->Hkv * c->plane_len * c->hd * (fp8 ? 1 : L->esz);
    hipError_t e = hipMalloc(&c->k, bytes);
    if (e == hipSuccess) e = hipMalloc(&c->v, bytes);
    // zero fill: positions past a slot's length are multiplied by zero weights and must be finite
    if (e == hipSuccess) e = hipMemset(c->k, 0, bytes);
    if (e == hipSuccess) e = hipMemset(c->v, 0, bytes);
    if (e == hipSuccess) e = hipMalloc((void **)&c->d_len, sizeof(int32_t) * max_seqs);
    if (e == hipSuccess) e = hipMemset(c->d_len, 0, sizeof(int32_t) * max_seqs);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        set_error("pd_kv_cache_create: %s (2 x %zu bytes)", hipGetErrorString(e), bytes);
        if (c->k) (void)hipFree(c->k);
        if (c->v) (void)hipFree(c->v);
        if (c->d_len) (void)hipFree(c->d_len);
        delete c;
        return e == hipErrorOutOfMemory ? PD_ERR_OOM : PD_ERR_DEVICE;
    }
    c->h_len.assign((size_t)max_seqs, 0);
    *out = c;
    return PD_OK;
}

extern "C" pd_status pd_kv_cache_create(const pd_layer *L, int32_t max_seqs, int32_t max_len,
                                        pd_kv_cache **out)
{
    return cache_create(L, max_seqs, max_len, 0, 1.0, 1.0, out);
}

extern "C" pd_status pd_kv_cache_create_fp8(const pd_layer *L, int32_t max_seqs, int32_t max_len,
                                            double k_scale, double v_scale, pd_kv_cache **out)
{
    return cache_create(L, max_seqs, max_len, 1, k_scale, v_scale, out);
}

extern "C" void pd_kv_cache_destroy(pd_kv_cache *c)
{
    if (!c) return;
    (void)hipDeviceSynchronize();
    (void)hipFree(c->k);
    (void)hipFree(c->v);
    (void)hipFree(c->d_len);
    delete c;
}

extern "C" pd_status pd_kv_cache_set_len(pd_kv_cache *c, int32_t slot, int32_t len, void *stream)
{
    if (!c || slot < 0 || slot >= c->max_seqs || len < 0) {
        set_error("pd_kv_cache_set_len: bad argument");
        return PD_ERR_INVALID_ARG;
    }
    if (len > c->max_len) {
        set_error("pd_kv_cache_set_len: len %d > max_len %d", len, c->max_len);
        return PD_ERR_KV_CAPACITY;
    }
    HIP_TRY(launch_write_ints(c->d_len + slot, &len, 1, (hipStream_t)stream), PD_ERR_DEVICE);
    c->h_len[(size_t)slot] = len;
    return PD_OK;
}

extern "C" pd_status pd_kv_cache_set(pd_kv_cache *c, int32_t slot, int32_t len, const void *k,
                                     const void *v, void *stream)
{
    if (!c || slot < 0 || slot >= c->max_seqs || len < 0 || (len > 0 && (!k || !v))) {
        set_error("pd_kv_cache_set: bad argument");
        return PD_ERR_INVALID_ARG;
    }
    if (len > c->max_len) {
        set_error("pd_kv_cache_set: len %d > max_len %d", len, c->max_len);
        return PD_ERR_KV_CAPACITY;
    }
    if (c->fp8)
        HIP_TRY(launch_kv_copy_fp8(c->k, c->v, k, v, slot, c->Hkv, len, c->plane_len, c->k_scale, c->v_scale, 1,
                                   (hipStream_t)stream),
                PD_ERR_DEVICE);
    else
        HIP_TRY(launch_kv_copy(c->dtype, c->k, c->v, k, v, slot, c->Hkv, len, c->hd, c->plane_len,
                               c->blocked, 1, (hipStream_t)stream),
                PD_ERR_DEVICE);
    return pd_kv_cache_set_len(c, slot, len, stream);
}

extern "C" pd_status pd_kv_cache_get(const pd_kv_cache *c, int32_t slot, int32_t len, void *k,
                                     void *v, void *stream)
{
    if (!c || slot < 0 || slot >= c->max_seqs || len < 0 || len > c->max_len || (len > 0 && (!k || !v))) {
        set_error("pd_kv_cache_get: bad argument");
        return PD_ERR_INVALID_ARG;
    }
    if (c->fp8)
        HIP_TRY(launch_kv_copy_fp8(c->k, c->v, k, v, slot, c->Hkv, len, c->plane_len, c->k_scale, c->v_scale, 0,
                                   (hipStream_t)stream),
                PD_ERR_DEVICE);
    else
        HIP_TRY(launch_kv_copy(c->dtype, c->k, c->v, k, v, slot, c->Hkv, len, c->hd, c->plane_len,
                               c->blocked, 0, (hipStream_t)stream),
                PD_ERR_DEVICE);
    return PD_OK;
}

extern "C" pd_status pd_kv_cache_len(const pd_kv_cache *c, int32_t slot, int32_t *len)
{
    if (!c || !len || slot < 0 || slot >= c->max_seqs) {
        set_error("pd_kv_cache_len: bad argument");
        return PD_ERR_INVALID_ARG;
    }
    *len = c->h_len[(size_t)slot];
    return PD_OK;
}

// ---- layer forward -------------------------------------------------------------------------------

static hipError_t run_gemm(const pd_layer *L, GemmArgs g, hipStream_t s)
{
    g.splitk_ws = L->splitk;
    g.splitk_ws_elems = L->splitk_elems;
    g.packed = L->packed ? 1 : 0;
    if (L->packed) {
        // packed weights are only understood by the matrix-core kernels
        if (L->w8) {
            // decode-sized products stream the 8-bit twin of the matrix; the tiled kernels take the bf16 pack
            const void *tiles = nullptr;
            if (g.B == L->w_qkv) { g.B8 = L->q_qkv; g.b_scale = L->s_qkv; tiles = L->t_qkv; }
            else if (g.B == L->w_o) { g.B8 = L->q_o; g.b_scale = L->s_o; tiles = L->t_o; }
            else if (g.B == L->w_gate) { g.B8 = L->q_gate; g.b_scale = L->s_gate; tiles = L->t_gate; }
            else if (g.B == L->w_down) { g.B8 = L->q_down; g.b_scale = L->s_down; tiles = L->t_down; }
            if (L->a8 && L->call_rows > kA8Rows && tiles) {
                // 8-bit activations: quantise the input rows (unless the norm before already did; a
                // gathered operand is quantised where it lies, once per token), then codes x codes on the
                // matrix cores
                if (L->a8_src != g.A) {
                    const int src_rows = g.a_gather ? L->call_rows : g.M;
                    hipError_t e = launch_quant_rows_e4m3(g.A, g.lda, src_rows, g.K, L->a8_codes, L->a8_scales, s);
                    if (e != hipSuccess) return e;
                }
                L->a8_src = nullptr;
                GemmArgs f = g;
                f.A = L->a8_codes;
                f.B = tiles;
                f.B8 = nullptr;
                f.a_scale = L->a8_scales;
                f.K = g.K / 2;
                f.lda = g.K / 2;
                f.ldb = g.K / 2;
                f.b_group_stride = g.b_group_stride / 2;
                if (!gemm_mfma_f8_supported(f)) return hipErrorInvalidValue;
                return launch_gemm_mfma_f8(f, s);
            }
        }
        if (gemv_mfma_supported(g)) return launch_gemv_mfma(g, s);
        if (wgemm_mfma_supported(g)) return launch_wgemm_mfma(g, s);
        if (gemm_mfma_supported(g)) return launch_gemm_mfma(g, s);
        return hipErrorInvalidValue;
    }
    return launch_gemm_generic(L->cfg.dtype, g, s);
}

// RMSNorm in front of a projection: where that projection will multiply codes, the normalised rows go
// straight to codes (y is then not written; nothing else reads it in a dense layer).
static hipError_t norm_for_gemm(const pd_layer *L, const void *x, const void *g, void *y, int T, hipStream_t s)
{
    const pd_layer_config &c = L->cfg;
    L->a8_src = nullptr;
    if (L->a8 && c.n_experts == 0 && T > kA8Rows && rmsnorm_quant_supported(c.d_model)) {
        hipError_t e = launch_rmsnorm_quant_e4m3(x, g, T, c.d_model, c.rms_eps, L->a8_codes, L->a8_scales, s);
        if (e == hipSuccess) L->a8_src = y;
        return e;
    }
    return launch_rmsnorm(c.dtype, x, g, y, T, c.d_model, c.rms_eps, s);
}

static bool cache_matches(const pd_layer *L, const pd_kv_cache *c)
{
    return c->dtype == L->cfg.dtype && c->Hkv == L->cfg.n_kv_heads && c->hd == L->cfg.head_dim;
}

// Everything after the attention output: O projection + residual, RMSNorm, FFN or MoE.
// append (decode step with the fused rotary embedding, bf16 layers): the step's cache append rides in the
// launch of the second RMSNorm.
static pd_status run_tail(pd_layer *L, const void *x, int T, const void *router_logits, void *out,
                          hipStream_t s, const RopeArgs *append = nullptr)
{
    const pd_layer_config &c = L->cfg;
    const int d = c.d_model, F = c.d_ff, E = c.n_experts;
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    // h = x + o Wo^T
    g.A = L->o; g.lda = L->Nq; g.B = L->w_o; g.ldb = L->Nq; g.C = L->h; g.ldc = d; g.R = x; g.ldr = d;
    g.M = T; g.N = d; g.K = L->Nq; g.epilogue = EPI_RESIDUAL; g.n_groups = 1;
    // where this product splits K over workgroups, the launch that adds the partials also normalises the
    // rows it forms (and carries the decode step's cache append): one launch fewer
    int norm_fused = 0;
    if (c.dtype == PD_BF16 && !(L->a8 && T > kA8Rows)) {
        g.fuse_g = L->g_ffn; g.fuse_y = L->y; g.fuse_eps = c.rms_eps; g.fuse_append = append; g.fuse_done = &norm_fused;
    }
    STEP("o_proj_residual", run_gemm(L, g, s));
    if (norm_fused) L->a8_src = nullptr;
    if (E == 0) {
        memset(&g, 0, sizeof(g));
        g.A = L->h; g.lda = d; g.B = L->w_gate; g.B1 = L->w_up; g.ldb = d; g.C = L->act; g.ldc = F;
        g.M = T; g.N = F; g.K = d; g.epilogue = EPI_SWIGLU; g.n_groups = 1;
        if (norm_fused) {
        } else if (append) {
            L->a8_src = nullptr;
            STEP("rmsnorm_ffn", launch_rmsnorm_append(*append, L->h, L->g_ffn, L->y, T, d, c.rms_eps, s));
        } else {
            STEP("rmsnorm_ffn", norm_for_gemm(L, L->h, L->g_ffn, L->y, T, s));
        }
        g.A = L->y;
        STEP("gate_up_swiglu", run_gemm(L, g, s));
        memset(&g, 0, sizeof(g));
        g.A = L->act; g.lda = F; g.B = L->w_down; g.ldb = F; g.C = out; g.ldc = d; g.R = L->h; g.ldr = d;
        g.M = T; g.N = d; g.K = F; g.epilogue = EPI_RESIDUAL; g.n_groups = 1;
        STEP("down_residual", run_gemm(L, g, s));
        return PD_OK;
    }
    if (norm_fused) {
    } else if (append) {
        STEP("rmsnorm_ffn", launch_rmsnorm_append(*append, L->h, L->g_ffn, L->y, T, d, c.rms_eps, s));
    } else {
        STEP("rmsnorm_ffn", launch_rmsnorm(c.dtype, L->h, L->g_ffn, L->y, T, d, c.rms_eps, s));
    }
    const float *logits = (const float *)router_logits;
    if (!logits) {
        STEP("router_logits", launch_router_logits(c.dtype, L->y, L->w_router, L->logits, T, d, E, s));
        logits = L->logits;
    }
    MoeRouteArgs r;
    r.logits = logits; r.T = T; r.E = E; r.top_k = c.top_k; r.expert_idx = L->eidx; r.expert_w = L->ew;
    r.sorted_token = L->sorted_token; r.pair_pos = L->pair_pos; r.offsets = L->offsets; r.block_hist = L->block_hist;
    STEP("moe_route_sort", launch_moe_route(r, s));
    const int P = T * c.top_k;
    memset(&g, 0, sizeof(g));
    g.A = L->y; g.lda = d; g.a_gather = L->sorted_token; g.B = L->w_gate; g.B1 = L->w_up; g.ldb = d;
    g.b_group_stride = (int64_t)(L->packed ? 2 : 1) * F * d; g.group_offsets = L->offsets; g.n_groups = E;
    g.C = L->act; g.ldc = F; g.M = P; g.N = F; g.K = d; g.epilogue = EPI_SWIGLU;
    STEP("moe_gate_up_swiglu", run_gemm(L, g, s));
    memset(&g, 0, sizeof(g));
    g.A = L->act; g.lda = F; g.B = L->w_down; g.ldb = F; g.b_group_stride = (int64_t)d * F;
    g.group_offsets = L->offsets; g.n_groups = E; g.C = L->eo; g.ldc = d; g.M = P; g.N = d; g.K = F;
    g.epilogue = EPI_NONE;
    STEP("moe_down", run_gemm(L, g, s));
    STEP("moe_combine", launch_moe_combine(c.dtype, L->h, L->eo, L->pair_pos, L->ew, out, T, d, c.top_k, s));
    return PD_OK;
}

// Shared body of pd_prefill (chunk = false: positions from 0, a cache slot is overwritten) and
// pd_prefill_chunk (chunk = true: positions behind the slot's cached prefix, appended).
static pd_status prefill_common(pd_layer *L, const pd_tokens *tk, pd_kv_cache *cache, void *out,
                                void *stream, bool chunk)
{
    if (!L || !tk || !tk->cu_seqlens) {
        set_error("pd_prefill: NULL argument");
        return PD_ERR_INVALID_ARG;
    }
    const int n = tk->n_seqs;
    if (n < 1 || n > kMaxSeqs) {
        set_error("pd_prefill: n_seqs %d outside 1..%d", n, kMaxSeqs);
        return PD_ERR_INVALID_ARG;
    }
    if (tk->cu_seqlens[0] != 0) {
        set_error("pd_prefill: cu_seqlens[0] must be 0");
        return PD_ERR_SHAPE;
    }
    int max_L = 0;
    for (int s = 0; s < n; ++s) {
        int Ls = tk->cu_seqlens[s + 1] - tk->cu_seqlens[s];
        if (Ls < 0) {
            set_error("pd_prefill: cu_seqlens decreases at %d", s);
            return PD_ERR_SHAPE;
        }
        if (Ls > max_L) max_L = Ls;
    }
    const int T = tk->cu_seqlens[n];
    if (chunk && (!cache || !tk->slots)) {
        set_error("pd_prefill_chunk: needs a cache and one slot per sequence");
        return PD_ERR_INVALID_ARG;
    }
    const bool keep = cache && tk->slots;
    std::vector<int32_t> prefix((size_t)n, 0);
    if (keep) {
        if (!cache_matches(L, cache)) {
            set_error("pd_prefill: cache was created for a different layer shape");
            return PD_ERR_INVALID_ARG;
        }
        std::vector<char> seen((size_t)cache->max_seqs, 0);
        for (int s = 0; s < n; ++s) {
            int sl = tk->slots[s];
            if (sl < 0 || sl >= cache->max_seqs || seen[(size_t)sl]) {
                set_error("pd_prefill: slot %d (sequence %d) out of range or repeated", sl, s);
                return PD_ERR_INVALID_ARG;
            }
            seen[(size_t)sl] = 1;
        }
        if (chunk)
            for (int s = 0; s < n; ++s) prefix[(size_t)s] = cache->h_len[(size_t)tk->slots[s]];
        for (int s = 0; s < n; ++s) {
            const int Ls = tk->cu_seqlens[s + 1] - tk->cu_seqlens[s];
            if (prefix[(size_t)s] + Ls > cache->max_len) {
                set_error("pd_prefill: sequence %d would hold %d tokens, the cache's max_len is %d", s,
                          prefix[(size_t)s] + Ls, cache->max_len);
                return PD_ERR_KV_CAPACITY;
            }
        }
    }
    if (T == 0) {
        if (keep && !chunk)
            for (int s = 0; s < n; ++s) {
                pd_status st = pd_kv_cache_set_len(cache, tk->slots[s], 0, stream);
                if (st != PD_OK) return st;
            }
        return PD_OK;
    }
    if (!tk->hidden || !out) {
        set_error("pd_prefill: NULL hidden or output");
        return PD_ERR_INVALID_ARG;
    }
    const pd_layer_config &c = L->cfg;
    if (c.n_experts > 0 && !tk->router_logits && !L->w_router) {
        set_error("pd_prefill: MoE layer needs router_logits or w_router");
        return PD_ERR_INVALID_ARG;
    }
    L->call_rows = T;
    pd_status st = pd_layer_reserve(L, T);
    if (st != PD_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    L->prof_names.clear();

    // padded key-row starts of the sequences (multiples of 64) for the matrix-core attention's
    // transposed-V scratch (and, chunked, the gathered key rows)
    std::vector<int32_t> pad((size_t)n + 1);
    pad[0] = 0;
    for (int q = 0; q < n; ++q)
        pad[(size_t)q + 1] = pad[(size_t)q] +
                             (prefix[(size_t)q] + tk->cu_seqlens[q + 1] - tk->cu_seqlens[q] + 63) / 64 * 64;
    {
        int32_t *const dst[4] = {L->d_cu, L->d_pad_cu, L->d_slots, L->d_prefix};
        const int32_t *const src[4] = {tk->cu_seqlens, pad.data(), tk->slots, prefix.data()};
        const int cnt[4] = {n + 1, n + 1, keep ? n : 0, chunk ? n : 0};
        HIP_TRY(launch_prefill_meta(dst, src, cnt, n, T, L->tok_seq, L->tok_pos, L->tok_slot, s), PD_ERR_DEVICE);
    }
    STEP("rmsnorm_attn", norm_for_gemm(L, tk->hidden, L->g_attn, L->y, T, s));
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.A = L->y; g.lda = c.d_model; g.B = L->w_qkv; g.ldb = c.d_model; g.C = L->qkv; g.ldc = L->Nqkv;
    g.M = T; g.N = L->Nqkv; g.K = c.d_model; g.epilogue = EPI_NONE; g.n_groups = 1;
    STEP("qkv_proj", run_gemm(L, g, s));
    RopeArgs r;
    r.qkv = L->qkv; r.ld = L->Nqkv; r.T = T; r.Hq = c.n_q_heads; r.Hkv = c.n_kv_heads; r.hd = c.head_dim;
    r.tok_pos = L->tok_pos; r.tok_slot = keep ? L->tok_slot : nullptr;
    r.k_cache = keep ? cache->k : nullptr; r.v_cache = keep ? cache->v : nullptr;
    r.max_len = keep ? cache->plane_len : 0; r.blocked = keep ? cache->blocked : 0; r.inv_freq = L->inv_freq;
    r.fp8 = keep ? cache->fp8 : 0; r.k_scale = keep ? cache->k_scale : 1.0; r.v_scale = keep ? cache->v_scale : 1.0;
    r.table = L->rope_table; r.table_len = kRopeTableLen;
    STEP("rope_kv_write", launch_rope_kv(c.dtype, r, s));
    AttnArgs a;
    memset(&a, 0, sizeof(a));
    a.qkv = L->qkv; a.ld = L->Nqkv; a.o = L->o; a.T = T; a.Hq = c.n_q_heads; a.Hkv = c.n_kv_heads;
    a.hd = c.head_dim; a.scale = (float)(1.0 / sqrt((double)c.head_dim)); a.tok_pos = L->tok_pos;
    a.decode = 0; a.d_cu = L->d_cu; a.n_seqs = n; a.max_seq_len = max_L;
    if (chunk && !cache->blocked) {
        // plain cache layout: every row reads keys 0 .. its own position of its slot
        a.decode = 1; a.tok_slot = L->tok_slot; a.k_cache = cache->k; a.v_cache = cache->v;
        a.max_len = cache->max_len;
        STEP("prefill_attention", launch_attn_generic(c.dtype, a, s));
    } else if (chunk && max_L <= kShortChunk) {
        // A few new tokens per sequence over a blocked cache (multi-token decode): the decode
        // attention kernel streams the cache once per unit of a few tokens instead of gathering the
        // prefix for the prefill kernel.
        // Units of up to 16 / group consecutive tokens of one sequence share one pass over the cache:
        // their (token, head) pairs are the 16 MFMA columns of the decode attention kernel.
        const int tb = 16 / (c.n_q_heads / c.n_kv_heads);
        std::vector<int32_t> u_slot, u_pos, u_row, u_cnt, u_keys;
        for (int q = 0; q < n; ++q) {
            const int Ls = tk->cu_seqlens[q + 1] - tk->cu_seqlens[q];
            for (int i0 = 0; i0 < Ls; i0 += tb) {
                const int cnt = Ls - i0 < tb ? Ls - i0 : tb;
                u_slot.push_back(tk->slots[q]);
                u_pos.push_back(prefix[(size_t)q] + i0);
                u_row.push_back(tk->cu_seqlens[q] + i0);
                u_cnt.push_back(cnt);
                u_keys.push_back(prefix[(size_t)q] + i0 + cnt);
            }
        }
        const int nu = (int)u_slot.size();
        // Partial results are rows of 130 floats, [chunk][kv head][16 columns]; the workspace part holds
        // what a one-token decode step of ws_tokens rows needs.  Every unit needs at least one chunk, so a
        // call of many short sequences can need more than that: the rest comes from the attention scratch
        // buffer (unused on this path), grown on demand like for an ordinary prefill.
        const size_t rows_per_chunk = (size_t)c.n_kv_heads * 16;
        const size_t ws_rows = decode_chunk_bound(L, L->ws_tokens) * c.n_q_heads;
        size_t max_chunks = ws_rows / rows_per_chunk;
        const size_t floor_chunks = (size_t)nu + (size_t)(8192 / c.n_kv_heads + 1);
        if (max_chunks < floor_chunks) max_chunks = floor_chunks;
        const int chunk_keys = pick_chunk_keys(u_keys, c.n_kv_heads, max_chunks);
        std::vector<int32_t> ccu((size_t)nu + 1);
        ccu[0] = 0;
        for (int u = 0; u < nu; ++u)
            ccu[(size_t)u + 1] = ccu[(size_t)u] + (u_pos[(size_t)u] + u_cnt[(size_t)u] + chunk_keys - 1) / chunk_keys;
        const int total_chunks = ccu[(size_t)nu];
        if ((size_t)total_chunks > max_chunks) {
            set_error("pd_prefill_chunk: internal chunk bound exceeded (%d chunks)", total_chunks);
            return PD_ERR_DEVICE;
        }
        float *part = L->dec_part;
        if ((size_t)total_chunks * rows_per_chunk > ws_rows) {
            const size_t need = (size_t)total_chunks * rows_per_chunk * 130 * sizeof(float);
            if (need > L->vt_cap) {
                HIP_TRY(hipDeviceSynchronize(), PD_ERR_DEVICE);
                if (L->vt) (void)hipFree(L->vt);
                L->vt = nullptr;
                L->vt_cap = 0;
                hipError_t e = hipMalloc(&L->vt, need);
                if (e != hipSuccess) {
                    set_error("pd_prefill_chunk: cannot allocate %zu bytes of attention scratch", need);
                    return PD_ERR_OOM;
                }
                L->vt_cap = need;
            }
            part = (float *)L->vt;
        }
        const size_t ws_t = (size_t)L->ws_tokens;
        HIP_TRY(launch_write_ints(L->chunk_cu, ccu.data(), nu + 1, s), PD_ERR_DEVICE);
        HIP_TRY(launch_write_ints(L->units, u_slot.data(), nu, s), PD_ERR_DEVICE);
        HIP_TRY(launch_write_ints(L->units + ws_t, u_pos.data(), nu, s), PD_ERR_DEVICE);
        HIP_TRY(launch_write_ints(L->units + 2 * ws_t, u_row.data(), nu, s), PD_ERR_DEVICE);
        HIP_TRY(launch_write_ints(L->units + 3 * ws_t, u_cnt.data(), nu, s), PD_ERR_DEVICE);
        DecodeAttnArgs da;
        memset(&da, 0, sizeof(da));
        da.qkv = L->qkv; da.ld = L->Nqkv; da.o = L->o; da.B = nu; da.Hq = c.n_q_heads; da.Hkv = c.n_kv_heads;
        da.scale = a.scale; da.slots = L->units; da.pos = L->units + ws_t;
        da.u_row0 = L->units + 2 * ws_t; da.u_ntok = L->units + 3 * ws_t;
        da.chunk_cu = L->chunk_cu; da.chunk_keys = chunk_keys; da.total_chunks = total_chunks;
        da.k_cache = cache->k; da.v_cache = cache->v; da.max_len_pad = cache->plane_len;
        da.fp8 = cache->fp8; da.k_scale = (float)cache->k_scale; da.v_scale = (float)cache->v_scale;
        da.part_o = part;
        da.part_ml = part + (size_t)total_chunks * c.n_kv_heads * 16 * 128;
        STEP("prefill_attention", launch_decode_attn_mfma(da, s));
    } else if (chunk || (L->use_mfma && attn_prefill_mfma_supported(a))) {
        if (chunk && !attn_prefill_mfma_supported(a)) {
            set_error("pd_prefill_chunk: blocked cache without the matrix-core attention path");
            return PD_ERR_SHAPE;
        }
        const int vt_ld = pad[(size_t)n];
        const size_t vt_bytes = (size_t)c.n_kv_heads * c.head_dim * vt_ld * 2;
        int n_split = 1, max_keys = 0;
        if (chunk) {
            for (int q = 0; q < n; ++q)
                max_keys = std::max(max_keys, prefix[(size_t)q] + tk->cu_seqlens[q + 1] - tk->cu_seqlens[q]);
            n_split = attn_chunk_splits(a, max_keys);
        }
        const size_t need = chunk ? 2 * vt_bytes + attn_chunk_split_bytes(a, n_split) : vt_bytes;
        if (need > L->vt_cap) {
            HIP_TRY(hipDeviceSynchronize(), PD_ERR_DEVICE);
            if (L->vt) (void)hipFree(L->vt);
            L->vt = nullptr;
            L->vt_cap = 0;
            hipError_t e = hipMalloc(&L->vt, need);
            if (e != hipSuccess) {
                set_error("pd_prefill: cannot allocate %zu bytes of attention scratch", need);
                return PD_ERR_OOM;
            }
            L->vt_cap = need;
        }
        if (chunk) {
            a.prefix = L->d_prefix; a.k_cache = cache->k; a.v_cache = cache->v; a.max_len = cache->plane_len;
            a.kv_fp8 = cache->fp8; a.k_scale = (float)cache->k_scale; a.v_scale = (float)cache->v_scale;
            STEP("prefill_attention",
                 launch_attn_chunk_mfma(a, L->d_slots, (uint16_t *)((char *)L->vt + vt_bytes), (uint16_t *)L->vt,
                                        vt_ld, L->d_pad_cu, n_split, (float *)((char *)L->vt + 2 * vt_bytes), s));
        } else {
            STEP("prefill_attention", launch_attn_prefill_mfma(a, (uint16_t *)L->vt, vt_ld, L->d_pad_cu, s));
        }
    } else {
        STEP("prefill_attention", launch_attn_generic(c.dtype, a, s));
    }
    st = run_tail(L, tk->hidden, T, tk->router_logits, out, s);
    if (st != PD_OK) return st;
    if (keep) {
        HIP_TRY(launch_prefill_set_len(L->d_slots, L->d_cu, n, cache->d_len, chunk ? 1 : 0, s), PD_ERR_DEVICE);
        for (int q = 0; q < n; ++q)
            cache->h_len[(size_t)tk->slots[q]] = prefix[(size_t)q] + tk->cu_seqlens[q + 1] - tk->cu_seqlens[q];
    }
    L->last_rows = T;
    return PD_OK;
}

extern "C" pd_status pd_prefill(pd_layer *L, const pd_tokens *tk, pd_kv_cache *cache, void *out,
                                void *stream)
{
    return prefill_common(L, tk, cache, out, stream, false);
}

extern "C" pd_status pd_prefill_chunk(pd_layer *L, const pd_tokens *tk, pd_kv_cache *cache, void *out,
                                      void *stream)
{
    return prefill_common(L, tk, cache, out, stream, true);
}

// ---- static scratch for the entry point that allocates nothing --------------------------------------
// One array per GPU, held from the moment the library's code is loaded on it until the process ends.
// Host code never uses the array's name as an address: the device address of the current device's
// copy comes from hipGetSymbolAddress, once per device.
static const size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static pd_status static_scratch_ptr(const pd_layer *L, char **ptr)
{
    static std::atomic<void *> ptrs[64];
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev), PD_ERR_DEVICE);
    if (dev != L->device || dev < 0 || dev >= 64) {
        set_error("pd_decode_step_noalloc: the layer's device %d must be the current device (it is %d)", L->device, dev);
        return PD_ERR_INVALID_ARG;
    }
    void *p = ptrs[dev].load(std::memory_order_acquire);
    if (!p) {
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), PD_ERR_DEVICE);
        if (!p) {
            set_error("pd_decode_step_noalloc: no address for the static scratch array");
            return PD_ERR_DEVICE;
        }
        ptrs[dev].store(p, std::memory_order_release);
    }
    *ptr = (char *)p;
    return PD_OK;
}

static pd_status decode_step_impl(pd_layer *L, const pd_batch *bt, pd_kv_cache *cache, void *out, void *stream,
                                  bool static_ws);

extern "C" pd_status pd_decode_step(pd_layer *L, const pd_batch *bt, pd_kv_cache *cache, void *out,
                                    void *stream)
{
    return decode_step_impl(L, bt, cache, out, stream, false);
}

extern "C" pd_status pd_decode_step_noalloc(pd_layer *L, const pd_batch *bt, pd_kv_cache *cache, void *out,
                                            void *stream)
{
    if (!L) {
        set_error("pd_decode_step_noalloc: NULL layer");
        return PD_ERR_INVALID_ARG;
    }
    // the step runs on the static array instead of the layer's workspace; the layer's own workspace (if
    // any) is bound again afterwards, untouched
    const int own_tokens = L->ws_tokens;
    const bool prof = L->prof_on;
    L->prof_on = false;                      // per-kernel events would have to be created
    L->chunk_slack_workers = kChunkSlackWorkersStatic;
    const pd_status st = decode_step_impl(L, bt, cache, out, stream, true);
    L->chunk_slack_workers = kChunkSlackWorkers;
    L->prof_on = prof;
    L->ws_tokens = 0;
    if (L->ws) ws_bind(L, L->ws, ws_layout(L, own_tokens), own_tokens);
    return st;
}

static pd_status decode_step_impl(pd_layer *L, const pd_batch *bt, pd_kv_cache *cache, void *out, void *stream,
                                  bool static_ws)
{
    if (!L || !bt || !cache || !bt->slots || !bt->hidden || !out) {
        set_error("pd_decode_step: NULL argument");
        return PD_ERR_INVALID_ARG;
    }
    const int B = bt->batch;
    if (B < 1 || B > kMaxSeqs) {
        set_error("pd_decode_step: batch %d outside 1..%d", B, kMaxSeqs);
        return PD_ERR_INVALID_ARG;
    }
    if (!cache_matches(L, cache)) {
        set_error("pd_decode_step: cache was created for a different layer shape");
        return PD_ERR_INVALID_ARG;
    }
    const pd_layer_config &c = L->cfg;
    if (c.n_experts > 0 && !bt->router_logits && !L->w_router) {
        set_error("pd_decode_step: MoE layer needs router_logits or w_router");
        return PD_ERR_INVALID_ARG;
    }
    {
        std::vector<char> seen((size_t)cache->max_seqs, 0);
        for (int b = 0; b < B; ++b) {
            int sl = bt->slots[b];
            if (sl < 0 || sl >= cache->max_seqs || seen[(size_t)sl]) {
                set_error("pd_decode_step: slot %d (row %d) out of range or repeated", sl, b);
                return PD_ERR_INVALID_ARG;
            }
            seen[(size_t)sl] = 1;
        }
        for (int b = 0; b < B; ++b)
            if (cache->h_len[(size_t)bt->slots[b]] + 1 > cache->max_len) {
                set_error("pd_decode_step: slot %d is full (%d positions)", bt->slots[b], cache->max_len);
                return PD_ERR_KV_CAPACITY;
            }
    }
    L->call_rows = B;
    pd_status st = PD_OK;
    if (static_ws) {
        const size_t rows = (size_t)B * (c.n_experts > 0 ? c.top_k : 1);
        // split-K partials: a launcher's splits x columns stay within 256 workgroups x 128 columns per row
        const WsLayout w = ws_layout(L, B, rows < 256 ? rows : 256, 256 * 128);
        if (w.total > kStaticScratchBytes) {
            set_error("pd_decode_step_noalloc: a batch of %d rows of this layer needs %zu bytes of scratch, the static "
                      "array holds %zu", B, w.total, kStaticScratchBytes);
            return PD_ERR_SHAPE;
        }
        char *base = nullptr;
        st = static_scratch_ptr(L, &base);
        if (st != PD_OK) return st;
        ws_bind(L, base, w, B);
    } else {
        st = pd_layer_reserve(L, B);
        if (st != PD_OK) return st;
    }
    hipStream_t s = (hipStream_t)stream;
    L->prof_names.clear();

    // decode attention work split (see pick_chunk_keys)
    const bool mfma_dec = cache->blocked != 0;
    int chunk_keys = 64, total_chunks = 0;
    if (mfma_dec) {
        std::vector<int32_t> keys((size_t)B);
        for (int b = 0; b < B; ++b) keys[(size_t)b] = cache->h_len[(size_t)bt->slots[b]] + 1;
        chunk_keys = pick_chunk_keys(keys, c.n_kv_heads, decode_chunk_bound(L, B));
        for (int b = 0; b < B; ++b)
            total_chunks += (cache->h_len[(size_t)bt->slots[b]] + 1 + chunk_keys - 1) / chunk_keys;
        if ((size_t)total_chunks > decode_chunk_bound(L, B)) {
            set_error("pd_decode_step: internal chunk bound exceeded (%d chunks)", total_chunks);
            return PD_ERR_DEVICE;
        }
    }
    // up to 256 rows of a bf16 layer: the step's bookkeeping rides in the launch of the first RMSNorm
    const bool meta_in_norm = mfma_dec && B <= 256 && c.dtype == PD_BF16 && c.d_model % 8 == 0 &&
                              !(L->a8 && B > kA8Rows);
    if (meta_in_norm) {
        L->a8_src = nullptr;
        STEP("rmsnorm_attn", launch_decode_meta_norm(bt->slots, L->d_slots, B, cache->d_len, L->tok_pos, L->chunk_cu,
                                                     L->chunk_seq, chunk_keys, bt->hidden, L->g_attn, L->y, c.d_model,
                                                     c.rms_eps, s));
    } else if (mfma_dec && B <= 256) {
        HIP_TRY(launch_decode_meta_chunks_upload(bt->slots, L->d_slots, B, cache->d_len, L->tok_pos, L->chunk_cu,
                                                 L->chunk_seq, chunk_keys, s),
                PD_ERR_DEVICE);
    } else {
        HIP_TRY(launch_write_ints(L->d_slots, bt->slots, B, s), PD_ERR_DEVICE);
        if (mfma_dec)
            HIP_TRY(launch_decode_meta_chunks(L->d_slots, B, cache->d_len, L->tok_pos, L->chunk_cu, L->chunk_seq,
                                              chunk_keys, s),
                    PD_ERR_DEVICE);
        else
            HIP_TRY(launch_decode_meta(L->d_slots, B, cache->d_len, L->tok_pos, s), PD_ERR_DEVICE);
    }
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.A = bt->hidden; g.lda = c.d_model; g.B = L->w_qkv; g.ldb = c.d_model; g.C = L->qkv; g.ldc = L->Nqkv;
    g.M = B; g.N = L->Nqkv; g.K = c.d_model; g.epilogue = EPI_NONE; g.n_groups = 1;
    if (!meta_in_norm) STEP("rmsnorm_attn", norm_for_gemm(L, bt->hidden, L->g_attn, L->y, B, s));
    g.A = L->y;
    STEP("qkv_proj", run_gemm(L, g, s));
    RopeArgs r;
    r.qkv = L->qkv; r.ld = L->Nqkv; r.T = B; r.Hq = c.n_q_heads; r.Hkv = c.n_kv_heads; r.hd = c.head_dim;
    r.tok_pos = L->tok_pos; r.tok_slot = L->d_slots; r.k_cache = cache->k; r.v_cache = cache->v;
    r.max_len = cache->plane_len; r.blocked = cache->blocked; r.inv_freq = L->inv_freq;
    r.fp8 = cache->fp8; r.k_scale = cache->k_scale; r.v_scale = cache->v_scale;
    r.table = L->rope_table; r.table_len = kRopeTableLen;
    // Fused form (matrix-core attention over a blocked cache, no 8-bit activations in this call): the
    // attention kernel rotates q and the new key itself and takes the new token from registers; the
    // append to the cache rides in the launch of the second RMSNorm.  Otherwise a launch of its own
    // rotates in place and appends first.
    const bool fused_rope = mfma_dec && c.d_model % 8 == 0 && !(L->a8 && B > kA8Rows);
    if (!fused_rope) STEP("rope_kv_append", launch_rope_kv(c.dtype, r, s));
    if (mfma_dec) {
        DecodeAttnArgs da;
        memset(&da, 0, sizeof(da));
        if (fused_rope) {
            da.rope_table = L->rope_table; da.rope_table_len = kRopeTableLen; da.inv_freq = L->inv_freq;
            da.k_scale_d = cache->k_scale; da.v_scale_d = cache->v_scale;
        }
        da.qkv = L->qkv; da.ld = L->Nqkv; da.o = L->o; da.B = B; da.Hq = c.n_q_heads; da.Hkv = c.n_kv_heads;
        da.scale = (float)(1.0 / sqrt((double)c.head_dim)); da.slots = L->d_slots; da.pos = L->tok_pos;
        da.chunk_cu = L->chunk_cu; da.chunk_seq = L->chunk_seq; da.chunk_keys = chunk_keys; da.total_chunks = total_chunks;
        da.k_cache = cache->k; da.v_cache = cache->v; da.max_len_pad = cache->plane_len;
        da.fp8 = cache->fp8; da.k_scale = (float)cache->k_scale; da.v_scale = (float)cache->v_scale;
        da.part_o = L->dec_part;
        da.part_ml = L->dec_part + (size_t)total_chunks * c.n_q_heads * 128;
        STEP("decode_attention", launch_decode_attn_mfma(da, s));
    } else {
        AttnArgs a;
        memset(&a, 0, sizeof(a));
        a.qkv = L->qkv; a.ld = L->Nqkv; a.o = L->o; a.T = B; a.Hq = c.n_q_heads; a.Hkv = c.n_kv_heads;
        a.hd = c.head_dim; a.scale = (float)(1.0 / sqrt((double)c.head_dim)); a.tok_pos = L->tok_pos;
        a.tok_slot = L->d_slots; a.k_cache = cache->k; a.v_cache = cache->v; a.max_len = cache->max_len;
        a.decode = 1;
        STEP("decode_attention", launch_attn_generic(c.dtype, a, s));
    }
    st = run_tail(L, bt->hidden, B, bt->router_logits, out, s, mfma_dec && fused_rope ? &r : nullptr);
    if (st != PD_OK) return st;
    for (int b = 0; b < B; ++b) cache->h_len[(size_t)bt->slots[b]] += 1;
    L->last_rows = B;
    return PD_OK;
}

extern "C" pd_status pd_last_expert_choice(const pd_layer *L, int32_t rows, void *expert_idx,
                                           void *stream)
{
    if (!L || !expert_idx || L->cfg.n_experts <= 0 || rows < 0 || rows > L->last_rows) {
        set_error("pd_last_expert_choice: bad argument");
        return PD_ERR_INVALID_ARG;
    }
    HIP_TRY(hipMemcpyAsync(expert_idx, L->eidx, sizeof(int32_t) * (size_t)rows * L->cfg.top_k,
                           hipMemcpyDeviceToDevice, (hipStream_t)stream),
            PD_ERR_DEVICE);
    return PD_OK;
}

extern "C" pd_status pd_profile_enable(pd_layer *L, int32_t on)
{
    if (!L) {
        set_error("pd_profile_enable: NULL layer");
        return PD_ERR_INVALID_ARG;
    }
    L->prof_on = on != 0;
    L->prof_names.clear();
    return PD_OK;
}

extern "C" pd_status pd_profile_read(pd_layer *L, int32_t max_entries, const char **names, float *ms,
                                     int32_t *n)
{
    if (!L || !n || max_entries < 0 || (max_entries > 0 && (!names || !ms))) {
        set_error("pd_profile_read: bad argument");
        return PD_ERR_INVALID_ARG;
    }
    const int cnt = (int)L->prof_names.size();
    int outn = 0;
    for (int i = 0; i < cnt && outn < max_entries; ++i) {
        HIP_TRY(hipEventSynchronize(L->prof_ev[2 * i + 1]), PD_ERR_DEVICE);
        float t = 0.f;
        HIP_TRY(hipEventElapsedTime(&t, L->prof_ev[2 * i], L->prof_ev[2 * i + 1]), PD_ERR_DEVICE);
        names[outn] = L->prof_names[(size_t)i];
        ms[outn] = t;
        ++outn;
    }
    *n = outn;
    return PD_OK;
}

extern "C" pd_status pd_stream_copy(void *dst, const void *src, int64_t bytes, void *stream)
{
    if (!dst || !src || bytes <= 0 || bytes % 16 != 0 || ((uintptr_t)dst | (uintptr_t)src) % 16 != 0) {
        set_error("pd_stream_copy: pointers must be non-NULL and 16-byte aligned, bytes a positive multiple of 16");
        return PD_ERR_INVALID_ARG;
    }
    HIP_TRY(launch_stream_copy(dst, src, (size_t)bytes / 16, (hipStream_t)stream), PD_ERR_DEVICE);
    return PD_OK;
}

extern "C" pd_status pd_mfma_probe(const void *a_vals, const void *b_vals, int32_t n_workgroups, int32_t iters,
                                   float *sink, void *stream)
{
    if (!a_vals || !b_vals || !sink || n_workgroups < 1 || n_workgroups > 65536 || iters < 1 ||
        ((uintptr_t)a_vals | (uintptr_t)b_vals) % 16 != 0) {
        set_error("pd_mfma_probe: NULL or misaligned pointer, or a count outside 1 .. 65536 workgroups / iters >= 1");
        return PD_ERR_INVALID_ARG;
    }
    HIP_TRY(launch_mfma_probe(sink, a_vals, b_vals, n_workgroups, iters, (hipStream_t)stream), PD_ERR_DEVICE);
    return PD_OK;
}

// ---- stack ends: embedding, final norm + vocabulary projection -------------------------------------

struct pd_head {
    int dtype, d, vocab, max_rows, device;
    float eps;
    size_t esz;
    bool packed;        // bf16 with shapes the matrix-core kernels take: w_lm is in the block layout
    bool w8;            // w_lm also held as E4M3 codes with one power-of-two scale per vocabulary row
    void *g, *w_lm, *w_embed, *y, *q_lm;
    float *s_lm;
};

static void free_head(pd_head *h)
{
    if (!h) return;
    void *ptrs[] = {h->g, h->w_lm, h->w_embed, h->y, h->q_lm, h->s_lm};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
    delete h;
}

static pd_status head_create(int32_t d_model, int32_t vocab, float rms_eps, pd_dtype dtype,
                             const void *g_final, const void *w_embed, const void *w_lm,
                             int32_t max_rows, bool w8, pd_head **out);

extern "C" pd_status pd_head_create(int32_t d_model, int32_t vocab, float rms_eps, pd_dtype dtype,
                                    const void *g_final, const void *w_embed, const void *w_lm,
                                    int32_t max_rows, pd_head **out)
{
    return head_create(d_model, vocab, rms_eps, dtype, g_final, w_embed, w_lm, max_rows, false, out);
}

extern "C" pd_status pd_head_create_w8(int32_t d_model, int32_t vocab, float rms_eps, pd_dtype dtype,
                                       const void *g_final, const void *w_embed, const void *w_lm,
                                       int32_t max_rows, pd_head **out)
{
    return head_create(d_model, vocab, rms_eps, dtype, g_final, w_embed, w_lm, max_rows, true, out);
}

static pd_status head_create(int32_t d_model, int32_t vocab, float rms_eps, pd_dtype dtype,
                             const void *g_final, const void *w_embed, const void *w_lm,
                             int32_t max_rows, bool w8, pd_head **out)
{
    if (!g_final || !w_lm || !out || max_rows <= 0) {
        set_error("pd_head_create: NULL argument or max_rows <= 0");
        return PD_ERR_INVALID_ARG;
    }
    if (dtype != PD_F32 && dtype != PD_BF16) {
        set_error("pd_head_create: dtype %d is neither fp32 nor bf16", (int)dtype);
        return PD_ERR_DTYPE;
    }
    if (d_model <= 0 || vocab <= 0 || !(rms_eps >= 0.f)) {
        set_error("pd_head_create: unsupported shape (d=%d vocab=%d)", d_model, vocab);
        return PD_ERR_SHAPE;
    }
    pd_head *h = new pd_head();
    h->dtype = dtype; h->d = d_model; h->vocab = vocab; h->max_rows = max_rows; h->eps = rms_eps;
    h->esz = dtype == PD_F32 ? 4 : 2;
    h->packed = dtype == PD_BF16 && d_model % 64 == 0 && vocab % 16 == 0 &&
                (int64_t)d_model * 2 * vocab < (1ll << 32);
    h->w8 = w8;
    if (w8 && !h->packed) {
        set_error("pd_head_create_w8: needs a bf16 head with d_model a multiple of 64 and vocab a multiple of 16");
        delete h;
        return PD_ERR_DTYPE;
    }
    const size_t wbytes = (size_t)vocab * d_model * h->esz;
#define HEAD_TRY(expr)                                                                 \
    do {                                                                               \
        hipError_t e__ = (expr);                                                       \
        if (e__ != hipSuccess) {                                                       \
            set_error("pd_head_create: %s failed: %s", #expr, hipGetErrorString(e__)); \
            free_head(h);                                                              \
            return e__ == hipErrorOutOfMemory ? PD_ERR_OOM : PD_ERR_DEVICE;            \
        }                                                                              \
    } while (0)
    HEAD_TRY(hipGetDevice(&h->device));
    HEAD_TRY(hipMalloc(&h->g, d_model * h->esz));
    HEAD_TRY(hipMalloc(&h->w_lm, wbytes));
    HEAD_TRY(hipMalloc(&h->y, (size_t)max_rows * d_model * h->esz));
    HEAD_TRY(hipMemcpy(h->g, g_final, d_model * h->esz, hipMemcpyDeviceToDevice));
    if (h->w8) {
        HEAD_TRY(hipMalloc(&h->q_lm, (size_t)vocab * d_model));
        HEAD_TRY(hipMalloc((void **)&h->s_lm, sizeof(float) * (size_t)vocab));
        w8_row_scale_kernel<<<(vocab + 3) / 4, 256>>>(h->s_lm, (const uint16_t *)w_lm, nullptr, vocab, d_model);
        HEAD_TRY(hipGetLastError());
        pack_weight_w8_kernel<<<2048, 256>>>((uint4 *)h->w_lm, (uint8_t *)h->q_lm, (const uint4 *)w_lm, nullptr,
                                             h->s_lm, vocab, d_model);
        HEAD_TRY(hipGetLastError());
    } else if (h->packed) {
        pack_weight_kernel<<<2048, 256>>>((uint4 *)h->w_lm, (const uint4 *)w_lm, nullptr, vocab, d_model);
        HEAD_TRY(hipGetLastError());
    } else {
        HEAD_TRY(hipMemcpy(h->w_lm, w_lm, wbytes, hipMemcpyDeviceToDevice));
    }
    if (w_embed) {
        HEAD_TRY(hipMalloc(&h->w_embed, wbytes));
        HEAD_TRY(hipMemcpy(h->w_embed, w_embed, wbytes, hipMemcpyDeviceToDevice));
    }
    HEAD_TRY(hipDeviceSynchronize());
#undef HEAD_TRY
    *out = h;
    return PD_OK;
}

extern "C" void pd_head_destroy(pd_head *h)
{
    if (!h) return;
    (void)hipDeviceSynchronize();
    free_head(h);
}

extern "C" pd_status pd_embed(pd_head *h, const int32_t *token_ids, int32_t T, void *hidden, void *stream)
{
    if (!h || T < 0 || (T > 0 && (!token_ids || !hidden))) {
        set_error("pd_embed: bad argument");
        return PD_ERR_INVALID_ARG;
    }
    if (!h->w_embed) {
        set_error("pd_embed: the head was created without an embedding table");
        return PD_ERR_INVALID_ARG;
    }
    HIP_TRY(launch_embed_rows(hidden, h->w_embed, token_ids, T, h->vocab, (size_t)h->d * h->esz,
                              (hipStream_t)stream),
            PD_ERR_DEVICE);
    return PD_OK;
}

extern "C" pd_status pd_lm_head(pd_head *h, const void *hidden, int32_t T, void *logits, void *stream)
{
    if (!h || T < 0 || (T > 0 && (!hidden || !logits))) {
        set_error("pd_lm_head: bad argument");
        return PD_ERR_INVALID_ARG;
    }
    if (T > h->max_rows) {
        set_error("pd_lm_head: %d rows > max_rows %d", T, h->max_rows);
        return PD_ERR_INVALID_ARG;
    }
    if (T == 0) return PD_OK;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(launch_rmsnorm(h->dtype, hidden, h->g, h->y, T, h->d, h->eps, s), PD_ERR_DEVICE);
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.A = h->y; g.lda = h->d; g.B = h->w_lm; g.ldb = h->d; g.C = logits; g.ldc = h->vocab;
    g.M = T; g.N = h->vocab; g.K = h->d; g.epilogue = EPI_NONE; g.n_groups = 1;
    g.packed = h->packed ? 1 : 0;
    if (h->w8) {
        g.B8 = h->q_lm;
        g.b_scale = h->s_lm;
    }
    if (h->packed) {
        // packed weights are only understood by the matrix-core kernels
        if (gemv_mfma_supported(g)) HIP_TRY(launch_gemv_mfma(g, s), PD_ERR_DEVICE);
        else if (wgemm_mfma_supported(g)) HIP_TRY(launch_wgemm_mfma(g, s), PD_ERR_DEVICE);
        else if (gemm_mfma_supported(g)) HIP_TRY(launch_gemm_mfma(g, s), PD_ERR_DEVICE);
        else {
            set_error("pd_lm_head: shape not covered by the matrix-core kernels");
            return PD_ERR_SHAPE;
        }
    } else {
        HIP_TRY(launch_gemm_generic(h->dtype, g, s), PD_ERR_DEVICE);
    }
    return PD_OK;
}

extern "C" pd_status pd_kv_cache_set_lens(pd_kv_cache *c, int32_t n, const int32_t *slots,
                                          const int32_t *lens, void *stream)
{
    if (!c || n < 0 || (n > 0 && (!slots || !lens))) {
        set_error("pd_kv_cache_set_lens: bad argument");
        return PD_ERR_INVALID_ARG;
    }
    for (int i = 0; i < n; ++i) {
        if (slots[i] < 0 || slots[i] >= c->max_seqs || lens[i] < 0) {
            set_error("pd_kv_cache_set_lens: entry %d out of range", i);
            return PD_ERR_INVALID_ARG;
        }
        if (lens[i] > c->max_len) {
            set_error("pd_kv_cache_set_lens: len %d > max_len %d", lens[i], c->max_len);
            return PD_ERR_KV_CAPACITY;
        }
    }
    HIP_TRY(launch_scatter_ints(c->d_len, slots, lens, n, (hipStream_t)stream), PD_ERR_DEVICE);
    for (int i = 0; i < n; ++i) c->h_len[(size_t)slots[i]] = lens[i];
    return PD_OK;
}
