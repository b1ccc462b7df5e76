// Causal grouped-query prefill attention for head_dim = 128, bf16, on the matrix cores.
//
// One workgroup (4 waves) owns 128 consecutive queries of one (sequence, query head); each wave
// owns 32 of them.  Keys/values are walked in tiles of 64 with an online softmax.  Everything is
// computed transposed so that no register shuffling is needed between the two contractions:
//
//   S^T[key, query] = K[key, :] . Q[query, :]      A operand = K rows from LDS, B operand = Q rows
//                                                  (held in registers for the whole kernel)
//   O^T[d, query]   = V^T[d, key] . P^T[key, query] A operand = rows of V^T from LDS, B operand =
//                                                  exp'd scores straight from the S^T accumulators
//
// In both accumulators a lane's column is one query, so the running max / sum are per-lane
// scalars and rescaling is a lane-local multiply.  A lane of the S^T accumulator holds keys
// {4h..4h+3, 8+4h..8+4h+3} of every 16 (h = lane / 32); one v_permlane32_swap per register pair
// turns that into the 8 consecutive keys the B operand wants.
//
// K tiles are read from the projection buffer and V^T tiles from a transposed copy of V made by
// v_transpose_kernel (sequence starts padded to 64 so every tile row is 16-byte aligned and
// zero-filled past the sequence end).  Both arrive with direct-to-LDS loads, XOR-swizzled on
// the global side like the GEMM, double buffered, one barrier per tile.
#include "pd_internal.h"

namespace pd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef const void __attribute__((address_space(1))) *gptr_t;
typedef void __attribute__((address_space(3))) *lptr_t;

constexpr int HD = 128, BQ = 128, BKV = 64;
constexpr int K_BYTES = BKV * HD * 2;   // 64 rows of 256 B
constexpr int V_BYTES = HD * BKV * 2;   // 128 rows of 128 B
constexpr int ASTAGE = K_BYTES + V_BYTES;

// ---------------------------------------------------------------------------------------------
// vt[g][d][pad_cu[s] + p] = V[token cu[s] + p][g][d]; zero for padded positions p >= L_s.
// Block = 64 padded positions of one kv head.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void v_transpose_kernel(const uint16_t *__restrict__ qkv, int ld,
                                                          int v_col0, const int32_t *__restrict__ cu,
                                                          const int32_t *__restrict__ pad_cu,
                                                          int n_seqs, uint16_t *__restrict__ vt,
                                                          int vt_ld)
{
    __shared__ uint16_t tile[64][HD + 2];
    const int p0 = blockIdx.x * 64, g = blockIdx.y;
    int lo = 0, hi = n_seqs;   // largest s with pad_cu[s] <= p0
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (pad_cu[mid] <= p0) lo = mid; else hi = mid;
    }
    const int s = lo;
    const int L = cu[s + 1] - cu[s];
    const int pos0 = p0 - pad_cu[s];
    for (int idx = threadIdx.x; idx < 64 * (HD / 8); idx += 256) {
        int r = idx / (HD / 8), c = idx % (HD / 8);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (pos0 + r < L)
            v = *(const uint4 *)(qkv + (size_t)(cu[s] + pos0 + r) * ld + v_col0 + g * HD + c * 8);
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            tile[r][c * 8 + 2 * j] = (uint16_t)(w[j] & 0xffffu);
            tile[r][c * 8 + 2 * j + 1] = (uint16_t)(w[j] >> 16);
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < HD * 8; idx += 256) {
        int d = idx >> 3, c = idx & 7;   // 8 positions per 16-byte chunk
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            w[j] = (uint32_t)tile[c * 8 + 2 * j][d] | ((uint32_t)tile[c * 8 + 2 * j + 1][d] << 16);
        *(uint4 *)(vt + ((size_t)g * HD + d) * vt_ld + p0 + c * 8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__global__ __launch_bounds__(256, 2) void attn_prefill_mfma_kernel(AttnArgs a,
                                                                   const uint16_t *__restrict__ vt,
                                                                   int vt_ld,
                                                                   const int32_t *__restrict__ pad_cu)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // Workgroups are dispatched in index order and a query block's work grows with its position in
    // the sequence (causal), so the index runs over the query blocks from the last one down, and
    // inside one block position over all (sequence, head) pairs: the longest workgroups start first
    // and the chip drains on the shortest ones.  Heads of a group are neighbours and share K / V in
    // the L2.
    const int per_qb = a.Hq * a.n_seqs;
    const int rank = blockIdx.x / per_qb, rest = blockIdx.x - rank * per_qb;
    const int seq = rest / a.Hq, head = rest - seq * a.Hq;
    const int s0 = a.d_cu[seq], L = a.d_cu[seq + 1] - s0;
    const int P = a.prefix ? a.prefix[seq] : 0;    // keys ahead of the first query (chunked prefill)
    const int Lk = P + L;                          // keys of the sequence
    const int nqb = (L + BQ - 1) / BQ;
    const int qb = (int)(gridDim.x / per_qb) - 1 - rank;   // block position, counted from the longest sequence's last
    if (qb >= nqb) return;
    const int q0 = qb * BQ;
    const int g = head / (a.Hq / a.Hkv);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, h = lane >> 5;
    const uint16_t *qkv = (const uint16_t *)a.qkv;
    const int ld = a.ld;

    // ---- Q fragments (B operand): query row q0 + 32*wave + n, 8 k-steps of 16 channels ------------
    bf16x8 qf[8];
    {
        int qr = q0 + wave * 32 + n;
        if (qr >= L) qr = L - 1;
        const uint16_t *qp = qkv + (size_t)(s0 + qr) * ld + head * HD + h * 8;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) qf[kk] = *(const bf16x8 *)(qp + kk * 16);
    }

    // ---- tile loaders ------------------------------------------------------------------------------
    // K tile: 64 rows x 16 slots; one wave instruction = 4 rows; wave w issues rows 16*i + 4*w ..
    // V^T tile: 128 rows x 8 slots; one wave instruction = 8 rows; wave w issues rows 32*i + 8*w ..
    const char *kbase = a.kx ? (const char *)((const uint16_t *)a.kx + (size_t)a.k_cu[seq] * a.kx_ld + g * HD)
                             : (const char *)(qkv + (size_t)s0 * ld + (a.Hq + g) * HD);
    const size_t k_stride = (size_t)(a.kx ? a.kx_ld : ld) * 2;
    const char *vbase = (const char *)(vt + (size_t)g * HD * vt_ld + pad_cu[seq]);
    uint32_t k_row[4], k_chunk[4], v_off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int r = 16 * i + 4 * wave + (lane >> 4);
        k_row[i] = r;
        k_chunk[i] = ((lane & 15) ^ (r & 15)) * 16;
        int d = 32 * i + 8 * wave + (lane >> 3);
        int c = (lane & 7) ^ ((d >> 1) & 7);
        v_off[i] = (uint32_t)d * (uint32_t)(vt_ld * 2) + c * 16;
    }
    auto issue_loads = [&](int j, unsigned char *st) {
        const int k0 = j * BKV;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int kr = k0 + (int)k_row[i];
            if (kr >= Lk) kr = Lk - 1;             // clamped rows are masked by causality
            __builtin_amdgcn_global_load_lds((gptr_t)(kbase + (size_t)kr * k_stride + k_chunk[i]),
                                             (lptr_t)(st + (16 * i + 4 * wave) * 256), 16, 0, 0);
        }
        const char *vb = vbase + (size_t)k0 * 2;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t)(vb + v_off[i]),
                                             (lptr_t)(st + K_BYTES + (32 * i + 8 * wave) * 128), 16, 0, 0);
    };

    f32x16 oacc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;          // log2-domain running max; this half's sum
    const float sl2e = a.scale * 1.4426950408889634f;

    const int q_hi_blk = min(q0 + BQ, L);          // keys needed: 0 .. P + q_hi_blk - 1
    const int n_tiles = (P + q_hi_blk + BKV - 1) / BKV;
    // last visible key of this wave's first / last query and of this lane's query
    const int wq_lo = P + q0 + wave * 32, wq_hi = wq_lo + 31;
    const int my_q = q0 + wave * 32 + n;
    const int my_last = P + my_q;

    issue_loads(0, smem);
    __syncthreads();
    for (int j = 0; j < n_tiles; ++j) {
        const unsigned char *st = smem + (j & 1) * ASTAGE;
        if (j + 1 < n_tiles) issue_loads(j + 1, smem + ((j + 1) & 1) * ASTAGE);
        const int k0 = j * BKV;
        if (k0 <= wq_hi) {                          // wave-uniform: some key of the tile is visible
            // ---- S^T = K Q^T -----------------------------------------------------------------------
            f32x16 sacc[2];
#pragma unroll
            for (int b = 0; b < 2; ++b) {
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[b][r] = 0.f;
                const int row = 32 * b + n;
#pragma unroll
                for (int kk = 0; kk < 8; ++kk) {
                    const int c = 2 * kk + h;
                    bf16x8 kf = *(const bf16x8 *)(st + row * 256 + ((c ^ (row & 15)) * 16));
                    sacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sacc[b], 0, 0, 0);
                }
            }
            // ---- online softmax (log2 domain): p = 2^(s * scale*log2e - m) ---------------------------
            if (k0 + BKV - 1 > wq_lo) {            // wave-uniform: only tiles on the diagonal are masked
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = k0 + 32 * b + 8 * (r >> 2) + 4 * h + (r & 3);
                        if (key > my_last) sacc[b][r] = -INFINITY;
                    }
            }
            float mx = -INFINITY;
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[b][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run, mx * sl2e);   // finite: key 0 is visible to every query
            const float alpha = fast_exp2(m_run - m_new);
            m_run = m_new;
            float psum = 0.f;
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float p = fast_exp2(fmaf(sacc[b][r], sl2e, -m_new));
                    sacc[b][r] = p;
                    psum += p;
                }
            l_run = l_run * alpha + psum;
            if (__any(alpha != 1.0f)) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
            }
            // ---- P^T as B operand: pack to bf16, then swap halves so each lane holds 8 consecutive keys
            bf16x8 pf[2][2];
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int sstep = 0; sstep < 2; ++sstep) {
                    const int r0 = 8 * sstep;
                    unsigned x0 = pack2bf(sacc[b][r0 + 0], sacc[b][r0 + 1]);
                    unsigned x1 = pack2bf(sacc[b][r0 + 2], sacc[b][r0 + 3]);
                    unsigned y0 = pack2bf(sacc[b][r0 + 4], sacc[b][r0 + 5]);
                    unsigned y1 = pack2bf(sacc[b][r0 + 6], sacc[b][r0 + 7]);
                    auto s0v = __builtin_amdgcn_permlane32_swap(x0, y0, false, false);
                    auto s1v = __builtin_amdgcn_permlane32_swap(x1, y1, false, false);
                    u32x4 packed = {s0v[0], s1v[0], s0v[1], s1v[1]};
                    pf[b][sstep] = __builtin_bit_cast(bf16x8, packed);
                }
            // ---- O^T += V^T P^T ------------------------------------------------------------------------
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const int row = 32 * db + n;
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int sstep = 0; sstep < 2; ++sstep) {
                        const int c = 4 * b + 2 * sstep + h;
                        bf16x8 vf = *(const bf16x8 *)(st + K_BYTES + row * 128 + ((c ^ ((row >> 1) & 7)) * 16));
                        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[b][sstep], oacc[db], 0, 0, 0);
                    }
            }
        }
        __syncthreads();
    }

    // ---- normalise and store: lane holds query my_q, channels 32*db + 8*(r/4) + 4*h + r%4 -------------
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_tot;
    if (my_q < L) {
        uint16_t *op = (uint16_t *)a.o + (size_t)(s0 + my_q) * (a.Hq * HD) + head * HD;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                uint2 w;
                w.x = pack2bf(oacc[db][4 * q4 + 0] * inv, oacc[db][4 * q4 + 1] * inv);
                w.y = pack2bf(oacc[db][4 * q4 + 2] * inv, oacc[db][4 * q4 + 3] * inv);
                *(uint2 *)(op + 32 * db + 8 * q4 + 4 * h) = w;
            }
    }
}

// Chunked prefill: keys and values of positions 0 .. prefix[s] + L_s - 1 of every sequence's cache
// slot, out of the blocked cache, as plain key rows kx[pad_cu[s] + pos][Hkv*128] and transposed
// values vt[g][d][pad_cu[s] + pos] (zero past the end).  One block = 64 positions of one kv head.
__global__ __launch_bounds__(256) void kv_gather_blocked_kernel(const uint16_t *__restrict__ kc,
                                                                const uint16_t *__restrict__ vc,
                                                                size_t plane, const int32_t *__restrict__ slots,
                                                                const int32_t *__restrict__ cu,
                                                                const int32_t *__restrict__ prefix,
                                                                const int32_t *__restrict__ pad_cu, int n_seqs,
                                                                int Hkv, uint16_t *__restrict__ kx,
                                                                uint16_t *__restrict__ vt, int vt_ld)
{
    const int p0 = blockIdx.x * 64, g = blockIdx.y;
    int lo = 0, hi = n_seqs;   // largest s with pad_cu[s] <= p0
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (pad_cu[mid] <= p0) lo = mid; else hi = mid;
    }
    const int s = lo;
    const int Lk = prefix[s] + cu[s + 1] - cu[s];
    const int pos0 = p0 - pad_cu[s];               // a multiple of 64
    const uint16_t *kp = kc + ((size_t)slots[s] * Hkv + g) * plane;
    const uint16_t *vp = vc + ((size_t)slots[s] * Hkv + g) * plane;
    const int tid = threadIdx.x;
    // keys: 64 positions x 16 chunks of 8 channels
    for (int e = tid; e < 64 * 16; e += 256) {
        const int r = e >> 4, c8 = (e & 15) * 8;
        if (pos0 + r < Lk)
            *(uint4 *)(kx + (size_t)(p0 + r) * (Hkv * HD) + g * HD + c8) =
                *(const uint4 *)(kp + kblk_off(pos0 + r, c8));
    }
    // values: vt row d, 64 consecutive positions = two cache blocks of 32 positions, whose 32
    // entries per channel are stored in the order sigma(16a + 4q + j) = 8q + 4a + j
    for (int e = tid; e < HD * 8; e += 256) {
        const int d = e >> 3, c8 = (e & 7) * 8;    // positions pos0 + c8 .. + 7
        uint16_t w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int pos = pos0 + c8 + j;
            w[j] = pos < Lk ? vp[vblk_off(pos, d)] : (uint16_t)0;
        }
        uint4 o;
        o.x = w[0] | ((uint32_t)w[1] << 16); o.y = w[2] | ((uint32_t)w[3] << 16);
        o.z = w[4] | ((uint32_t)w[5] << 16); o.w = w[6] | ((uint32_t)w[7] << 16);
        *(uint4 *)(vt + ((size_t)g * HD + d) * vt_ld + p0 + c8) = o;
    }
}

// The same gather out of the 8-bit E4M3 blocked cache: codes are expanded to bf16 (code * scale).
__global__ __launch_bounds__(256) void kv_gather_blocked_fp8_kernel(
    const uint8_t *__restrict__ kc, const uint8_t *__restrict__ vc, size_t plane,
    const int32_t *__restrict__ slots, const int32_t *__restrict__ cu, const int32_t *__restrict__ prefix,
    const int32_t *__restrict__ pad_cu, int n_seqs, int Hkv, uint16_t *__restrict__ kx,
    uint16_t *__restrict__ vt, int vt_ld, float k_scale, float v_scale)
{
    const int p0 = blockIdx.x * 64, g = blockIdx.y;
    int lo = 0, hi = n_seqs;   // largest s with pad_cu[s] <= p0
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (pad_cu[mid] <= p0) lo = mid; else hi = mid;
    }
    const int s = lo;
    const int Lk = prefix[s] + cu[s + 1] - cu[s];
    const int pos0 = p0 - pad_cu[s];               // a multiple of 64
    const uint8_t *kp = kc + ((size_t)slots[s] * Hkv + g) * plane;
    const uint8_t *vp = vc + ((size_t)slots[s] * Hkv + g) * plane;
    const int tid = threadIdx.x;
    // keys: 64 positions x 16 runs of 8 channels (8 consecutive bytes of the cache)
    for (int e = tid; e < 64 * 16; e += 256) {
        const int r = e >> 4, c8 = (e & 15) * 8;
        if (pos0 + r < Lk) {
            const uint2 w = *(const uint2 *)(kp + kblk8_off(pos0 + r, c8));
            uint4 o;
            auto f = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.x, false);
            o.x = pack2bf(f[0] * k_scale, f[1] * k_scale);
            f = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.x, true);
            o.y = pack2bf(f[0] * k_scale, f[1] * k_scale);
            f = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.y, false);
            o.z = pack2bf(f[0] * k_scale, f[1] * k_scale);
            f = __builtin_amdgcn_cvt_pk_f32_fp8((int)w.y, true);
            o.w = pack2bf(f[0] * k_scale, f[1] * k_scale);
            *(uint4 *)(kx + (size_t)(p0 + r) * (Hkv * HD) + g * HD + c8) = o;
        }
    }
    // values: vt row d, 8 consecutive positions per thread
    for (int e = tid; e < HD * 8; e += 256) {
        const int d = e >> 3, c8 = (e & 7) * 8;    // positions pos0 + c8 .. + 7
        float w[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int pos = pos0 + c8 + j;
            w[j] = pos < Lk ? e4m3_decode(vp[vblk8_off(pos, d)]) * v_scale : 0.f;
        }
        uint4 o;
        o.x = pack2bf(w[0], w[1]); o.y = pack2bf(w[2], w[3]);
        o.z = pack2bf(w[4], w[5]); o.w = pack2bf(w[6], w[7]);
        *(uint4 *)(vt + ((size_t)g * HD + d) * vt_ld + p0 + c8) = o;
    }
}

bool attn_prefill_mfma_supported(const AttnArgs &a)
{
    return a.hd == HD && !a.decode && a.ld % 8 == 0 && a.T > 0 &&
           (int64_t)a.T * a.ld * 2 < (1ll << 31);
}

// vt: transposed-V scratch [Hkv][128][vt_ld]; pad_cu: device [n_seqs+1] padded sequence starts.
hipError_t launch_attn_prefill_mfma(const AttnArgs &a, uint16_t *vt, int vt_ld, const int32_t *pad_cu,
                                    hipStream_t s)
{
    v_transpose_kernel<<<dim3(vt_ld / 64, a.Hkv), 256, 0, s>>>((const uint16_t *)a.qkv, a.ld,
                                                               (a.Hq + a.Hkv) * HD, a.d_cu, pad_cu,
                                                               a.n_seqs, vt, vt_ld);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    static bool attr_set = false;
    const int smem = 2 * ASTAGE;
    if (!attr_set) {
        e = hipFuncSetAttribute((const void *)attn_prefill_mfma_kernel,
                                hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int nqb = (a.max_seq_len + BQ - 1) / BQ;
    attn_prefill_mfma_kernel<<<dim3((unsigned)(nqb * a.Hq * a.n_seqs)), 256, smem, s>>>(a, vt, vt_ld, pad_cu);
    return hipGetLastError();
}

hipError_t launch_attn_chunk_mfma(const AttnArgs &a_in, const int32_t *d_slots, uint16_t *kx, uint16_t *vt,
                                  int vt_ld, const int32_t *pad_cu, hipStream_t s)
{
    AttnArgs a = a_in;
    if (a.kv_fp8)
        kv_gather_blocked_fp8_kernel<<<dim3(vt_ld / 64, a.Hkv), 256, 0, s>>>(
            (const uint8_t *)a.k_cache, (const uint8_t *)a.v_cache, (size_t)a.max_len * HD, d_slots, a.d_cu,
            a.prefix, pad_cu, a.n_seqs, a.Hkv, kx, vt, vt_ld, a.k_scale, a.v_scale);
    else
        kv_gather_blocked_kernel<<<dim3(vt_ld / 64, a.Hkv), 256, 0, s>>>(
            (const uint16_t *)a.k_cache, (const uint16_t *)a.v_cache, (size_t)a.max_len * HD, d_slots, a.d_cu,
            a.prefix, pad_cu, a.n_seqs, a.Hkv, kx, vt, vt_ld);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    a.kx = kx;
    a.kx_ld = a.Hkv * HD;
    a.k_cu = pad_cu;
    static bool attr_set = false;
    const int smem = 2 * ASTAGE;
    if (!attr_set) {
        e = hipFuncSetAttribute((const void *)attn_prefill_mfma_kernel,
                                hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int nqb = (a.max_seq_len + BQ - 1) / BQ;
    attn_prefill_mfma_kernel<<<dim3((unsigned)(nqb * a.Hq * a.n_seqs)), 256, smem, s>>>(a, vt, vt_ld, pad_cu);
    return hipGetLastError();
}

}  // namespace pd
