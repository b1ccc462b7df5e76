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
#include <type_traits>

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
constexpr float kLazy = 8.0f;
// s_waitcnt with only the vector-memory count set: at most n of the wave's loads still in flight
#define PD_ATT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (7 << 4) | (15 << 8) | (((n) >> 4) << 14))
constexpr int kAttnSplitGrid = 512;   // four-wave workgroups a split launch aims for: two per CU

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

//
// SPLIT: the key tiles of a query block are divided over gridDim.y workgroups, each of which
// leaves its unnormalised O (fp32), running max and sum in part_o / part_ml for
// attn_split_reduce_kernel.  For chunked prefill with few query blocks and a long prefix, where
// the unsplit grid fills a fraction of the chip with long serial walks.
//
// NW: waves per workgroup.  Four waves are the 128 queries of one head; eight are the same 128
// queries of two neighbouring heads of one K/V group, which halves the K/V bytes the L2 has to
// deliver per flop (at 128 queries per tile that delivery, not the matrix pipe, sets the pace).
template <bool SPLIT, int NW>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void attn_prefill_mfma_kernel(AttnArgs a,
                                                                   const uint16_t *__restrict__ vt,
                                                                   int vt_ld,
                                                                   const int32_t *__restrict__ pad_cu,
                                                                   float *__restrict__ part_o,
                                                                   float *__restrict__ part_ml)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // Workgroups are dispatched in index order and a query block's work grows with its position in
    // the sequence (causal), so the index runs over the query blocks from the last one down, and
    // inside one block position over all (sequence, head) pairs: the longest workgroups start first
    // and the chip drains on the shortest ones.  Heads of a group are neighbours and share K / V in
    // the L2.
    constexpr int HPW = NW / 4;                    // heads per workgroup
    constexpr int NST = NW == 8 ? 4 : 2;           // stages of the K / V^T ring in the LDS
    constexpr int AHEAD = NST - 1;                 // tiles requested ahead of the one being computed
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: the tile tests below are wave-uniform branches
    const int wq = wave & 3;                       // the wave's 32 queries of the block
    const int hgroups = a.Hq / HPW;
    const int per_qb = hgroups * a.n_seqs;
    const int rank = blockIdx.x / per_qb, rest = blockIdx.x - rank * per_qb;
    const int seq = rest / hgroups, head = (rest - seq * hgroups) * HPW + (wave >> 2);
    const int s0 = a.d_cu[seq], L = a.d_cu[seq + 1] - s0;
    const int P = a.prefix ? a.prefix[seq] : 0;    // keys ahead of the first query (chunked prefill)
    const int Lk = P + L;                          // keys of the sequence
    const int nqb = (L + BQ - 1) / BQ;
    const int qb = (int)(gridDim.x / per_qb) - 1 - rank;   // block position, counted from the longest sequence's last
    if (qb >= nqb) return;
    const int q0 = qb * BQ;
    const int g = head / (a.Hq / a.Hkv);
    const int n = lane & 31, h = lane >> 5;
    const uint16_t *qkv = (const uint16_t *)a.qkv;
    const int ld = a.ld;

    // ---- Q fragments (B operand): query row q0 + 32*wave + n, 8 k-steps of 16 channels ------------
    bf16x8 qf[8];
    {
        int qr = q0 + wq * 32 + n;
        if (qr >= L) qr = L - 1;
        const uint16_t *qp = qkv + (size_t)(s0 + qr) * ld + head * HD + h * 8;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) qf[kk] = *(const bf16x8 *)(qp + kk * 16);
    }

    // ---- tile loaders ------------------------------------------------------------------------------
    // K tile: 64 rows x 16 slots; one wave instruction = 4 rows; wave w issues rows 4*(NW*i + w) ..
    // V^T tile: 128 rows x 8 slots; one wave instruction = 8 rows; wave w issues rows 8*(NW*i + w) ..
    const char *kbase = a.kx ? (const char *)((const uint16_t *)a.kx + (size_t)a.k_cu[seq] * a.kx_ld + g * HD)
                             : (const char *)(qkv + (size_t)s0 * ld + (a.Hq + g) * HD);
    const size_t k_stride = (size_t)(a.kx ? a.kx_ld : ld) * 2;
    const char *vbase = (const char *)(vt + (size_t)g * HD * vt_ld + pad_cu[seq]);
    // A lane's byte offsets from the tile's first key row / first V^T column do not change from
    // tile to tile: the tile's position goes into the (scalar) base, and the offsets of the last,
    // possibly ragged tile (rows clamped) are a second set chosen by a uniform select, so every
    // tile issues the same instructions.
    const int q_hi_blk = min(q0 + BQ, L);          // keys needed: 0 .. P + q_hi_blk - 1
    const int n_tiles = (P + q_hi_blk + BKV - 1) / BKV;
    constexpr int LPW = 16 / NW;                   // load instructions per wave for each of K and V^T
    constexpr int LPT = 2 * LPW;                   // ... per tile
    uint32_t k_off[LPW], k_off_last[LPW], v_off[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int r = 4 * (NW * i + wave) + (lane >> 4);
        const uint32_t k_chunk = ((lane & 15) ^ (r & 15)) * 16;
        k_off[i] = (uint32_t)r * (uint32_t)k_stride + k_chunk;
        // rows of the last tile past the last key read that key's row again (masked by causality)
        const int r_last = min(r, Lk - 1 - (n_tiles - 1) * BKV);
        k_off_last[i] = (uint32_t)r_last * (uint32_t)k_stride + k_chunk;
        int d = 8 * (NW * i + wave) + (lane >> 3);
        int c = (lane & 7) ^ ((d >> 1) & 7);
        v_off[i] = (uint32_t)d * (uint32_t)(vt_ld * 2) + c * 16;
    }
    auto issue_loads = [&](int j, unsigned char *st) {
        const int k0 = j * BKV;
        const bool last = j == n_tiles - 1;        // the only tile that can reach past the last key
        const char *kb = kbase + (size_t)k0 * k_stride;
#pragma unroll
        for (int i = 0; i < LPW; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t)(kb + (last ? k_off_last[i] : k_off[i])),
                                             (lptr_t)(st + 4 * (NW * i + wave) * 256), 16, 0, 0);
        const char *vb = vbase + (size_t)k0 * 2;
#pragma unroll
        for (int i = 0; i < LPW; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t)(vb + v_off[i]),
                                             (lptr_t)(st + K_BYTES + 8 * (NW * i + wave) * 128), 16, 0, 0);
    };

    f32x16 oacc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
    // log2-domain running max; this half's sum.  A split may see no visible key for a query: a
    // finite floor keeps its rescale factors defined (exp2(-inf - -inf) is not) and weighs nothing.
    float m_run = SPLIT ? -1e30f : -INFINITY, l_run = 0.f;
    const float sl2e = a.scale * 1.4426950408889634f;

    // last visible key of this wave's first / last query and of this lane's query
    const int wq_lo = P + q0 + wq * 32, wq_hi = wq_lo + 31;
    const int my_q = q0 + wq * 32 + n;
    const int my_last = P + my_q;

    const int t_lo = SPLIT ? (int)(((long)blockIdx.y * n_tiles) / gridDim.y) : 0;
    const int t_hi = SPLIT ? (int)(((long)(blockIdx.y + 1) * n_tiles) / gridDim.y) : n_tiles;
    // One tile out of stage STG of the ring (a compile-time constant, so the LDS addresses of the
    // fragment reads are a per-lane register plus an immediate).  Loads retire in order: once at
    // most the requests of the AHEAD - 1 later tiles are in flight, this wave's part of tile j has
    // landed; after the barrier every wave's part has, and every wave has finished tile j - 1, whose
    // stage the request for tile j + AHEAD overwrites.  Past the last tile the last one is requested
    // again, so that the count in flight stays the same to the end.
    auto tile = [&](const int j, auto STG) {
        constexpr int stg = decltype(STG)::value;
        const unsigned char *st = smem + stg * ASTAGE;
        PD_ATT_VMCNT((AHEAD - 1) * LPT);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        issue_loads(min(j + AHEAD, t_hi - 1), smem + ((stg + AHEAD) % NST) * ASTAGE);
        __builtin_amdgcn_sched_barrier(0);
        const int k0 = j * BKV;
        if (k0 <= wq_hi) {                          // wave-uniform: some key of the tile is visible
            // ---- S^T = K Q^T -----------------------------------------------------------------------
            // All 16 K fragments are requested before the first MFMA (one LDS round trip per tile,
            // which the SIMD's other wave covers); the 16 V^T fragments are requested right behind
            // the MFMAs and land while the softmax runs.  Left to itself the compiler reads each
            // fragment right before the MFMA that consumes it and drains the LDS queue every time.
            f32x16 sacc[2];
            bf16x8 kf[16], vf[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int row = 32 * (i >> 3) + n, c = 2 * (i & 7) + h;
                kf[i] = *(const bf16x8 *)(st + row * 256 + ((c ^ (row & 15)) * 16));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[b][r] = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i)
                sacc[i >> 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i], qf[i & 7], sacc[i >> 3], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int row = 32 * (i >> 2) + n, c = 2 * (i & 3) + h;   // c = 4 b + 2 sstep + h
                vf[i] = *(const bf16x8 *)(st + K_BYTES + row * 128 + ((c ^ ((row >> 1) & 7)) * 16));
            }
            __builtin_amdgcn_sched_barrier(0);
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
            {   // the query's other 32 keys sit in lane + 32: exchanged in registers, since an LDS shuffle
                // would queue behind the V^T fragment reads
                const unsigned mb = __builtin_bit_cast(unsigned, mx);
                auto sw = __builtin_amdgcn_permlane32_swap(mb, mb, false, false);
                mx = fmaxf(__builtin_bit_cast(float, (unsigned)sw[0]), __builtin_bit_cast(float, (unsigned)sw[1]));
            }
            // The running max is raised only when some query of the wave outgrows it by more than
            // kLazy (log2 units): probabilities then reach 2^kLazy at most, which fp32 sums and bf16
            // operands hold without loss, and the rescale of O is skipped on most tiles.
            const float m_cand = fmaxf(m_run, mx * sl2e);  // finite: key 0 is visible to every query (or the floor)
            if (__any(m_cand - m_run > kLazy)) {
                const float alpha = fast_exp2(m_run - m_cand);
                m_run = m_cand;
                l_run *= alpha;
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
            }
            float psum = 0.f;
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float p = fast_exp2(fmaf(sacc[b][r], sl2e, -m_run));
                    sacc[b][r] = p;
                    psum += p;
                }
            l_run += psum;
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
            for (int i = 0; i < 16; ++i)
                oacc[i >> 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i], pf[(i >> 1) & 1][i & 1], oacc[i >> 2], 0, 0, 0);
        }
    };
    if (t_lo < t_hi) {
#pragma unroll
        for (int p = 0; p < AHEAD; ++p) {
            issue_loads(min(t_lo + p, t_hi - 1), smem + p * ASTAGE);
            __builtin_amdgcn_sched_barrier(0);
        }
        for (int j = t_lo; j < t_hi; j += NST) {
            tile(j, std::integral_constant<int, 0>{});
            if (j + 1 < t_hi) tile(j + 1, std::integral_constant<int, 1>{});
            if (NST == 4) {
                if (j + 2 < t_hi) tile(j + 2, std::integral_constant<int, 2 % NST>{});
                if (j + 3 < t_hi) tile(j + 3, std::integral_constant<int, 3 % NST>{});
            }
        }
        PD_ATT_VMCNT(0);                           // the repeated requests of the last tile: none may outlive the workgroup's LDS
    }

    // ---- normalise and store: lane holds query my_q, channels 32*db + 8*(r/4) + 4*h + r%4 -------------
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (SPLIT) {
        if (my_q < L) {
            const size_t row = ((size_t)blockIdx.y * a.T + (s0 + my_q)) * a.Hq + head;
            float *op = part_o + row * HD;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    *(float4 *)(op + 32 * db + 8 * q4 + 4 * h) =
                        make_float4(oacc[db][4 * q4 + 0], oacc[db][4 * q4 + 1], oacc[db][4 * q4 + 2],
                                    oacc[db][4 * q4 + 3]);
            if (h == 0) *(float2 *)(part_ml + row * 2) = make_float2(m_run, l_tot);
        }
        return;
    }
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

// Merges the partial results of the split kernel: out[row] = sum_s 2^(m_s - m) O_s / sum_s 2^(m_s - m) l_s
// with m = max_s m_s, row = (token, head).  32 threads per row, 4 channels each.
__global__ __launch_bounds__(256) void attn_split_reduce_kernel(const float *__restrict__ part_o,
                                                                const float *__restrict__ part_ml,
                                                                int n_split, int rows, uint16_t *__restrict__ o)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    const int row = idx >> 5, c4 = (idx & 31) * 4;
    if (row >= rows) return;
    float m = -INFINITY;
    for (int s = 0; s < n_split; ++s) m = fmaxf(m, part_ml[((size_t)s * rows + row) * 2]);
    float l = 0.f, acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < n_split; ++s) {
        const float2 ml = *(const float2 *)(part_ml + ((size_t)s * rows + row) * 2);
        const float w = fast_exp2(ml.x - m);
        const float4 v = *(const float4 *)(part_o + ((size_t)s * rows + row) * HD + c4);
        l += w * ml.y;
        acc[0] += w * v.x; acc[1] += w * v.y; acc[2] += w * v.z; acc[3] += w * v.w;
    }
    const float inv = 1.0f / l;
    uint2 w;
    w.x = pack2bf(acc[0] * inv, acc[1] * inv);
    w.y = pack2bf(acc[2] * inv, acc[3] * inv);
    *(uint2 *)(o + (size_t)row * HD + c4) = w;
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

// Eight-wave workgroups (two heads share the K/V tiles) whenever a K/V group has an even number of heads.
static bool attn_two_heads(const AttnArgs &a) { return (a.Hq / a.Hkv) % 2 == 0; }

static hipError_t attn_kernel_attrs()
{
    static OncePerDevice attr;
    int dev;
    if (!attr.need(&dev)) return hipSuccess;
    const void *fns[4] = {(const void *)attn_prefill_mfma_kernel<false, 4>, (const void *)attn_prefill_mfma_kernel<true, 4>,
                          (const void *)attn_prefill_mfma_kernel<false, 8>, (const void *)attn_prefill_mfma_kernel<true, 8>};
    for (const void *f : fns) {
        hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 4 * ASTAGE);
        if (e != hipSuccess) return e;
    }
    attr.mark(dev);
    return hipSuccess;
}

template <bool SPLIT>
static hipError_t launch_attn_kernel(const AttnArgs &a, const uint16_t *vt, int vt_ld, const int32_t *pad_cu,
                                     int n_split, float *part_o, float *part_ml, hipStream_t s)
{
    hipError_t e = attn_kernel_attrs();
    if (e != hipSuccess) return e;
    const int nqb = (a.max_seq_len + BQ - 1) / BQ;
    if (attn_two_heads(a))
        attn_prefill_mfma_kernel<SPLIT, 8><<<dim3((unsigned)(nqb * (a.Hq / 2) * a.n_seqs), (unsigned)n_split), 512,
                                             4 * ASTAGE, s>>>(a, vt, vt_ld, pad_cu, part_o, part_ml);
    else
        attn_prefill_mfma_kernel<SPLIT, 4><<<dim3((unsigned)(nqb * a.Hq * a.n_seqs), (unsigned)n_split), 256,
                                             2 * ASTAGE, s>>>(a, vt, vt_ld, pad_cu, part_o, part_ml);
    return hipGetLastError();
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
    return launch_attn_kernel<false>(a, vt, vt_ld, pad_cu, 1, nullptr, nullptr, s);
}

int attn_chunk_splits(const AttnArgs &a, int max_keys)
{
    // one round of workgroups: two four-wave or one eight-wave workgroup per CU
    const bool two = attn_two_heads(a);
    const int grid = (a.max_seq_len + BQ - 1) / BQ * (two ? a.Hq / 2 : a.Hq) * a.n_seqs;
    const int tiles = (max_keys + BKV - 1) / BKV;
    int n = (two ? kAttnSplitGrid / 2 : kAttnSplitGrid) / grid;
    if (n > tiles / 8) n = tiles / 8;              // at least eight key tiles per split
    if (n > 8) n = 8;
    return n < 2 ? 1 : n;
}

size_t attn_chunk_split_bytes(const AttnArgs &a, int n_split)
{
    return n_split < 2 ? 0 : (size_t)n_split * a.T * a.Hq * (HD + 2) * sizeof(float);
}

hipError_t launch_attn_chunk_mfma(const AttnArgs &a_in, const int32_t *d_slots, uint16_t *kx, uint16_t *vt,
                                  int vt_ld, const int32_t *pad_cu, int n_split, float *part, hipStream_t s)
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
    if (n_split < 2) return launch_attn_kernel<false>(a, vt, vt_ld, pad_cu, 1, nullptr, nullptr, s);
    const int rows = a.T * a.Hq;
    float *part_ml = part + (size_t)n_split * rows * HD;
    e = launch_attn_kernel<true>(a, vt, vt_ld, pad_cu, n_split, part, part_ml, s);
    if (e != hipSuccess) return e;
    attn_split_reduce_kernel<<<dim3((unsigned)((rows * 32 + 255) / 256)), 256, 0, s>>>(part, part_ml, n_split, rows,
                                                                                       (uint16_t *)a.o);
    return hipGetLastError();
}

}  // namespace pd
