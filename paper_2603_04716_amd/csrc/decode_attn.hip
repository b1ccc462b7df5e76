// Decode attention (one query token per sequence) over the blocked bf16 KV cache, head_dim 128.
//
// The step is bound by streaming the cache from HBM once, so the kernel is organised around the
// loads: one wavefront is an independent worker that owns a chunk of consecutive keys of one
// (sequence, kv head) and serves all query heads of that GQA group at once, so every cache byte
// is fetched exactly once.  Thanks to the blocked layout each 16-byte-per-lane load instruction
// reads 1 KB of contiguous memory straight into MFMA operand registers: no LDS, no barriers.
// The score and value contractions run on v_mfma_f32_16x16x32_bf16 with the (up to 16) query
// heads of the group as the N dimension; that wastes matrix-core columns, which are free here.
//
//   S^T[key, q] = K[key, :] . Q[q, :]       A = keys (16 per block), B = the group's query rows
//   O^T[d, q]   = V^T[d, key] . P^T[key, q] A = transposed value block, B = exp'd scores taken
//                                           from the S^T accumulators in place
//
// Workers write un-normalised partial outputs with their running max and sum; a small merge
// kernel combines the chunks of each (sequence, head).  A sequence of n keys is cut into
// ceil(n / chunk_keys) chunks of equal size (rounded up to 64 keys); the caller picks chunk_keys
// so that a launch has enough workers to saturate the memory system and no more (each extra
// chunk costs a start-up and a row of partials to merge).
#include "pd_internal.h"

namespace pd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float dexp2(float x) { return __builtin_amdgcn_exp2f(x); }

// One block: pos / len update and the prefix sum of chunks per sequence (B <= 4096).  BYVAL: the
// slots arrive in the kernel arguments (B <= 256) and are also stored to slots_out for the kernels
// that follow, which saves the separate upload launch of a small decode step.
template <bool BYVAL>
__device__ __forceinline__ void decode_meta_chunks_body(const int32_t *__restrict__ slots, const IntChunk &sv,
                                                        int32_t *slots_out, int B, int32_t *len, int32_t *pos,
                                                        int32_t *chunk_cu, int32_t *chunk_seq, int chunk_keys,
                                                        int *wave_tot)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int cnt[4], sum = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int b = tid * 4 + i;
        cnt[i] = 0;
        if (b < B) {
            int s;
            if (BYVAL) {
                s = sv.v[b];
                slots_out[b] = s;
            } else {
                s = slots[b];
            }
            int p = len[s];
            pos[b] = p;
            len[s] = p + 1;
            cnt[i] = (p + 1 + chunk_keys - 1) / chunk_keys;
        }
        sum += cnt[i];
    }
    int inc = sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int v = __shfl_up(inc, off, 64);
        if (lane >= off) inc += v;
    }
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    int base = 0;
    for (int w = 0; w < wave; ++w) base += wave_tot[w];
    int run = base + inc - sum;
    if (tid == 0) chunk_cu[0] = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int b = tid * 4 + i;
        // the attention workers find their sequence with one load instead of a bisection of chunk_cu
        for (int c = run; c < run + cnt[i]; ++c) chunk_seq[c] = b;
        run += cnt[i];
        if (b < B) chunk_cu[b + 1] = run;
    }
}

template <bool BYVAL>
__global__ __launch_bounds__(1024) void decode_meta_chunks_kernel(const int32_t *__restrict__ slots, IntChunk sv,
                                                                  int32_t *slots_out, int B, int32_t *len,
                                                                  int32_t *pos, int32_t *chunk_cu, int32_t *chunk_seq,
                                                                  int chunk_keys)
{
    __shared__ int wave_tot[16];
    decode_meta_chunks_body<BYVAL>(slots, sv, slots_out, B, len, pos, chunk_cu, chunk_seq, chunk_keys, wave_tot);
}

// The bookkeeping of a decode step of up to 256 rows (block B) and the RMSNorm of its rows (blocks
// 0 .. B-1) in one launch: neither needs the other, and a launch of its own costs each of them more than
// the work itself.
__global__ __launch_bounds__(256) void decode_meta_norm_kernel(IntChunk sv, int32_t *slots_out, int B, int32_t *len,
                                                               int32_t *pos, int32_t *chunk_cu, int32_t *chunk_seq,
                                                               int chunk_keys,
                                                               const uint4 *__restrict__ x, const uint4 *__restrict__ g,
                                                               uint4 *__restrict__ y, int d8, float d_inv, float eps)
{
    __shared__ int wave_tot[16];
    __shared__ float red[4];
    if ((int)blockIdx.x == B) {
        decode_meta_chunks_body<true>(nullptr, sv, slots_out, B, len, pos, chunk_cu, chunk_seq, chunk_keys, wave_tot);
        return;
    }
    rmsnorm_bf16_row(x + (size_t)blockIdx.x * d8, g, y + (size_t)blockIdx.x * d8, d8, d_inv, eps, red);
}

hipError_t launch_decode_meta_norm(const int32_t *host_slots, int32_t *d_slots, int B, int32_t *d_len, int32_t *d_pos,
                                   int32_t *chunk_cu, int32_t *chunk_seq, int chunk_keys, const void *x, const void *g,
                                   void *y, int d, float eps, hipStream_t s)
{
    if (B > 256 || B < 1 || d % 8 != 0) return hipErrorInvalidValue;
    IntChunk sv;
    for (int i = 0; i < B; ++i) sv.v[i] = host_slots[i];
    decode_meta_norm_kernel<<<B + 1, 256, 0, s>>>(sv, d_slots, B, d_len, d_pos, chunk_cu, chunk_seq, chunk_keys, (const uint4 *)x,
                                                  (const uint4 *)g, (uint4 *)y, d / 8, 1.0f / (float)d, eps);
    return hipGetLastError();
}

hipError_t launch_decode_meta_chunks(const int32_t *d_slots, int B, int32_t *d_len, int32_t *d_pos,
                                     int32_t *chunk_cu, int32_t *chunk_seq, int chunk_keys, hipStream_t s)
{
    IntChunk none;
    none.v[0] = 0;
    decode_meta_chunks_kernel<false><<<1, 1024, 0, s>>>(d_slots, none, nullptr, B, d_len, d_pos, chunk_cu, chunk_seq, chunk_keys);
    return hipGetLastError();
}

hipError_t launch_decode_meta_chunks_upload(const int32_t *host_slots, int32_t *d_slots, int B, int32_t *d_len,
                                            int32_t *d_pos, int32_t *chunk_cu, int32_t *chunk_seq, int chunk_keys,
                                            hipStream_t s)
{
    if (B > 256) return hipErrorInvalidValue;
    IntChunk sv;
    for (int i = 0; i < B; ++i) sv.v[i] = host_slots[i];
    decode_meta_chunks_kernel<true><<<1, 256, 0, s>>>(nullptr, sv, d_slots, B, d_len, d_pos, chunk_cu, chunk_seq, chunk_keys);
    return hipGetLastError();
}

// 8 consecutive E4M3 codes (two words) -> one bf16 operand register set (every code is exact in bf16)
__device__ __forceinline__ bf16x8 fp8x8_to_bf16(unsigned w0, unsigned w1)
{
    auto f0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w0, false);
    auto f1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w0, true);
    auto f2 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w1, false);
    auto f3 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w1, true);
    u32x4 r = {pack2bf(f0[0], f0[1]), pack2bf(f1[0], f1[1]), pack2bf(f2[0], f2[1]), pack2bf(f3[0], f3[1])};
    return __builtin_bit_cast(bf16x8, r);
}

// FP8: the cache holds E4M3 codes in the 8-bit blocked layout (half the bytes per key); the codes are
// widened to bf16 in registers, the key scale is folded into the score scale and the value scale
// into the final normalisation.
// (cos, sin) of pos * inv_freq[i .. i + 3]: from the table, or in double beyond it (as the stand-alone
// rotary kernel does)
__device__ __forceinline__ void rope_factors4(const DecodeAttnArgs &a, int pos, int i, float (&c)[4], float (&s)[4])
{
    if (pos < a.rope_table_len) {
        const float4 *t = (const float4 *)(a.rope_table + (size_t)pos * 64 + i);
        const float4 t0 = t[0], t1 = t[1];
        c[0] = t0.x; s[0] = t0.y; c[1] = t0.z; s[1] = t0.w;
        c[2] = t1.x; s[2] = t1.y; c[3] = t1.z; s[3] = t1.w;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            double sv, cv;
            sincos((double)pos * a.inv_freq[i + e], &sv, &cv);
            c[e] = (float)cv;
            s[e] = (float)sv;
        }
    }
}

// ROPE (one-token step): q and the new key arrive unrotated and are rotated here; the new token is not
// read from the cache but joins the softmax from registers (see DecodeAttnArgs).  Storing it into the
// cache is left to a later launch of the step: the 2-byte stores into the transposed value blocks cost
// this kernel 19 us at batch 256 when it issued them itself.
template <bool MULTI, bool FP8, bool ROPE = false>
__global__ __launch_bounds__(256, 2) void decode_attn_kernel(DecodeAttnArgs a, int n_workers)
{
    static_assert(!(MULTI && ROPE), "the fused rotary embedding serves the one-token step");
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int w = blockIdx.x * 4 + wave;
    if (w >= n_workers) return;
    const int g = w % a.Hkv, cid = w / a.Hkv;
    int lo = 0;
    if (a.chunk_seq) {
        lo = a.chunk_seq[cid];
    } else {
        int hi = a.B;       // largest b with chunk_cu[b] <= cid (every sequence has >= 1 chunk)
        while (hi - lo > 1) {
            int mid = (lo + hi) >> 1;
            if (a.chunk_cu[mid] <= cid) lo = mid; else hi = mid;
        }
    }
    const int b = lo;
    const int ntok = MULTI ? a.u_ntok[b] : 1;
    const int n_keys = a.pos[b] + ntok;                // keys visible to the unit's last token
    const int n_chunks = a.chunk_cu[b + 1] - a.chunk_cu[b];
    const int csz = ((n_keys + n_chunks - 1) / n_chunks + 63) & ~63;   // equal chunks, 64-key granules
    const int key0 = (cid - a.chunk_cu[b]) * csz;                       // < n_keys since csz <= chunk_keys
    // ROPE: the chunks cover the cached keys only; the new token (position pos, not yet in the cache)
    // is added from registers by the worker of the last chunk
    const int key1 = min(ROPE ? n_keys - 1 : n_keys, key0 + csz);
    const bool own_new = ROPE && cid - a.chunk_cu[b] == n_chunks - 1;
    const int group = a.Hq / a.Hkv;
    const int qi = lane & 15, kg = lane >> 4;
    // MFMA column qi: head qh of the group (and, multi-token, token qt of the unit)
    const int qt = MULTI ? qi / group : 0, qh = MULTI ? qi - qt * group : qi;
    const bool col_ok = MULTI ? qt < ntok : qi < group;
    const int row = MULTI ? a.u_row0[b] + qt : b;      // row of qkv / o
    // keys this column may see: all n_keys (one token), or 0 .. pos + qt
    const int limit = MULTI ? min(n_keys, a.pos[b] + qt + 1) : n_keys;
    const int limit_min = MULTI ? a.pos[b] + 1 : n_keys;

    // query rows as B operand: lane (n = qi, kg) holds channels 32s + 8kg .. +7
    bf16x8 qf[4];
    {
        const uint16_t *qp = (const uint16_t *)a.qkv + (size_t)(col_ok ? row : 0) * a.ld +
                             (size_t)(g * group + (col_ok ? qh : 0)) * 128 + kg * 8;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            u32x4 z = {0u, 0u, 0u, 0u};
            if (col_ok) z = *(const u32x4 *)(qp + 32 * s);
            qf[s] = __builtin_bit_cast(bf16x8, z);
        }
    }
    if (ROPE) {
        // rotate-half pairs channel i with i + 64: fragment s (channels 32 s + 8 kg + e) with fragment s + 2
        const int pos = a.pos[b];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const u32x4 lo = __builtin_bit_cast(u32x4, qf[s]), hi = __builtin_bit_cast(u32x4, qf[s + 2]);
            u32x4 nlo, nhi;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float c[4], sn[4];
                rope_factors4(a, pos, 32 * s + 8 * kg + 4 * h, c, sn);
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const unsigned wl = lo[2 * h + e], wh = hi[2 * h + e];
                    const float x0a = bfbits2f(wl & 0xffffu), x0b = bfbits2f(wl >> 16);
                    const float x1a = bfbits2f(wh & 0xffffu), x1b = bfbits2f(wh >> 16);
                    nlo[2 * h + e] = pack2bf(x0a * c[2 * e] - x1a * sn[2 * e], x0b * c[2 * e + 1] - x1b * sn[2 * e + 1]);
                    nhi[2 * h + e] = pack2bf(x1a * c[2 * e] + x0a * sn[2 * e], x1b * c[2 * e + 1] + x0b * sn[2 * e + 1]);
                }
            }
            qf[s] = __builtin_bit_cast(bf16x8, nlo);
            qf[s + 2] = __builtin_bit_cast(bf16x8, nhi);
        }
    }
    const size_t plane = ((size_t)a.slots[b] * a.Hkv + g) * (size_t)a.max_len_pad * 128;
    const uint16_t *Kp = (const uint16_t *)a.k_cache + plane + qi * 32 + kg * 8;
    const uint16_t *Vp = (const uint16_t *)a.v_cache + plane + qi * 32 + kg * 8;
    const uint8_t *Kp8 = (const uint8_t *)a.k_cache + plane + lane * 16;
    const uint8_t *Vp8 = (const uint8_t *)a.v_cache + plane + lane * 16;
    f32x4 oacc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) oacc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;
    const float sl2e = a.scale * 1.4426950408889634f * (FP8 ? a.k_scale : 1.f);
    const float o_scale = FP8 ? a.v_scale : 1.f;

    // one 64-key step on operands handed in by get_k(key block, k-step) / get_v(key half, channel block)
    auto process = [&](int k, auto get_k, auto get_v) {
        // scores: lane (qi, kg), block kb, register j  <->  key k + 16*kb + 4*kg + j
        f32x4 sacc[4];
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
            sacc[kb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s)
                sacc[kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(get_k(kb, s), qf[s], sacc[kb], 0, 0, 0);
        }
        const int last = MULTI ? min(key1, limit) : key1;    // first key this column must not see
        const bool tail = k + 64 > (MULTI ? min(key1, limit_min) : key1);
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (tail && k + 16 * kb + 4 * kg + j >= last) sacc[kb][j] = -INFINITY;
                mx = fmaxf(mx, sacc[kb][j]);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        // one token: finite, key k < key1 is always unmasked.  Multi-token: a later chunk may hold
        // no key that an early token sees; its running max then stays -inf and every weight is 0
        float m_new = fmaxf(m_run, mx * sl2e);
        const float m_ref = (MULTI && m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = dexp2(m_run - m_ref);
        m_run = m_new;
        m_new = m_ref;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float p = dexp2(fmaf(sacc[kb][j], sl2e, -m_new));
                sacc[kb][j] = p;
                psum += p;
            }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) oacc[i][j] *= alpha;
        // exp'd scores as B operand of the value contraction: k-index 8kg+i  <->  key 16*(i/4)+4kg+i%4
        bf16x8 pf[2];
#pragma unroll
        for (int vb = 0; vb < 2; ++vb) {
            u32x4 pk = {pack2bf(sacc[2 * vb][0], sacc[2 * vb][1]), pack2bf(sacc[2 * vb][2], sacc[2 * vb][3]),
                        pack2bf(sacc[2 * vb + 1][0], sacc[2 * vb + 1][1]),
                        pack2bf(sacc[2 * vb + 1][2], sacc[2 * vb + 1][3])};
            pf[vb] = __builtin_bit_cast(bf16x8, pk);
        }
#pragma unroll
        for (int db = 0; db < 8; ++db)
#pragma unroll
            for (int vb = 0; vb < 2; ++vb)
                oacc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(get_v(vb, db), pf[vb], oacc[db], 0, 0, 0);
    };

    if (FP8) {
        // Two register sets: the loads of the next 64-key step are issued before the current one is
        // computed, so a wave always has a step's worth of bytes in flight.  The issue is unconditional
        // - past the end of the chunk the last step is requested again (a cache hit, never used) -
        // because after a conditional issue the compiler no longer knows which loads are the older
        // ones and waits for the prefetched step before it starts on the current one.
        const int k_last = key0 + ((key1 - key0 - 1) >> 6 << 6);     // first key of the last step (key1 > key0)
        // 16 loads of 16 bytes per lane per step: [0..7] keys (block kb, half t -> 2 kb + t), [8..15]
        // values (channel block db); the codes are widened operand by operand right before their MFMA
        u32x4 ra[16], rb[16];
        auto issue = [&](int k, u32x4 (&r)[16]) {
            const uint8_t *kb_ptr = Kp8 + (size_t)(k >> 4) * 2048;
            const uint8_t *vb_ptr = Vp8 + (size_t)(k >> 6) * 8192;
#pragma unroll
            for (int i = 0; i < 8; ++i) r[i] = *(const u32x4 *)(kb_ptr + i * 1024);
#pragma unroll
            for (int db = 0; db < 8; ++db) r[8 + db] = *(const u32x4 *)(vb_ptr + db * 1024);
        };
        auto run = [&](int k, u32x4 (&r)[16]) {
            process(
                k,
                [&](int kb, int s) { return fp8x8_to_bf16(r[2 * kb + (s >> 1)][2 * (s & 1)], r[2 * kb + (s >> 1)][2 * (s & 1) + 1]); },
                [&](int vb, int db) { return fp8x8_to_bf16(r[8 + db][2 * vb], r[8 + db][2 * vb + 1]); });
        };
        if (key0 < key1) {
            issue(key0, ra);
            for (int k = key0;; k += 128) {
                issue(min(k + 64, k_last), rb);
                __builtin_amdgcn_sched_barrier(0);
                run(k, ra);
                if (k + 64 >= key1) break;
                issue(min(k + 128, k_last), ra);
                __builtin_amdgcn_sched_barrier(0);
                run(k + 64, rb);
                if (k + 128 >= key1) break;
            }
        }
    } else {
        // 32 loads of 16 bytes per lane per step.  All of them (32 KB per wave) are issued before
        // anything consumes them: bytes in flight, not instruction count, is what this kernel lives
        // on.  (A second register set for the next step does not fit beside the accumulators at two
        // workgroups per CU, and with 2048 resident waves the memory system is saturated anyway.)
        for (int k = key0; k < key1; k += 64) {
            bf16x8 kf[4][4], vf[2][8];
            const uint16_t *kb_ptr = Kp + (size_t)(k >> 4) * 2048;
            const uint16_t *vb_ptr = Vp + (size_t)(k >> 5) * 4096;
#pragma unroll
            for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                for (int s = 0; s < 4; ++s) kf[kb][s] = *(const bf16x8 *)(kb_ptr + kb * 2048 + s * 512);
#pragma unroll
            for (int vb = 0; vb < 2; ++vb)
#pragma unroll
                for (int db = 0; db < 8; ++db) vf[vb][db] = *(const bf16x8 *)(vb_ptr + vb * 4096 + db * 512);
            __builtin_amdgcn_sched_barrier(0);
            process(k, [&](int kb, int s) { return kf[kb][s]; }, [&](int vb, int db) { return vf[vb][db]; });
        }
    }

    if (own_new) {
        // The new token as one more key, from registers: its rotated key exactly as the cache now holds it
        // (rounded to bf16, or the value of its E4M3 code), the score on the lane's 32 channels summed over
        // the four lanes of a column, then one step of the online softmax with p in fp32.
        const int pos = a.pos[b];
        const uint16_t *kr = (const uint16_t *)a.qkv + (size_t)b * a.ld + (size_t)(a.Hq + g) * 128 + kg * 8;
        const uint16_t *vr = (const uint16_t *)a.qkv + (size_t)b * a.ld + (size_t)(a.Hq + a.Hkv + g) * 128;
        float dot = 0.f;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const u32x4 klo = *(const u32x4 *)(kr + 32 * s), khi = *(const u32x4 *)(kr + 32 * s + 64);
            const u32x4 qlo = __builtin_bit_cast(u32x4, qf[s]), qhi = __builtin_bit_cast(u32x4, qf[s + 2]);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float c[4], sn[4];
                rope_factors4(a, pos, 32 * s + 8 * kg + 4 * h, c, sn);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int wi = 2 * h + (e >> 1), sh = 16 * (e & 1);
                    const float x0 = bfbits2f((klo[wi] >> sh) & 0xffffu), x1 = bfbits2f((khi[wi] >> sh) & 0xffffu);
                    float y0 = x0 * c[e] - x1 * sn[e], y1 = x1 * c[e] + x0 * sn[e];
                    if (FP8) {
                        y0 = e4m3_decode(e4m3_encode((double)y0 / a.k_scale_d));
                        y1 = e4m3_decode(e4m3_encode((double)y1 / a.k_scale_d));
                    } else {
                        y0 = bf2f(f2bf(y0));
                        y1 = bf2f(f2bf(y1));
                    }
                    dot += bfbits2f((qlo[wi] >> sh) & 0xffffu) * y0 + bfbits2f((qhi[wi] >> sh) & 0xffffu) * y1;
                }
            }
        }
        dot += __shfl_xor(dot, 16, 64);
        dot += __shfl_xor(dot, 32, 64);
        const float x = dot * sl2e;
        const float m_new = fmaxf(m_run, x);
        const float alpha = dexp2(m_run - m_new), pnew = dexp2(x - m_new);
        m_run = m_new;
        l_run = l_run * alpha + (kg == 0 ? pnew : 0.f);
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            const uint2 vv = *(const uint2 *)(vr + 16 * db + 4 * kg);     // channels 16 db + 4 kg + j
            float v[4] = {bfbits2f(vv.x & 0xffffu), bfbits2f(vv.x >> 16), bfbits2f(vv.y & 0xffffu), bfbits2f(vv.y >> 16)};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (FP8) v[j] = e4m3_decode(e4m3_encode((double)v[j] / a.v_scale_d));
                oacc[db][j] = oacc[db][j] * alpha + pnew * v[j];
            }
        }
    }
    float l_tot = l_run + __shfl_xor(l_run, 16, 64);
    l_tot += __shfl_xor(l_tot, 32, 64);
    if (col_ok && n_chunks == 1) {
        // the only chunk of its sequence: normalise and store the output row directly
        const int head = g * group + qh;
        const float inv = o_scale / l_tot;
        uint16_t *op = (uint16_t *)a.o + ((size_t)row * a.Hq + head) * 128 + 4 * kg;
#pragma unroll
        for (int db = 0; db < 8; ++db) {
            uint2 w2;
            w2.x = pack2bf(oacc[db][0] * inv, oacc[db][1] * inv);
            w2.y = pack2bf(oacc[db][2] * inv, oacc[db][3] * inv);
            *(uint2 *)(op + 16 * db) = w2;            // channels 16*db + 4*kg + j
        }
    } else if (col_ok) {
        // partial row index: (chunk, head), or multi-token (chunk, kv head, column)
        const size_t pidx = MULTI ? ((size_t)cid * a.Hkv + g) * 16 + qi : (size_t)cid * a.Hq + g * group + qi;
        float *po = a.part_o + pidx * 128;
#pragma unroll
        for (int db = 0; db < 8; ++db)
            *(f32x4 *)(po + 16 * db + 4 * kg) = oacc[db];   // rows 16*db + 4*kg + j of O^T
        if (kg == 0) {
            float *pm = a.part_ml + pidx * 2;
            pm[0] = m_run;
            pm[1] = l_tot;
        }
    }
}

// o[b, head, :] = sum_c 2^(m_c - M) o_c / sum_c 2^(m_c - M) l_c over the chunks of sequence b
// (sequences with a single chunk are finished by the attention kernel and skipped here).
// The chunk weights are formed once per block (one chunk per thread, in parallel); the weighted
// sum then reads the partial rows with independent loads.
template <bool MULTI>
__global__ __launch_bounds__(128) void decode_attn_merge_kernel(DecodeAttnArgs a)
{
    __shared__ float wgt_s[128];
    __shared__ float red[2];
    // one token: blockIdx.y = head.  Multi-token: blockIdx.y = 16 * kv head + column (token, head of group)
    const int b = blockIdx.x, d = threadIdx.x;
    const int c0 = a.chunk_cu[b], c1 = a.chunk_cu[b + 1];
    if (c1 - c0 == 1) return;                          // written by the attention kernel itself
    const int group = a.Hq / a.Hkv;
    int head = blockIdx.y, row = b, pstride = a.Hq, pcol = blockIdx.y;
    if (MULTI) {
        const int g = blockIdx.y >> 4, col = blockIdx.y & 15;
        const int qt = col / group;
        if (qt >= a.u_ntok[b]) return;
        head = g * group + (col - qt * group);
        row = a.u_row0[b] + qt;
        pstride = a.Hkv * 16;
    }
    float M = -INFINITY;
    for (int c = c0 + d; c < c1; c += 128) M = fmaxf(M, a.part_ml[((size_t)c * pstride + pcol) * 2]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
    if ((d & 63) == 0) red[d >> 6] = M;
    __syncthreads();
    M = fmaxf(red[0], red[1]);
    float L = 0.f, acc = 0.f;
    for (int base = c0; base < c1; base += 128) {
        const int c = base + d;
        float w = 0.f, l = 0.f;
        if (c < c1) {
            const float *pm = a.part_ml + ((size_t)c * pstride + pcol) * 2;
            w = dexp2(pm[0] - M);
            l = pm[1];
        }
        __syncthreads();
        wgt_s[d] = w;
        L += w * l;
        __syncthreads();
        const int cnt = min(128, c1 - base);
        const float *po = a.part_o + ((size_t)base * pstride + pcol) * 128 + d;
        const size_t stride = (size_t)pstride * 128;
        int j = 0;
        for (; j + 4 <= cnt; j += 4) {
            float v0 = po[(size_t)j * stride], v1 = po[(size_t)(j + 1) * stride];
            float v2 = po[(size_t)(j + 2) * stride], v3 = po[(size_t)(j + 3) * stride];
            acc += wgt_s[j] * v0 + wgt_s[j + 1] * v1 + wgt_s[j + 2] * v2 + wgt_s[j + 3] * v3;
        }
        for (; j < cnt; ++j) acc += wgt_s[j] * po[(size_t)j * stride];
    }
    // total weight: sum of the per-thread partial sums
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) L += __shfl_xor(L, off, 64);
    __syncthreads();
    if ((d & 63) == 0) red[d >> 6] = L;
    __syncthreads();
    L = red[0] + red[1];
    ((uint16_t *)a.o)[((size_t)row * a.Hq + head) * 128 + d] = f2bf(acc / L * (a.fp8 ? a.v_scale : 1.f)).x;
}

template <bool FP8>
static hipError_t launch_decode_attn_t(const DecodeAttnArgs &a, int n_workers, hipStream_t s)
{
    if (a.u_ntok) {
        decode_attn_kernel<true, FP8><<<(n_workers + 3) / 4, 256, 0, s>>>(a, n_workers);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        decode_attn_merge_kernel<true><<<dim3(a.B, a.Hkv * 16), 128, 0, s>>>(a);
        return hipGetLastError();
    }
    if (a.rope_table) decode_attn_kernel<false, FP8, true><<<(n_workers + 3) / 4, 256, 0, s>>>(a, n_workers);
    else decode_attn_kernel<false, FP8><<<(n_workers + 3) / 4, 256, 0, s>>>(a, n_workers);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // every sequence has at least one chunk: with as many chunks as sequences each worker has normalised
    // and stored its sequence itself and nothing is left to merge
    if (a.total_chunks == a.B) return hipSuccess;
    decode_attn_merge_kernel<false><<<dim3(a.B, a.Hq), 128, 0, s>>>(a);
    return hipGetLastError();
}

hipError_t launch_decode_attn_mfma(const DecodeAttnArgs &a, hipStream_t s)
{
    const int n_workers = a.total_chunks * a.Hkv;
    if (n_workers <= 0) return hipSuccess;
    return a.fp8 ? launch_decode_attn_t<true>(a, n_workers, s) : launch_decode_attn_t<false>(a, n_workers, s);
}

}  // namespace pd
