// Mixture-of-experts routing: router logits, softmax + top-k selection, a stable counting sort of
// the (token, expert) pairs by expert, and the weighted combine of the expert outputs.
#include "pd_internal.h"

namespace pd {

// logits[t][e] = sum_i y[t][i] * Wr[e][i], fp32 output.  One wavefront per token.
template <typename T>
__global__ __launch_bounds__(256) void router_logits_kernel(const T *__restrict__ y,
                                                            const T *__restrict__ wr,
                                                            float *__restrict__ logits, int Tn, int d,
                                                            int E)
{
    int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    int lane = threadIdx.x & 63;
    if (t >= Tn) return;
    const T *yr = y + (size_t)t * d;
    for (int e = 0; e < E; ++e) {
        const T *w = wr + (size_t)e * d;
        float acc = 0.f;
        for (int i = lane; i < d; i += 64) acc = fmaf(Elem<T>::ld(yr + i), Elem<T>::ld(w + i), acc);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
        if (lane == 0) logits[(size_t)t * E + e] = acc;
    }
}

hipError_t launch_router_logits(int dtype, const void *y, const void *w_router, float *logits,
                                int T, int d, int E, hipStream_t s)
{
    if (T <= 0) return hipSuccess;
    if (dtype == PD_F32)
        router_logits_kernel<float><<<(T + 3) / 4, 256, 0, s>>>((const float *)y, (const float *)w_router, logits, T, d, E);
    else
        router_logits_kernel<bf16_t><<<(T + 3) / 4, 256, 0, s>>>((const bf16_t *)y, (const bf16_t *)w_router, logits, T, d, E);
    return hipGetLastError();
}

// p = softmax(logits) over all experts; the top_k largest p (ties: lower index); weights
// renormalised to sum 1.  The probabilities are exp(r - max) / denom in double with one denom per
// token, a non-decreasing function of the logit, so a clearly larger logit is a larger probability
// and the selection compares logits; logits closer than 1e-6 (where rounding could make two
// probabilities equal, which the lower index then wins) are decided on the probabilities
// themselves.  Only those and the chosen experts' weights need exponentials.
__device__ __forceinline__ void moe_topk_token(const MoeRouteArgs &a, int t, int *chosen = nullptr)
{
    const float *r = a.logits + (size_t)t * a.E;
    double mx = -INFINITY;
    for (int e = 0; e < a.E; ++e) mx = fmax(mx, (double)r[e]);
    double denom = 0.0;
    for (int e = 0; e < a.E; ++e) denom += exp((double)r[e] - mx);
    unsigned long long taken = 0ull;
    double sum = 0.0;
    double pk[8];
    int ik[8];
    for (int k = 0; k < a.top_k; ++k) {
        int best = -1;
        float rbest = 0.f;
        for (int e = 0; e < a.E; ++e) {
            if ((taken >> e) & 1ull) continue;
            bool better = best < 0 || r[e] > rbest;      // strict: the lower index wins a tie
            if (better && best >= 0 && (double)r[e] - (double)rbest < 1e-6)
                better = exp((double)r[e] - mx) / denom > exp((double)rbest - mx) / denom;   // nearly equal: decide on the probabilities themselves
            if (better) {
                best = e;
                rbest = r[e];
            }
        }
        taken |= 1ull << best;
        pk[k] = exp((double)rbest - mx) / denom;
        ik[k] = best;
        sum += pk[k];
    }
    for (int k = 0; k < a.top_k; ++k) {
        a.expert_idx[(size_t)t * a.top_k + k] = ik[k];
        a.expert_w[(size_t)t * a.top_k + k] = (float)(pk[k] / sum);
        if (chosen) chosen[t * a.top_k + k] = ik[k];
    }
}

__global__ void moe_topk_kernel(MoeRouteArgs a)
{
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < a.T) moe_topk_token(a, t);
}

// Decode-sized routing, at most 64 (token, expert) pairs: one wavefront selects the experts and
// sorts the pairs in a single launch.  Lane i owns pair i; for every expert a ballot gives the
// lanes that chose it, so a pair's place is the expert's base plus the number of lower lanes with
// the same expert: the same stable order as the general kernel.
__global__ __launch_bounds__(64) void moe_route_small_kernel(MoeRouteArgs a)
{
    __shared__ int chosen[64];
    const int lane = threadIdx.x;
    const int P = a.T * a.top_k;
    if (lane < a.T) moe_topk_token(a, lane, chosen);
    __syncthreads();
    const int e = lane < P ? chosen[lane] : -1;
    int base = 0;
    if (lane == 0) a.offsets[0] = 0;
    for (int ex = 0; ex < a.E; ++ex) {
        const unsigned long long mask = __ballot(e == ex);
        if (e == ex) {
            const int pos = base + __popcll(mask & ((1ull << lane) - 1ull));
            a.sorted_token[pos] = lane / a.top_k;
            a.pair_pos[lane] = pos;
        }
        base += __popcll(mask);
        if (lane == 0) a.offsets[ex + 1] = base;
    }
}

// Stable counting sort of the T*top_k pairs by expert, one 1024-thread block.  Pair index is
// t*top_k + k; within an expert the pairs keep that order.
__global__ __launch_bounds__(1024) void moe_sort_kernel(MoeRouteArgs a)
{
    __shared__ int wave_tot[16];
    __shared__ int base_s;
    const int P = a.T * a.top_k;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = (P + 1023) / 1024;
    const int lo = tid * per, hi = min(P, lo + per);
    if (tid == 0) {
        base_s = 0;
        a.offsets[0] = 0;
    }
    __syncthreads();
    for (int e = 0; e < a.E; ++e) {
        int cnt = 0;
        for (int i = lo; i < hi; ++i) cnt += (a.expert_idx[i] == e);
        // inclusive scan inside the wave
        int inc = cnt;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            int v = __shfl_up(inc, off, 64);
            if (lane >= off) inc += v;
        }
        if (lane == 63) wave_tot[wave] = inc;
        __syncthreads();
        int wbase = 0, total = 0;
        for (int w = 0; w < 16; ++w) {
            if (w < wave) wbase += wave_tot[w];
            total += wave_tot[w];
        }
        int pos = base_s + wbase + inc - cnt;
        for (int i = lo; i < hi; ++i)
            if (a.expert_idx[i] == e) {
                a.sorted_token[pos] = i / a.top_k;
                a.pair_pos[i] = pos;
                ++pos;
            }
        __syncthreads();
        if (tid == 0) {
            base_s += total;
            a.offsets[e + 1] = base_s;
        }
        __syncthreads();
    }
}

// The same order from many blocks of 256 pairs.  First kernel: how many pairs of each expert a block
// holds.  Second kernel: a pair's place is the expert's first place, plus the pairs of that expert
// in earlier blocks, in earlier waves of its block and in lower lanes of its wave (ballots).
__global__ __launch_bounds__(256) void moe_block_hist_kernel(MoeRouteArgs a)
{
    __shared__ int wcnt[64][4];
    const int P = a.T * a.top_k, i = blockIdx.x * 256 + threadIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int e = i < P ? a.expert_idx[i] : -1;
    for (int ex = 0; ex < a.E; ++ex) {
        const unsigned long long mask = __ballot(e == ex);
        if (lane == 0) wcnt[ex][wave] = __popcll(mask);
    }
    __syncthreads();
    if (threadIdx.x < a.E)
        a.block_hist[(size_t)blockIdx.x * a.E + threadIdx.x] =
            wcnt[threadIdx.x][0] + wcnt[threadIdx.x][1] + wcnt[threadIdx.x][2] + wcnt[threadIdx.x][3];
}

__global__ __launch_bounds__(256) void moe_block_scatter_kernel(MoeRouteArgs a, int n_blocks)
{
    __shared__ int wcnt[64][4];
    __shared__ int before[64], total[64], first[65];
    const int P = a.T * a.top_k, i = blockIdx.x * 256 + threadIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int e = i < P ? a.expert_idx[i] : -1;
    int rank = 0;
    for (int ex = 0; ex < a.E; ++ex) {
        const unsigned long long mask = __ballot(e == ex);
        if (e == ex) rank = __popcll(mask & ((1ull << lane) - 1ull));
        if (lane == 0) wcnt[ex][wave] = __popcll(mask);
    }
    if (threadIdx.x < a.E) {
        int b = 0, t = 0;
        for (int j = 0; j < n_blocks; ++j) {
            const int c = a.block_hist[(size_t)j * a.E + threadIdx.x];
            if (j < (int)blockIdx.x) b += c;
            t += c;
        }
        before[threadIdx.x] = b;
        total[threadIdx.x] = t;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int acc = 0;
        for (int ex = 0; ex < a.E; ++ex) {
            first[ex] = acc;
            acc += total[ex];
        }
        first[a.E] = acc;
    }
    __syncthreads();
    if (blockIdx.x == 0 && threadIdx.x <= a.E) a.offsets[threadIdx.x] = first[threadIdx.x];
    if (e >= 0) {
        int pos = first[e] + before[e] + rank;
        for (int w = 0; w < wave; ++w) pos += wcnt[e][w];
        a.sorted_token[pos] = i / a.top_k;
        a.pair_pos[i] = pos;
    }
}

hipError_t launch_moe_route(const MoeRouteArgs &a, hipStream_t s)
{
    if (a.T <= 0) return hipSuccess;
    if (a.T * a.top_k <= 64) {
        moe_route_small_kernel<<<1, 64, 0, s>>>(a);
        return hipGetLastError();
    }
    moe_topk_kernel<<<(a.T + 255) / 256, 256, 0, s>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (a.block_hist) {
        const int nb = (a.T * a.top_k + 255) / 256;
        moe_block_hist_kernel<<<nb, 256, 0, s>>>(a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        moe_block_scatter_kernel<<<nb, 256, 0, s>>>(a, nb);
        return hipGetLastError();
    }
    moe_sort_kernel<<<1, 1024, 0, s>>>(a);
    return hipGetLastError();
}

// out[t] = h[t] + sum_k w[t,k] * expert_out[pair_pos[t,k]]
template <typename T>
__global__ __launch_bounds__(256) void moe_combine_kernel(const T *__restrict__ h,
                                                          const T *__restrict__ eo,
                                                          const int32_t *__restrict__ pair_pos,
                                                          const float *__restrict__ w,
                                                          T *__restrict__ out, int d, int top_k)
{
    // blockIdx.x = token, the gridDim.y blocks of a token share its channels round-robin; the
    // (at most 8) pair positions and weights are read once, not once per channel
    const int t = blockIdx.x;
    int pp[8];
    float ww[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        pp[k] = k < top_k ? pair_pos[(size_t)t * top_k + k] : 0;
        ww[k] = k < top_k ? w[(size_t)t * top_k + k] : 0.f;
    }
    for (int i = blockIdx.y * 256 + threadIdx.x; i < d; i += gridDim.y * 256) {
        float acc = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (k < top_k) acc = fmaf(ww[k], Elem<T>::ld(eo + (size_t)pp[k] * d + i), acc);
        Elem<T>::st(out + (size_t)t * d + i, Elem<T>::ld(h + (size_t)t * d + i) + acc);
    }
}

// bf16 rows with d % 8 == 0: 8 channels (16 bytes) per thread step
__global__ __launch_bounds__(256) void moe_combine_bf16_vec_kernel(const uint4 *__restrict__ h, const uint4 *__restrict__ eo,
                                                                   const int32_t *__restrict__ pair_pos,
                                                                   const float *__restrict__ w, uint4 *__restrict__ out,
                                                                   int d8, int top_k)
{
    const int t = blockIdx.x;
    int pp[8];
    float ww[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        pp[k] = k < top_k ? pair_pos[(size_t)t * top_k + k] : 0;
        ww[k] = k < top_k ? w[(size_t)t * top_k + k] : 0.f;
    }
    for (int i = blockIdx.y * 256 + threadIdx.x; i < d8; i += gridDim.y * 256) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (k < top_k) {
                const uint4 v = eo[(size_t)pp[k] * d8 + i];
                const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[2 * j] = fmaf(ww[k], bfbits2f(u[j] & 0xffffu), acc[2 * j]);
                    acc[2 * j + 1] = fmaf(ww[k], bfbits2f(u[j] >> 16), acc[2 * j + 1]);
                }
            }
        const uint4 hv = h[(size_t)t * d8 + i];
        const uint32_t u[4] = {hv.x, hv.y, hv.z, hv.w};
        uint32_t o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            o[j] = pack2bf(bfbits2f(u[j] & 0xffffu) + acc[2 * j], bfbits2f(u[j] >> 16) + acc[2 * j + 1]);
        out[(size_t)t * d8 + i] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

hipError_t launch_moe_combine(int dtype, const void *h, const void *expert_out,
                              const int32_t *pair_pos, const float *expert_w, void *out, int T,
                              int d, int top_k, hipStream_t s)
{
    if (T <= 0) return hipSuccess;
    // few tokens: spread a row over several blocks so that no thread chains many memory round trips
    const int slices = T >= 512 ? 1 : (d + 511) / 512;
    const dim3 grid((unsigned)T, (unsigned)(slices < 1 ? 1 : slices));
    if (dtype == PD_F32)
        moe_combine_kernel<float><<<grid, 256, 0, s>>>((const float *)h, (const float *)expert_out, pair_pos, expert_w, (float *)out, d, top_k);
    else if (d % 8 == 0 && T >= 512)
        moe_combine_bf16_vec_kernel<<<dim3((unsigned)T, 1), 256, 0, s>>>((const uint4 *)h, (const uint4 *)expert_out, pair_pos, expert_w, (uint4 *)out, d / 8, top_k);
    else
        moe_combine_kernel<bf16_t><<<grid, 256, 0, s>>>((const bf16_t *)h, (const bf16_t *)expert_out, pair_pos, expert_w, (bf16_t *)out, d, top_k);
    return hipGetLastError();
}

}  // namespace pd
