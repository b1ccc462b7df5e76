// Skinny bf16 GEMM for decode batches of up to 16 rows:  C[M<=16, N] = epilogue(A[M,K] * B[N,K]^T).
//
// The step is bound by streaming the weight matrix B from HBM exactly once, so the weights are
// the MFMA A operand and go straight from global memory into operand registers: in the packed
// weight layout one 16-row x 32-k block is the register image of the operand, so every load
// instruction reads 1 KB of contiguous memory (several blocks in flight per wave); the (tiny, L2-resident)
// activations are the B operand with the batch as the N dimension of v_mfma_f32_16x16x32_bf16,
// padded with zero columns.  A workgroup owns 16 weight rows (one output column block); its
// waves split K and combine through LDS in a fixed order, so results are deterministic.
// Epilogues as in the tiled GEMM; for SwiGLU the workgroup takes the gate block and the matching
// up block of the interleaved weight pack.
//
// Grouped form (mixture-of-experts decode): blockIdx.y is the group; its rows
// group_offsets[g] .. group_offsets[g+1]-1 (gathered through a_gather) multiply the group's own
// weight matrix, 16 rows per pass over the weights (a group of more than 16 rows streams them
// again, so the launcher takes this kernel only while groups average 8 rows or fewer); a group
// without rows exits at once, so only the experts that were chosen are streamed.
//
// W8 form: the weights are E4M3 codes with one power-of-two scale per weight row (half the bytes).
// One 16-byte-per-lane load then carries the operands of two k-steps; the codes are widened to bf16
// in registers (exact) and the row scale multiplies the accumulated sum in the epilogue.
#include "pd_internal.h"

namespace pd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// GV_WAVES waves split K; each keeps GV_UNROLL blocks per row block in flight.  Measured on the 8B
// shapes: the SwiGLU pair streams fastest with 2 waves x 16 blocks, a long K (the down projection)
// with 8 waves x 4, the short square ones with 4 x 8.
__device__ __forceinline__ bf16x8 w8_to_bf16(unsigned w0, unsigned w1)
{
    auto f0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w0, false);
    auto f1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w0, true);
    auto f2 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w1, false);
    auto f3 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w1, true);
    u32x4 r = {pack2bf(f0[0], f0[1]), pack2bf(f1[0], f1[1]), pack2bf(f2[0], f2[1]), pack2bf(f3[0], f3[1])};
    return __builtin_bit_cast(bf16x8, r);
}

template <int EPI, int GV_WAVES, int GV_UNROLL, bool W8 = false>
__global__ __launch_bounds__(64 * GV_WAVES) void gemv_mfma_kernel(GemmArgs a)
{
    constexpr int RB = EPI == EPI_SWIGLU ? 2 : 1;
    __shared__ f32x4 red[GV_WAVES][RB][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, kg = lane >> 4;
    const int blk = blockIdx.x;
    // first weight row of each row block
    int row0[RB];
    if (EPI == EPI_SWIGLU) {
        row0[0] = (blk >> 1) * 64 + (blk & 1) * 16;   // gate rows of output columns 16*blk .. +15
        row0[RB - 1] = row0[0] + 32;                  // matching up rows
    } else {
        row0[0] = blk * 16;
    }
    // k-steps of 32 (W8: pairs of them, one load each), split evenly over the waves
    const int ksteps = W8 ? a.K / 64 : a.K / 32;
    const int per = (ksteps + GV_WAVES - 1) / GV_WAVES;
    const int s_begin = wave * per, s_end = min(ksteps, s_begin + per);

    // rows of this workgroup: all M, or the rows of group blockIdx.y
    int lo = 0, n_rows = a.M;
    const uint16_t *W = (const uint16_t *)a.B;
    const uint8_t *W8p = (const uint8_t *)a.B8;
    const float *row_scale = a.b_scale;
    if (a.group_offsets) {
        lo = a.group_offsets[blockIdx.y];
        n_rows = a.group_offsets[blockIdx.y + 1] - lo;
        if (n_rows <= 0) return;                      // uniform over the workgroup
        W += (size_t)blockIdx.y * a.b_group_stride;
        if (W8) {
            W8p += (size_t)blockIdx.y * a.b_group_stride;
            row_scale += (size_t)blockIdx.y * (EPI == EPI_SWIGLU ? 2 * a.N : a.N);
        }
    }
    const uint16_t *wp[RB];   // block (row0/16, 0) of the packed layout, this lane's 16 bytes
    const uint8_t *wp8[RB];
#pragma unroll
    for (int i = 0; i < RB; ++i) {
        wp[i] = W + (size_t)(row0[i] >> 4) * (a.K >> 5) * 512 + lane * 8;
        wp8[i] = W8p + (size_t)(row0[i] >> 4) * (a.K >> 6) * 1024 + lane * 16;
    }
    for (int rb0 = 0; rb0 < n_rows; rb0 += 16) {      // one pass per 16 rows (uniform over the workgroup)
    const bool xrow = rb0 + r < n_rows;
    int arow = xrow ? lo + rb0 + r : lo;
    if (a.a_gather) arow = a.a_gather[arow];
    const uint16_t *xp = (const uint16_t *)a.A + (size_t)arow * a.lda + kg * 8;

    f32x4 acc[RB];
#pragma unroll
    for (int i = 0; i < RB; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    int s = s_begin;
    if (W8) {
        constexpr int U = GV_UNROLL / 2 > 0 ? GV_UNROLL / 2 : 1;     // pairs of k-steps per batch
        for (; s + U <= s_end; s += U) {
            u32x4 wr[RB][U];
            bf16x8 xf[U][2];
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int i = 0; i < RB; ++i) wr[i][u] = *(const u32x4 *)(wp8[i] + (size_t)(s + u) * 1024);
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    u32x4 z = {0u, 0u, 0u, 0u};
                    if (xrow) z = *(const u32x4 *)(xp + (size_t)(2 * (s + u) + h) * 32);
                    xf[u][h] = __builtin_bit_cast(bf16x8, z);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w8_to_bf16(wr[i][u][0], wr[i][u][1]), xf[u][0],
                                                                     acc[i], 0, 0, 0);
                    acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w8_to_bf16(wr[i][u][2], wr[i][u][3]), xf[u][1],
                                                                     acc[i], 0, 0, 0);
                }
        }
        for (; s < s_end; ++s) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                u32x4 z = {0u, 0u, 0u, 0u};
                if (xrow) z = *(const u32x4 *)(xp + (size_t)(2 * s + h) * 32);
                bf16x8 xf = __builtin_bit_cast(bf16x8, z);
#pragma unroll
                for (int i = 0; i < RB; ++i) {
                    const uint2 wr = *(const uint2 *)(wp8[i] + (size_t)s * 1024 + h * 8);
                    acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w8_to_bf16(wr.x, wr.y), xf, acc[i], 0, 0, 0);
                }
            }
        }
    } else {
    for (; s + GV_UNROLL <= s_end; s += GV_UNROLL) {
        bf16x8 wf[RB][GV_UNROLL], xf[GV_UNROLL];
#pragma unroll
        for (int u = 0; u < GV_UNROLL; ++u) {
#pragma unroll
            for (int i = 0; i < RB; ++i) wf[i][u] = *(const bf16x8 *)(wp[i] + (size_t)(s + u) * 512);
            u32x4 z = {0u, 0u, 0u, 0u};
            if (xrow) z = *(const u32x4 *)(xp + (size_t)(s + u) * 32);
            xf[u] = __builtin_bit_cast(bf16x8, z);
        }
        __builtin_amdgcn_sched_barrier(0);   // every load of the batch is in flight before the first MFMA
#pragma unroll
        for (int u = 0; u < GV_UNROLL; ++u)
#pragma unroll
            for (int i = 0; i < RB; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[i][u], xf[u], acc[i], 0, 0, 0);
    }
    for (; s < s_end; ++s) {
        u32x4 z = {0u, 0u, 0u, 0u};
        if (xrow) z = *(const u32x4 *)(xp + (size_t)s * 32);
        bf16x8 xf = __builtin_bit_cast(bf16x8, z);
#pragma unroll
        for (int i = 0; i < RB; ++i) {
            bf16x8 wf = *(const bf16x8 *)(wp[i] + (size_t)s * 512);
            acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xf, acc[i], 0, 0, 0);
        }
    }
    }
#pragma unroll
    for (int i = 0; i < RB; ++i) red[wave][i][lane] = acc[i];
    __syncthreads();
    if (wave == 0 && xrow) {
        f32x4 tot[RB];
#pragma unroll
        for (int i = 0; i < RB; ++i) {
            tot[i] = red[0][i][lane];
#pragma unroll
            for (int w = 1; w < GV_WAVES; ++w) tot[i] += red[w][i][lane];
            if (W8) {   // register j belongs to weight row row0 + 4*kg + j
                const f32x4 sc = *(const f32x4 *)(row_scale + row0[i] + 4 * kg);
                tot[i] *= sc;
            }
        }
        // lane (batch row rb0 + r, kg): register j is weight row 4*kg + j of the block
        const int m = lo + rb0 + r;
        uint16_t *C = (uint16_t *)a.C + (size_t)m * a.ldc;
        const int col = blk * 16 + 4 * kg;            // first of 4 consecutive output columns
        float v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (EPI == EPI_SWIGLU) {
                float gte = tot[0][j];
                v[j] = gte / (1.0f + __expf(-gte)) * tot[RB - 1][j];
            } else {
                v[j] = tot[0][j];
            }
        }
        if (EPI == EPI_RESIDUAL) {
            uint2 rr = *(const uint2 *)((const uint16_t *)a.R + (size_t)m * a.ldr + col);
            v[0] += bfbits2f(rr.x & 0xffffu);
            v[1] += bfbits2f(rr.x >> 16);
            v[2] += bfbits2f(rr.y & 0xffffu);
            v[3] += bfbits2f(rr.y >> 16);
        }
        uint2 o;
        o.x = pack2bf(v[0], v[1]);
        o.y = pack2bf(v[2], v[3]);
        *(uint2 *)(C + col) = o;
    }
    __syncthreads();                                  // red is reused by the next pass
    }
}

bool gemv_mfma_supported(const GemmArgs &a)
{
    if (a.M < 1) return false;
    if (a.group_offsets) {
        if (a.n_groups < 1 || a.n_groups > 65535 || a.M > 8 * a.n_groups) return false;
    } else if (a.M > 16 || a.a_gather) {
        return false;
    }
    if (a.K % 32 != 0 || a.N % 16 != 0 || a.lda % 8 != 0 || a.ldb % 8 != 0) return false;
    if (a.ldc % 4 != 0 || (a.epilogue == EPI_RESIDUAL && a.ldr % 4 != 0)) return false;
    if (!a.packed || a.ldb != a.K) return false;
    if (a.epilogue == EPI_SWIGLU && a.N % 32 != 0) return false;
    if (a.B8 && (a.K % 64 != 0 || !a.b_scale)) return false;
    return true;
}

template <bool W8>
static void launch_gemv_t(const GemmArgs &a, hipStream_t s)
{
    const dim3 grid(a.N / 16, a.group_offsets ? a.n_groups : 1);
    const bool long_k = a.K >= 8192;
    switch (a.epilogue) {
    case EPI_NONE:
        if (long_k) gemv_mfma_kernel<EPI_NONE, 8, 4, W8><<<grid, 512, 0, s>>>(a);
        else gemv_mfma_kernel<EPI_NONE, 4, 8, W8><<<grid, 256, 0, s>>>(a);
        break;
    case EPI_RESIDUAL:
        if (long_k) gemv_mfma_kernel<EPI_RESIDUAL, 8, 4, W8><<<grid, 512, 0, s>>>(a);
        else gemv_mfma_kernel<EPI_RESIDUAL, 4, 8, W8><<<grid, 256, 0, s>>>(a);
        break;
    default: gemv_mfma_kernel<EPI_SWIGLU, 2, 16, W8><<<grid, 128, 0, s>>>(a); break;
    }
}

hipError_t launch_gemv_mfma(const GemmArgs &a, hipStream_t s)
{
    if (a.B8) launch_gemv_t<true>(a, s);
    else launch_gemv_t<false>(a, s);
    return hipGetLastError();
}

}  // namespace pd
