// GEMM for a decode batch of 17 .. 128 rows over 8-bit weights (and of 17 .. 32 rows over bf16 weights):
//   C[M, N] = epilogue(A[M, K] * (scale[n] * value(code[n, k]))^T), bf16 activations, fp32 accumulation.
//
// At these sizes the bf16 GEMM is bound by the weight stream (the gate / up projection at 64 rows
// reads its weights at 5.6 TB/s), so E4M3 codes with one power-of-two scale per weight row halve
// the time as they do for the skinny kernel.  The tiled kernel cannot take them: its weights go
// from memory straight into LDS in MFMA operand order, and an 8-bit tile would have to be widened
// on the way.  Here only the activations go through LDS (a ring of [M, 64] k-chunks, direct-to-LDS
// loads, an XOR swizzle of the 16-byte slots).  The weights are the MFMA A operand and come from global
// memory into registers, one contiguous 1 KB block of the 8-bit pack (16 rows x 64 k) per load
// instruction, are widened to bf16 there (the hardware conversion is exact) and multiplied; the row
// scale is applied to the fp32 sums.  One workgroup = 128 packed weight rows, 4 waves along them (each
// wave two blocks of 16); the batch is the N dimension of v_mfma_f32_16x16x32_bf16, 16 rows per MFMA, all
// MT = ceil(M / 16) row blocks kept in accumulators.
//
// Memory latency under load is 2 - 3 us, so a CU needs about 40 KB of weights in flight to keep its
// share of the stream going: chunks are requested WG_AHEAD = 6 steps before they are multiplied.
// The vector-memory counter retires in order, so the activations have to be requested equally far
// ahead (a wait for chunk c's activations is a wait for everything requested before them).
//
// Every workgroup reads all M rows of the activations (from L2), so the time grows with M although
// the weight stream does not: measured on the 8B gate / up shape 24 us at 32 rows (the 117 MB of
// codes at 4.9 TB/s), 33 us at 64, 41 us at 128, against 46 - 52 us for the bf16 tiled kernel.
//
// Small N (the square projections) would give fewer workgroups than CUs, so K is split over
// gridDim.y like the tiled GEMM: fp32 partials (already scaled), then splitk_reduce_kernel applies
// the epilogue in a fixed order.  Without a split the epilogue (plain, residual, SwiGLU on the
// gate / up block pair of a wave) is applied here.
#include "pd_internal.h"

namespace pd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef const void __attribute__((address_space(1))) *gptr_t;
typedef void __attribute__((address_space(3))) *lptr_t;

constexpr int WG_KC = 64;        // k per chunk: one 128-byte activation row segment, two 32-wide MFMA k-steps
constexpr int WG_SETS = 8;       // LDS stages and weight register sets; chunk c lives in set c % WG_SETS
constexpr int WG_AHEAD = 6;      // a chunk is requested this many steps before its first fragment is read
                                 // (measured: a ring twice as deep changes nothing)

// 16-byte slot of a row's k-chunk in LDS: 8 consecutive rows (one 128-byte beat of a fragment read) use 8 different slots
__device__ __forceinline__ int wg_swz(int row, int chunk) { return chunk ^ (row & 7); }
__device__ __forceinline__ float wg_silu(float z) { return z / (1.0f + __expf(-z)); }

__device__ __forceinline__ bf16x8 wg_widen(unsigned w0, unsigned w1)
{
    auto f0 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w0, false);
    auto f1 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w0, true);
    auto f2 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w1, false);
    auto f3 = __builtin_amdgcn_cvt_pk_f32_fp8((int)w1, true);
    u32x4 r = {pack2bf(f0[0], f0[1]), pack2bf(f1[0], f1[1]), pack2bf(f2[0], f2[1]), pack2bf(f3[0], f3[1])};
    return __builtin_bit_cast(bf16x8, r);
}

// vmcnt(n): n in bits [3:0] and [15:14]; the other counters at "no wait"
#define PD_WG_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (7 << 4) | (15 << 8) | (((n) >> 4) << 14))

// The launcher makes every split a whole number of WG_SETS chunks, so the loop below has no
// conditional step: the compiler's own wait counts for the weight registers stay exact (after a
// conditional request it waits for everything outstanding).  Requests past the end of the split
// repeat its last chunk: they hit in cache, land in a stage or register set nobody reads again, and
// keep the number of requests per step constant.
// W8 = false: the same with bf16 weights from the block pack of wpack_off (two 1 KB blocks per row block
// and chunk, no widening, no scales).
template <int EPI, int MT, int WM, bool W8>
__global__ __launch_bounds__(256 * WM) void wgemm_kernel(GemmArgs a, int chunks_per_split)
{
    constexpr int NW = 4 * WM;                         // waves: 4 along the weight rows x WM along the batch
    constexpr int MTW = MT / WM;                       // row blocks of 16 batch rows per wave
    constexpr int ROWS = MT * 16;                      // padded batch rows held in LDS
    constexpr int A_BYTES = ROWS * WG_KC * 2;          // one stage
    static_assert(MT % (2 * WM) == 0, "a stage is loaded 8 rows per wave at a time");
    constexpr int A_LD = ROWS / 8 / NW;                // direct-to-LDS instructions per wave per stage
    constexpr int WL = W8 ? 2 : 4;                     // weight loads per wave per chunk (16 bytes per lane each)
    constexpr int LPC = A_LD + WL;                     // vector-memory instructions per wave per chunk
    static_assert(WG_AHEAD * LPC <= 63, "vector-memory counter range");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave & 3, wm = wave >> 2;
    const int n16 = lane & 15, kg = lane >> 4;
    const bool swiglu = EPI == EPI_SWIGLU || (EPI == EPI_PARTIAL && a.epilogue == EPI_SWIGLU);
    int rowblk[2];                                     // blocks of 16 packed weight rows of this wave
    if (swiglu) {
        // 64-row groups of the pack: gate rows 0-31, up rows 32-63; a wave takes a gate block and the up
        // block of the same 16 output columns
        const int ob = blockIdx.x * 4 + wn;
        rowblk[0] = (ob >> 1) * 4 + (ob & 1);
        rowblk[1] = rowblk[0] + 2;
    } else {
        rowblk[0] = (blockIdx.x * 4 + wn) * 2;
        rowblk[1] = rowblk[0] + 1;
    }
    const int n_cols = swiglu ? 2 * a.N : a.N;
    const int last_blk = (n_cols >> 4) - 1;
    const bool blk_ok0 = rowblk[0] <= last_blk, blk_ok1 = rowblk[1] <= last_blk;
    const size_t chunk_bytes = W8 ? 1024 : 2048;       // one row block's weights of a 64-k chunk
    const size_t blk_bytes = (size_t)(a.K >> 6) * chunk_bytes;
    const uint8_t *wbase = (const uint8_t *)(W8 ? a.B8 : a.B);
    const uint8_t *wp0 = wbase + (size_t)min(rowblk[0], last_blk) * blk_bytes + lane * 16;
    const uint8_t *wp1 = wbase + (size_t)min(rowblk[1], last_blk) * blk_bytes + lane * 16;

    // activation loader: instruction i of wave w moves rows 8 * (NW i + w) .. + 7; lane l owns LDS slot
    // (row, l % 8) and fetches chunk (l % 8) ^ swizzle(row) of that row (MT is even: ROWS / 8 is a
    // multiple of the 4 waves)
    uint32_t a_off[A_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        const int r = (i * NW + wave) * 8 + (lane >> 3);
        const int gr = r < a.M ? r : a.M - 1;          // padded rows repeat the last one; never stored
        a_off[i] = (uint32_t)gr * (uint32_t)(a.lda * 2) + wg_swz(r, lane & 7) * 16;
    }
    const int c_begin = blockIdx.y * chunks_per_split;
    const int n_chunks = min(a.K / WG_KC, c_begin + chunks_per_split) - c_begin;   // a multiple of WG_SETS
    // Every workgroup reads the same activations, and a [M, 64] chunk of a matrix whose rows are a
    // multiple of 4 KB apart sits in one or two L2 channels: workgroups that walk K in step all queue
    // on that channel.  So the workgroups of an XCD (every 8th one) start at evenly spread chunks and
    // wrap around; the order of the fp32 sums differs per workgroup and is fixed for a given launch shape.
    const int rot = (int)(((blockIdx.x >> 3) * (unsigned)n_chunks) / ((gridDim.x + 7) >> 3));
    auto issue = [&](int c, int set, u32x4 (&w)[WL]) { // chunk c (relative to c_begin) into stage / register set `set`
        int cr = min(c, n_chunks - 1) + rot;
        if (cr >= n_chunks) cr -= n_chunks;
        const int cc = c_begin + cr;
        const char *ab = (const char *)a.A + (size_t)cc * (WG_KC * 2);
        unsigned char *st = smem + set * A_BYTES;
#pragma unroll
        for (int i = 0; i < A_LD; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t)(ab + a_off[i]), (lptr_t)(st + (i * NW + wave) * 1024), 16, 0, 0);
        if (W8) {                                      // one load = both k-steps of a row block
            w[0] = *(const u32x4 *)(wp0 + (size_t)cc * 1024);
            w[1] = *(const u32x4 *)(wp1 + (size_t)cc * 1024);
        } else {                                       // [row block][k-step]
            w[0] = *(const u32x4 *)(wp0 + (size_t)cc * 2048);
            w[1] = *(const u32x4 *)(wp0 + (size_t)cc * 2048 + 1024);
            w[WL - 2] = *(const u32x4 *)(wp1 + (size_t)cc * 2048);
            w[WL - 1] = *(const u32x4 *)(wp1 + (size_t)cc * 2048 + 1024);
        }
    };

    f32x4 acc[2][MTW];                               // [weight row block][batch row block of this wave]
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int mb = 0; mb < MTW; ++mb) acc[rb][mb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // activation fragment (this wave's row block mb, k-step ks) of the chunk in stage `set`
    auto frag = [&](int set, int ks, int mb) -> bf16x8 {
        const int r = (wm * MTW + mb) * 16 + n16;
        return *(const bf16x8 *)(smem + set * A_BYTES + r * 128 + wg_swz(r, 4 * ks + kg) * 16);
    };
    // piece p of widening one chunk's weights: [row block p / 2][k-step p % 2]
    auto widen = [&](const u32x4 (&w)[WL], bf16x8 (&o)[2][2], int p) {
        if (W8) o[p >> 1][p & 1] = wg_widen(w[p >> 1][2 * (p & 1)], w[p >> 1][2 * (p & 1) + 1]);
        else o[p >> 1][p & 1] = __builtin_bit_cast(bf16x8, w[W8 ? 0 : p]);
    };

    u32x4 w[WG_SETS][WL];
    bf16x8 x0[MTW], x1[MTW];                             // fragments of k-step 0 and 1
    bf16x8 wf[2][2][2];                                // widened weights of this and the next chunk: [c % 2][row block][k-step]
    // start-up: requests in the order of the steady state (the waits below count on it); then chunk 0's
    // first fragments and weights
#pragma unroll
    for (int j = 0; j <= WG_AHEAD; ++j) {
        issue(j, j, w[j]);
        __builtin_amdgcn_sched_barrier(0);
    }
    PD_WG_VMCNT(WG_AHEAD * LPC);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int mb = 0; mb < MTW; ++mb) x0[mb] = frag(0, 0, mb);
#pragma unroll
    for (int p = 0; p < 4; ++p) widen(w[0], wf[0], p);
    __builtin_amdgcn_sched_barrier(0);

    // The waves of a workgroup move in step (one barrier per chunk) and a SIMD holds one or two of
    // them, so little hides an LDS round trip or a conversion unless the overlap is written out:
    // every pair of MFMAs is preceded by the LDS read of a fragment needed one phase later, and the
    // widening of the next chunk's weights is spread between the MFMAs of the second k-step.
    //   phase A: MFMAs of k-step 0 of chunk c          | reads: k-step 1 of chunk c
    //   middle : chunk c + 1 has landed (wait, barrier) | requests: chunk c + 1 + WG_AHEAD, into the stage
    //            of chunk c - 1, which every wave finished reading before this barrier
    //   phase B: MFMAs of k-step 1 of chunk c          | reads: k-step 0 of chunk c + 1; widen chunk c + 1
    // Requests retire in order, so "chunk c + 1 has landed" is "at most the requests of the
    // WG_AHEAD - 1 steps after its own are outstanding".
    for (int c = 0; c < n_chunks; c += WG_SETS) {
#pragma unroll
        for (int j = 0; j < WG_SETS; ++j) {
            const int nxt = (j + 1) % WG_SETS;
#pragma unroll
            for (int mb = 0; mb < MTW; ++mb) {
                x1[mb] = frag(j, 1, mb);
                acc[0][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j & 1][0][0], x0[mb], acc[0][mb], 0, 0, 0);
                acc[1][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j & 1][1][0], x0[mb], acc[1][mb], 0, 0, 0);
            }
#pragma unroll
            for (int mb = 0; mb < MTW; ++mb) {          // issue order: one LDS read, two MFMAs, ...
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            PD_WG_VMCNT((WG_AHEAD - 1) * LPC);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            issue(c + j + 1 + WG_AHEAD, (j + 1 + WG_AHEAD) % WG_SETS, w[(j + 1 + WG_AHEAD) % WG_SETS]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mb = 0; mb < MTW; ++mb) {
                x0[mb] = frag(nxt, 0, mb);
                acc[0][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j & 1][0][1], x1[mb], acc[0][mb], 0, 0, 0);
                acc[1][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[j & 1][1][1], x1[mb], acc[1][mb], 0, 0, 0);
            }
#pragma unroll
            for (int p = 0; p < 4; ++p) widen(w[nxt], wf[nxt & 1], p);
#pragma unroll
            for (int mb = 0; mb < MTW; ++mb) {          // one LDS read, a share of the 32 conversions, two MFMAs, ...
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                if (W8) __builtin_amdgcn_sched_group_barrier(0x002, (32 + MTW - 1) / MTW, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // ---- epilogue: lane (batch row 16 mb + n16, kg) holds packed weight rows 4 kg + j of each block --
    if (W8) {
        const f32x4 sc0 = *(const f32x4 *)(a.b_scale + min(rowblk[0], last_blk) * 16 + 4 * kg);
        const f32x4 sc1 = *(const f32x4 *)(a.b_scale + min(rowblk[1], last_blk) * 16 + 4 * kg);
#pragma unroll
        for (int mb = 0; mb < MTW; ++mb) {
            acc[0][mb] *= sc0;
            acc[1][mb] *= sc1;
        }
    }
    if (EPI == EPI_PARTIAL) {
        float *P = a.splitk_ws + (size_t)blockIdx.y * a.M * n_cols;
#pragma unroll
        for (int mb = 0; mb < MTW; ++mb) {
            const int m = (wm * MTW + mb) * 16 + n16;
            if (m >= a.M) continue;
            if (blk_ok0) *(f32x4 *)(P + (size_t)m * n_cols + rowblk[0] * 16 + 4 * kg) = acc[0][mb];
            if (blk_ok1) *(f32x4 *)(P + (size_t)m * n_cols + rowblk[1] * 16 + 4 * kg) = acc[1][mb];
        }
        return;
    }
    uint16_t *C = (uint16_t *)a.C;
    const uint16_t *R = (const uint16_t *)a.R;
#pragma unroll
    for (int mb = 0; mb < MTW; ++mb) {
        const int m = (wm * MTW + mb) * 16 + n16;
        if (m >= a.M) continue;
        if (EPI == EPI_SWIGLU) {
            if (!blk_ok1) continue;
            const int col = (blockIdx.x * 4 + wn) * 16 + 4 * kg;       // output columns of this wave
            uint2 o;
            o.x = pack2bf(wg_silu(acc[0][mb][0]) * acc[1][mb][0], wg_silu(acc[0][mb][1]) * acc[1][mb][1]);
            o.y = pack2bf(wg_silu(acc[0][mb][2]) * acc[1][mb][2], wg_silu(acc[0][mb][3]) * acc[1][mb][3]);
            *(uint2 *)(C + (size_t)m * a.ldc + col) = o;
        } else {
#pragma unroll
            for (int rb = 0; rb < 2; ++rb) {
                if (!(rb == 0 ? blk_ok0 : blk_ok1)) continue;
                const int col = rowblk[rb] * 16 + 4 * kg;
                float v0 = acc[rb][mb][0], v1 = acc[rb][mb][1], v2 = acc[rb][mb][2], v3 = acc[rb][mb][3];
                if (EPI == EPI_RESIDUAL) {
                    const uint2 rr = *(const uint2 *)(R + (size_t)m * a.ldr + col);
                    v0 += bfbits2f(rr.x & 0xffffu); v1 += bfbits2f(rr.x >> 16);
                    v2 += bfbits2f(rr.y & 0xffffu); v3 += bfbits2f(rr.y >> 16);
                }
                uint2 o;
                o.x = pack2bf(v0, v1);
                o.y = pack2bf(v2, v3);
                *(uint2 *)(C + (size_t)m * a.ldc + col) = o;
            }
        }
    }
}

bool wgemm_mfma_supported(const GemmArgs &a)
{
    if ((a.B8 && !a.b_scale) || (!a.B8 && !a.B) || a.group_offsets || a.a_gather || !a.packed) return false;
    // bf16 weights: only up to 32 rows does this beat the tiled kernels (decode step 0.189 -> 0.184 ms at
    // 32 rows, but 0.246 -> 0.269 at 64 and 0.367 -> 0.392 at 128: twice the bytes per weight make the
    // waves wait where the tiled kernel's LDS ring does not)
    if (a.M <= 16 || a.M > (a.B8 ? 128 : 32)) return false;
    const int64_t n_cols = a.epilogue == EPI_SWIGLU ? 2 * (int64_t)a.N : a.N;
    // whole register-set rounds of chunks; whole 16-row weight blocks; 8-byte stores
    if (a.K % (WG_KC * 8) != 0 || n_cols % 16 != 0 || a.ldb != a.K) return false;
    if (a.lda % 8 != 0 || a.ldc % 4 != 0 || (a.epilogue == EPI_RESIDUAL && a.ldr % 4 != 0)) return false;
    if (a.epilogue == EPI_SWIGLU && a.N % 32 != 0) return false;
    if ((int64_t)a.lda * 2 * a.M >= (1ll << 32)) return false;
    return true;
}

template <int MT, int WM, bool W8>
static hipError_t launch_wgemm_t(const GemmArgs &a, hipStream_t s)
{
    const int n_cols = a.epilogue == EPI_SWIGLU ? 2 * a.N : a.N;
    const int wgs = (n_cols + 127) / 128;
    const int rounds = a.K / (WG_KC * WG_SETS);        // a split is a whole number of these
    // K split: about one workgroup per CU; the partials must fit the scratch
    int splits = 1;
    if (a.splitk_ws && a.N % 4 == 0 && wgs < 192) {
        splits = 256 / wgs;
        if (splits > rounds) splits = rounds;
        while (splits > 1 && (size_t)splits * a.M * n_cols > a.splitk_ws_elems) --splits;
    }
    const int per = (rounds + splits - 1) / splits;
    splits = (rounds + per - 1) / per;
    const size_t smem = (size_t)WG_SETS * MT * 16 * WG_KC * 2;
    const dim3 grid((unsigned)wgs, (unsigned)splits);
#define PD_WG_LAUNCH(EPI)                                                                                    \
    do {                                                                                                     \
        auto kern = wgemm_kernel<EPI, MT, WM, W8>;                                                           \
        static OncePerDevice attr;                                                                           \
        int dev;                                                                                             \
        if (attr.need(&dev)) {                                                                               \
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                               (int)smem);                                                   \
            if (e != hipSuccess) return e;                                                                   \
            attr.mark(dev);                                                                                  \
        }                                                                                                    \
        kern<<<grid, 256 * WM, smem, s>>>(a, per * WG_SETS);                                                 \
    } while (0)
    if (splits > 1) {
        PD_WG_LAUNCH(EPI_PARTIAL);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        return launch_splitk_reduce(a, splits, s);
    }
    switch (a.epilogue) {
    case EPI_NONE: PD_WG_LAUNCH(EPI_NONE); break;
    case EPI_RESIDUAL: PD_WG_LAUNCH(EPI_RESIDUAL); break;
    default: PD_WG_LAUNCH(EPI_SWIGLU); break;
    }
#undef PD_WG_LAUNCH
    return hipGetLastError();
}

hipError_t launch_wgemm_mfma(const GemmArgs &a, hipStream_t s)
{
    if (!a.B8) return launch_wgemm_t<2, 1, false>(a, s);    // bf16 weights: up to 32 rows only
    // 4 waves, or 8 with the batch rows split between two waves per SIMD (fewer registers each; the
    // measured times are the same)
    if (a.M <= 32) return launch_wgemm_t<2, 1, true>(a, s);
    if (a.M <= 64) return launch_wgemm_t<4, 2, true>(a, s);
    if (a.M <= 96) return launch_wgemm_t<6, 1, true>(a, s);
    return launch_wgemm_t<8, 2, true>(a, s);
}

}  // namespace pd
