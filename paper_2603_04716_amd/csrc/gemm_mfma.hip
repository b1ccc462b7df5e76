// bf16 GEMM on the CDNA4 matrix cores:  C[M,N] = epilogue(A[M,K] * B[N,K]^T), fp32 accumulation.
//
// Both operands are K-contiguous, which is exactly the per-lane operand layout of
// v_mfma_f32_32x32x16_bf16 (each lane supplies 8 consecutive k of one row / column), so tiles go
// global -> LDS with the direct-to-LDS 16-byte loads of gfx950 (no staging registers, no LDS
// write instructions) and LDS -> registers with 16-byte reads, with no transposition anywhere.
// A direct load puts lane i's 16 bytes at LDS offset base + 16*i, so the XOR swizzle that keeps
// the fragment reads free of bank conflicts is applied on the global side: the lane that owns LDS
// slot (row, s) fetches chunk s ^ ((row >> 1) & 7) of that row.  LDS holds NS stages: the loads of
// the next NS-1 k-tiles are in flight while the matrix cores work on tile k; one barrier per tile.
//
// The weight operand B arrives in the packed block layout of pd_internal.h (1 KB blocks of 16 rows
// x 32 k): one direct-to-LDS instruction moves one block, blocks sit linearly in LDS, and the
// fragment reads of 16 consecutive lanes are 256 contiguous bytes, so B needs no swizzle.
//
// Epilogues: plain store, residual add, and SwiGLU.  For SwiGLU the weight is packed at layer
// creation as alternating 32-row blocks (gate rows j..j+31, then up rows j..j+31); an MFMA output
// block pair then holds gate and up of the same (row, column) in the same lane and register, and
// silu(gate)*up is formed without any data exchange.
//
// Optional row gather on A and per-group B matrices serve the mixture-of-experts grouped GEMM.
//
// Decode-sized problems (M <= 256) have too few output tiles to occupy 256 CUs while the weights
// stream from HBM, so K is split over gridDim.y: each split writes an fp32 partial tile and a
// second small kernel adds the splits in a fixed order and applies the epilogue (deterministic,
// no atomics).
#include <string.h>

#include "pd_internal.h"

namespace pd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ i32x8 cat32(bf16x8 lo, bf16x8 hi)
{
    const i32x4 l = __builtin_bit_cast(i32x4, lo), h = __builtin_bit_cast(i32x4, hi);
    return i32x8{l[0], l[1], l[2], l[3], h[0], h[1], h[2], h[3]};
}

constexpr int BK = 64;  // k per tile: 8 chunks of 16 bytes per row

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

__device__ __forceinline__ float silu_fast(float z) { return z / (1.0f + __expf(-z)); }

// F8: both operands are E4M3 codes and the caller passes them as if two codes were one bf16 element
// (K, lda, ldb halved; the weight pack is the bf16 pack of that view), so every byte moves exactly as
// above.  Two consecutive 16-byte fragments of a lane form the 32-byte operand of
// v_mfma_f32_32x32x64_f8f6f4: which of the 64 k of the step a byte stands for does not matter as long
// as both operands are assembled the same way, and they are.  The fp32 sums are multiplied by the
// scale of their activation row and of their weight row before any epilogue.
template <int BM, int BN, int WAVES_M, int WAVES_N, int EPI, int NS, bool F8 = false>
__global__ __launch_bounds__(64 * WAVES_M *WAVES_N) void gemm_mfma_kernel(GemmArgs a, int tiles_m,
                                                                          int tiles_n, int kt_per_split)
{
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;   // wave tile
    constexpr int MB = WM / 32, NB = WN / 32;             // 32x32 blocks per wave
    static_assert(EPI != EPI_SWIGLU || NB % 2 == 0, "SwiGLU pairs two column blocks");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2, STAGE = A_BYTES + B_BYTES;

    // ---- tile id: contiguous ranges of tiles per XCD, 8-row bands inside ------------------------
    const int n_tiles = tiles_m * tiles_n;
    int pid = blockIdx.x;
    {
        const int per = n_tiles / 8, rem = n_tiles % 8;
        if (per > 0) {
            // blocks are dealt to the 8 XCDs round-robin; give each XCD one contiguous range
            int xcd = pid % 8, j = pid / 8;
            if (j < per) pid = xcd * per + j;
            else pid = 8 * per + (pid - 8 * per);   // leftover tiles keep their order
            (void)rem;
        }
    }
    int tm, tn;
    {
        constexpr int GM = 8;
        int band = pid / (GM * tiles_n);
        int first = band * GM;
        int rows = tiles_m - first < GM ? tiles_m - first : GM;
        int in = pid - band * GM * tiles_n;
        tm = first + in % rows;
        tn = in / rows;
    }

    // ---- rows of this tile (virtual m-tiles map to groups for the grouped GEMM) -----------------
    int row0, row_end, group = 0;
    if (a.group_offsets) {
        int acc = 0;
        row0 = -1;
        row_end = 0;
        for (int g = 0; g < a.n_groups; ++g) {
            int lo = a.group_offsets[g], hi = a.group_offsets[g + 1];
            int nt = (hi - lo + BM - 1) / BM;
            if (tm < acc + nt) {
                group = g;
                row0 = lo + (tm - acc) * BM;
                row_end = hi;
                break;
            }
            acc += nt;
        }
        if (row0 < 0) return;
    } else {
        row0 = tm * BM;
        row_end = a.M;
    }
    const int col0 = tn * BN;
    // rows of (packed) B; a split-K launch of a SwiGLU GEMM works on the packed columns
    const int n_cols = (EPI == EPI_SWIGLU || (EPI == EPI_PARTIAL && a.epilogue == EPI_SWIGLU)) ? 2 * a.N : a.N;
    const __bf16 *A = (const __bf16 *)a.A;
    const __bf16 *B = (const __bf16 *)a.B + (size_t)group * a.b_group_stride;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    // ---- loader: wave instruction i covers 8 rows x 128 bytes = 1 KB of LDS; lane l owns slot
    //      (row = 8*blk + l/8, s = l%8) and fetches chunk s ^ swizzle(row) of that row ------------------
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int A_LD = BM / 8 / NW, B_LD = BN / 8 / NW;   // load instructions per wave
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "loader mapping");
    uint32_t a_off[A_LD], b_off[B_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        int r = (i * NW + wave) * 8 + (lane >> 3);
        int c = swz(r, lane & 7);
        int gr = row0 + r;
        if (gr >= row_end) gr = row_end - 1;          // clamp: loaded but never stored
        if (a.a_gather) gr = a.a_gather[gr];
        a_off[i] = (uint32_t)gr * (uint32_t)(a.lda * 2) + c * 16;
    }
    // B: instruction j = i*NW + wave moves packed block (row block j/2, k block j%2 of the tile)
    const int kblocks = a.K >> 5;                      // 32-k blocks per row block
    const int last_rb = (n_cols - 1) >> 4;
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        const int j = i * NW + wave;
        int rb = (col0 >> 4) + (j >> 1);
        if (rb > last_rb) rb = last_rb;               // clamp: loaded but never stored
        b_off[i] = ((uint32_t)rb * (uint32_t)kblocks + (j & 1)) * 1024u + lane * 16;
    }
    typedef const void __attribute__((address_space(1))) *gptr_t;
    typedef void __attribute__((address_space(3))) *lptr_t;
    auto issue_loads = [&](int kt, unsigned char *st) {
        const char *ab = (const char *)A + (size_t)kt * (BK * 2);
        const char *bb = (const char *)B + (size_t)kt * 2048;   // two 1 KB k-blocks per tile
#pragma unroll
        for (int i = 0; i < A_LD; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t)(ab + a_off[i]),
                                             (lptr_t)(st + (i * NW + wave) * 1024), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < B_LD; ++i)
            __builtin_amdgcn_global_load_lds((gptr_t)(bb + b_off[i]),
                                             (lptr_t)(st + A_BYTES + (i * NW + wave) * 1024), 16, 0, 0);
    };

    f32x16 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int kt0 = blockIdx.y * kt_per_split;
    const int kt1 = min(a.K / BK, kt0 + kt_per_split);
    // Software pipeline over NS LDS stages: the loads of k-tile kt + NS - 1 are issued while tile
    // kt is multiplied, so up to NS - 1 tiles are in flight per workgroup.  Direct-to-LDS loads
    // retire in order through this wave's vector-memory counter, so "tile kt has landed" is
    // "at most (tiles issued after kt) * loads-per-tile still outstanding", followed by a barrier
    // that makes every wave's part visible.  The same barrier orders the refill of the stage that
    // was multiplied in the previous iteration.
    constexpr int LPS = A_LD + B_LD;                  // load instructions per tile per wave
    static_assert(LPS * (NS - 1) <= 63, "vector-memory counter range");
    auto wait_tiles_after = [&](int tiles_after) {
        // s_waitcnt vmcnt(n): n in bits [3:0] and [15:14]; expcnt / lgkmcnt fields left at "no wait"
#define PD_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (7 << 4) | (15 << 8) | (((n) >> 4) << 14))
        if (NS >= 7 && tiles_after >= 5) PD_VMCNT((5 * LPS) & 63);
        else if (NS >= 6 && tiles_after >= 4) PD_VMCNT((4 * LPS) & 63);
        else if (NS >= 5 && tiles_after >= 3) PD_VMCNT((3 * LPS) & 63);
        else if (NS >= 4 && tiles_after >= 2) PD_VMCNT(2 * LPS);
        else if (NS >= 3 && tiles_after >= 1) PD_VMCNT(1 * LPS);
        else PD_VMCNT(0);
#undef PD_VMCNT
    };
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (kt0 + s < kt1) issue_loads(kt0 + s, smem + s * STAGE);
    if (NS == 2) __syncthreads();

    // fragment addresses inside a stage: row and the two chunk parities of this lane
    const int frow = lane & 31, fhalf = lane >> 5;
    // Fragment reads of one 16-wide k-step, then its MFMAs; with two waves per SIMD the other
    // wave's matrix work covers this wave's LDS latency (measured: explicit register double
    // buffering of the fragments changes nothing).
    auto load_frags = [&](const unsigned char *st, int kk, bf16x8 (&fa)[MB], bf16x8 (&fb)[NB]) {
        const int c = kk * 2 + fhalf;
#pragma unroll
        for (int i = 0; i < MB; ++i) {
            int r = wm * WM + i * 32 + frow;
            fa[i] = *(const bf16x8 *)(st + r * 128 + swz(r, c) * 16);
        }
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            // column wn*WN + 32j + frow, k chunk c of the tile, in the linear packed blocks
            const int rbl = ((wn * WN + j * 32) >> 4) + (frow >> 4);
            fb[j] = *(const bf16x8 *)(st + A_BYTES + (rbl * 2 + (c >> 2)) * 1024 + (c & 3) * 256 + (frow & 15) * 16);
        }
    };
    auto mma = [&](bf16x8 (&fa)[MB], bf16x8 (&fb)[NB]) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    };
    auto compute = [&](const unsigned char *st) {
        if (F8) {
#pragma unroll
            for (int kk = 0; kk < BK / 16; kk += 2) {
                bf16x8 fa[2][MB], fb[2][NB];
                load_frags(st, kk, fa[0], fb[0]);
                load_frags(st, kk + 1, fa[1], fb[1]);
                i32x8 pb[NB];
#pragma unroll
                for (int j = 0; j < NB; ++j) pb[j] = cat32(fb[0][j], fb[1][j]);
#pragma unroll
                for (int i = 0; i < MB; ++i) {
                    const i32x8 pa = cat32(fa[0][i], fa[1][i]);
#pragma unroll
                    for (int j = 0; j < NB; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(pa, pb[j], acc[i][j], 0, 0, 0, 0, 0, 0);
                }
            }
            return;
        }
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 fa[MB], fb[NB];
            load_frags(st, kk, fa, fb);
            mma(fa, fb);
        }
    };
    if (NS == 2) {
        // double buffer: the barrier that ends an iteration also waits for the loads issued at its
        // start; the compiler may sink trailing MFMAs below it, which hides the barrier wait
        for (int kt = kt0; kt + 1 < kt1; ++kt) {
            issue_loads(kt + 1, smem + ((kt + 1 - kt0) & 1) * STAGE);
            __builtin_amdgcn_sched_barrier(0);     // keep the loads ahead of the compute phase
            compute(smem + ((kt - kt0) & 1) * STAGE);
            __syncthreads();
        }
        compute(smem + ((kt1 - 1 - kt0) & 1) * STAGE);
    } else {
        for (int kt = kt0; kt < kt1; ++kt) {
            const int issued_after = min(NS - 2, kt1 - 1 - kt);   // tiles already issued beyond kt
            wait_tiles_after(issued_after);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            if (kt + NS - 1 < kt1) issue_loads(kt + NS - 1, smem + ((kt + NS - 1 - kt0) % NS) * STAGE);
            __builtin_amdgcn_sched_barrier(0);     // keep the loads ahead of the compute phase
            compute(smem + ((kt - kt0) % NS) * STAGE);
        }
    }

    // ---- epilogue: lane holds column (lane % 32) of each block; register r is row
    //      8*(r/4) + 4*(lane/32) + r%4 ----------------------------------------------------------------
    if (F8) {
        float sb[NB];
#pragma unroll
        for (int j = 0; j < NB; ++j)
            sb[j] = a.b_scale[(size_t)group * n_cols + min(col0 + wn * WN + j * 32 + frow, n_cols - 1)];
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = row0 + wm * WM + i * 32 + 8 * (r >> 2) + 4 * fhalf + (r & 3);
                int mr = min(m, row_end - 1);
                if (a.a_gather) mr = a.a_gather[mr];        // the scale belongs to the row the codes came from
                const float sa = a.a_scale[mr];
#pragma unroll
                for (int j = 0; j < NB; ++j) acc[i][j][r] *= sa * sb[j];
            }
    }
    if (EPI == EPI_PARTIAL) {
        float *P = a.splitk_ws + (size_t)blockIdx.y * a.M * n_cols;
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = row0 + wm * WM + i * 32 + 8 * (r >> 2) + 4 * fhalf + (r & 3);
                if (m >= row_end) continue;
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const int n = col0 + wn * WN + j * 32 + frow;
                    if (n < n_cols) P[(size_t)m * n_cols + n] = acc[i][j][r];
                }
            }
        return;
    }
    uint16_t *C = (uint16_t *)a.C;
    const uint16_t *R = (const uint16_t *)a.R;
    // Row-contiguous stores: the accumulators hold one column per lane, which would make every store
    // (and residual load) a 2-byte access.  Each wave instead passes its 32-row blocks through a
    // private 8 KB of the (now idle) operand stages as fp32 and reads them back with 4 consecutive
    // columns per lane, so a wave instruction moves whole 128-byte row segments; the residual is
    // added in fp32 before the one rounding to bf16.
    constexpr bool kStage = WN == 64 && NB == 2;
    if (kStage && a.N % 4 == 0 && a.ldc % 4 == 0 && (EPI != EPI_RESIDUAL || a.ldr % 4 == 0)) {
        constexpr int OC = EPI == EPI_SWIGLU ? 32 : 64;   // output columns of a staged block
        constexpr int LPR = OC / 4, RPI = 64 / LPR;      // lanes per row, rows per wave instruction
        __syncthreads();                                  // every wave is done with the operand stages
        float *stg = (float *)smem + wave * 2048;
        const int out_col0 = EPI == EPI_SWIGLU ? ((col0 + wn * WN) >> 6) * 32 : col0 + wn * WN;
#pragma unroll
        for (int i = 0; i < MB; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = 8 * (r >> 2) + 4 * fhalf + (r & 3);
                if (EPI == EPI_SWIGLU) {
                    stg[row * OC + frow] = silu_fast(acc[i][0][r]) * acc[i][1][r];
                } else {
                    stg[row * OC + frow] = acc[i][0][r];
                    stg[row * OC + 32 + frow] = acc[i][1][r];
                }
            }
#pragma unroll
            for (int it = 0; it < 32 / RPI; ++it) {
                const int row = it * RPI + lane / LPR, cg = (lane % LPR) * 4;
                const f32x4 v = *(const f32x4 *)(stg + row * OC + cg);
                const int m = row0 + wm * WM + i * 32 + row, n = out_col0 + cg;
                if (m < row_end && n < a.N) {
                    float o0 = v[0], o1 = v[1], o2 = v[2], o3 = v[3];
                    if (EPI == EPI_RESIDUAL) {
                        const uint2 rr = *(const uint2 *)(R + (size_t)m * a.ldr + n);
                        o0 += bfbits2f(rr.x & 0xffffu); o1 += bfbits2f(rr.x >> 16);
                        o2 += bfbits2f(rr.y & 0xffffu); o3 += bfbits2f(rr.y >> 16);
                    }
                    uint2 o;
                    o.x = pack2bf(o0, o1);
                    o.y = pack2bf(o2, o3);
                    *(uint2 *)(C + (size_t)m * a.ldc + n) = o;
                }
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < MB; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = row0 + wm * WM + i * 32 + 8 * (r >> 2) + 4 * fhalf + (r & 3);
            if (m >= row_end) continue;
            if (EPI == EPI_SWIGLU) {
#pragma unroll
                for (int j = 0; j < NB; j += 2) {
                    const int np = col0 + wn * WN + j * 32;       // packed column of the gate block
                    const int f = (np >> 6) * 32 + frow;
                    if (f < a.N) {
                        float v = silu_fast(acc[i][j][r]) * acc[i][j + 1][r];
                        C[(size_t)m * a.ldc + f] = f2bf(v).x;
                    }
                }
            } else {
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const int n = col0 + wn * WN + j * 32 + frow;
                    if (n < a.N) {
                        float v = acc[i][j][r];
                        if (EPI == EPI_RESIDUAL) v += bfbits2f(R[(size_t)m * a.ldr + n]);
                        C[(size_t)m * a.ldc + n] = f2bf(v).x;
                    }
                }
            }
        }
    }
}

// out = epilogue(sum over splits of the fp32 partials); 4 consecutive output columns per thread.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmArgs a, int splits)
{
    const int n4 = a.N / 4;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)a.M * n4) return;
    const int m = (int)(idx / n4), n = (int)(idx % n4) * 4;
    const int n_cols = a.epilogue == EPI_SWIGLU ? 2 * a.N : a.N;
    const size_t plane = (size_t)a.M * n_cols;
    float v[4];
    if (a.epilogue == EPI_SWIGLU) {
        const int pc = (n >> 5) * 64 + (n & 31);     // packed gate column; up is 32 further
        float4 g = make_float4(0.f, 0.f, 0.f, 0.f), u = g;
        for (int z = 0; z < splits; ++z) {
            const float *p = a.splitk_ws + z * plane + (size_t)m * n_cols + pc;
            float4 gz = *(const float4 *)p, uz = *(const float4 *)(p + 32);
            g.x += gz.x; g.y += gz.y; g.z += gz.z; g.w += gz.w;
            u.x += uz.x; u.y += uz.y; u.z += uz.z; u.w += uz.w;
        }
        v[0] = silu_fast(g.x) * u.x; v[1] = silu_fast(g.y) * u.y;
        v[2] = silu_fast(g.z) * u.z; v[3] = silu_fast(g.w) * u.w;
    } else {
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int z = 0; z < splits; ++z) {
            float4 tz = *(const float4 *)(a.splitk_ws + z * plane + (size_t)m * n_cols + n);
            t.x += tz.x; t.y += tz.y; t.z += tz.z; t.w += tz.w;
        }
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
        if (a.epilogue == EPI_RESIDUAL) {
            uint2 rr = *(const uint2 *)((const uint16_t *)a.R + (size_t)m * a.ldr + n);
            v[0] += bfbits2f(rr.x & 0xffffu); v[1] += bfbits2f(rr.x >> 16);
            v[2] += bfbits2f(rr.y & 0xffffu); v[3] += bfbits2f(rr.y >> 16);
        }
    }
    uint2 o;
    o.x = pack2bf(v[0], v[1]);
    o.y = pack2bf(v[2], v[3]);
    *(uint2 *)((uint16_t *)a.C + (size_t)m * a.ldc + n) = o;
}

// The same sum for an EPI_RESIDUAL product whose rows are normalised next: one workgroup per row adds the
// partials and the residual, stores the row (bf16) and its RMSNorm (statistics in fp32 on the stored,
// rounded values, exactly what a separate norm launch would read); the workgroups behind the M rows do
// the cache append of a decode step (rmsnorm_append_kernel's second half).
__global__ __launch_bounds__(512) void splitk_reduce_norm_kernel(GemmArgs a, int splits, RopeArgs ap, int n_append)
{
    __shared__ float red[8];
    __shared__ float cs[128], sn[128];
    const int m = blockIdx.x;
    if (m >= a.M) {
        if (m - a.M < n_append) append_token_body(ap, m - a.M, cs, sn);
        return;
    }
    const int n8 = a.N / 8, nt = blockDim.x;
    const size_t plane = (size_t)a.M * a.N;
    const uint16_t *R = (const uint16_t *)a.R + (size_t)m * a.ldr;
    uint16_t *C = (uint16_t *)a.C + (size_t)m * a.ldc;
    uint4 hrow[4];                                    // this thread's stored values: up to 4 chunks of 8 columns
    float ss = 0.f;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int c8 = it * nt + threadIdx.x;
        if (c8 >= n8) break;
        const int n = c8 * 8;
        float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        const float *p = a.splitk_ws + (size_t)m * a.N + n;
        const uint4 rr = *(const uint4 *)(R + n);
        int z = 0;
        // four splits' loads in flight at a time: one round trip to the L2 per four splits
        for (; z + 4 <= splits; z += 4) {
            float4 t[8];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                t[2 * u] = *(const float4 *)(p + (z + u) * plane);
                t[2 * u + 1] = *(const float4 *)(p + (z + u) * plane + 4);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {             // in split order: the sum does not depend on the grouping
                v[0] += t[2 * u].x; v[1] += t[2 * u].y; v[2] += t[2 * u].z; v[3] += t[2 * u].w;
                v[4] += t[2 * u + 1].x; v[5] += t[2 * u + 1].y; v[6] += t[2 * u + 1].z; v[7] += t[2 * u + 1].w;
            }
        }
        for (; z < splits; ++z) {
            const float4 t0 = *(const float4 *)(p + z * plane), t1 = *(const float4 *)(p + z * plane + 4);
            v[0] += t0.x; v[1] += t0.y; v[2] += t0.z; v[3] += t0.w;
            v[4] += t1.x; v[5] += t1.y; v[6] += t1.z; v[7] += t1.w;
        }
        const uint32_t rw[4] = {rr.x, rr.y, rr.z, rr.w};
        uint32_t o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            o[j] = pack2bf(v[2 * j] + bfbits2f(rw[j] & 0xffffu), v[2 * j + 1] + bfbits2f(rw[j] >> 16));
            const float x0 = bfbits2f(o[j] & 0xffffu), x1 = bfbits2f(o[j] >> 16);
            ss += x0 * x0 + x1 * x1;
        }
        hrow[it] = make_uint4(o[0], o[1], o[2], o[3]);
        *(uint4 *)(C + n) = hrow[it];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
    for (int w = 0; w < nt / 64; ++w) tot += red[w];
    const float inv = rsqrtf(tot * (1.0f / (float)a.N) + a.fuse_eps);
    uint16_t *Y = (uint16_t *)a.fuse_y + (size_t)m * a.N;
    const uint16_t *G = (const uint16_t *)a.fuse_g;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int c8 = it * nt + threadIdx.x;
        if (c8 >= n8) break;
        const int n = c8 * 8;
        const uint4 gg = *(const uint4 *)(G + n);
        const uint32_t w[4] = {hrow[it].x, hrow[it].y, hrow[it].z, hrow[it].w}, gw[4] = {gg.x, gg.y, gg.z, gg.w};
        uint32_t o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            o[j] = pack2bf(bfbits2f(w[j] & 0xffffu) * inv * bfbits2f(gw[j] & 0xffffu),
                           bfbits2f(w[j] >> 16) * inv * bfbits2f(gw[j] >> 16));
        *(uint4 *)(Y + n) = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

hipError_t launch_splitk_reduce(const GemmArgs &a, int splits, hipStream_t s)
{
    if (a.fuse_y && a.fuse_g && a.fuse_done && a.epilogue == EPI_RESIDUAL && a.N % 8 == 0 && a.N <= 8192 &&
        a.ldc % 8 == 0 && a.ldr % 8 == 0) {
        RopeArgs none;
        memset(&none, 0, sizeof(none));
        const int n_append = a.fuse_append ? a.fuse_append->T : 0;
        splitk_reduce_norm_kernel<<<a.M + n_append, a.N > 2048 ? 512 : 256, 0, s>>>(a, splits, a.fuse_append ? *a.fuse_append : none, n_append);
        *a.fuse_done = 1;
        return hipGetLastError();
    }
    const size_t n_out = (size_t)a.M * (a.N / 4);
    splitk_reduce_kernel<<<(unsigned)((n_out + 255) / 256), 256, 0, s>>>(a, splits);
    return hipGetLastError();
}

bool gemm_mfma_supported(const GemmArgs &a)
{
    if (a.K % BK != 0 || a.K <= 0 || a.M <= 0) return false;
    if (a.lda % 8 != 0 || a.ldb % 8 != 0) return false;
    // 32-bit byte offsets inside A and inside one group of B
    const int64_t brows = a.epilogue == EPI_SWIGLU ? 2 * (int64_t)a.N : a.N;
    if ((int64_t)a.ldb * 2 * brows >= (1ll << 32)) return false;
    if (!a.a_gather && (int64_t)a.lda * 2 * a.M >= (1ll << 32)) return false;
    if (a.a_gather && (int64_t)a.lda * 2 * a.M >= (1ll << 31)) return false;
    if (!a.packed || a.ldb != a.K || a.K % 32 != 0 || brows % 16 != 0) return false;
    if (a.epilogue == EPI_SWIGLU) return a.N % 32 == 0;
    return true;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int NS = 2, bool F8 = false>
static hipError_t launch_cfg(const GemmArgs &a, hipStream_t s, int splits = 1)
{
    const int n_cols = a.epilogue == EPI_SWIGLU ? 2 * a.N : a.N;
    const int tiles_n = (n_cols + BN - 1) / BN;
    const int tiles_m = (a.M + BM - 1) / BM + (a.group_offsets ? a.n_groups : 0);
    const size_t smem = NS * (size_t)(BM + BN) * BK * 2;
    const int nk = a.K / BK;
    const int kt_per = (nk + splits - 1) / splits;
    splits = (nk + kt_per - 1) / kt_per;               // no empty split
    const dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)splits);
    const dim3 block(64 * WAVES_M * WAVES_N);
#define LAUNCH(EPI)                                                                              \
    do {                                                                                         \
        auto kern = gemm_mfma_kernel<BM, BN, WAVES_M, WAVES_N, EPI, NS, F8>;                         \
        static OncePerDevice attr;                                                               \
        int dev;                                                                                 \
        if (attr.need(&dev)) {                                                                   \
            hipError_t e = hipFuncSetAttribute((const void *)kern,                               \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem); \
            if (e != hipSuccess) return e;                                                       \
            attr.mark(dev);                                                                      \
        }                                                                                        \
        kern<<<grid, block, smem, s>>>(a, tiles_m, tiles_n, kt_per);                             \
    } while (0)
    if (splits > 1) {
        // fp32 partials of every split must fit the scratch buffer
        if (!a.splitk_ws || (size_t)splits * a.M * n_cols > a.splitk_ws_elems) return hipErrorInvalidValue;
        LAUNCH(EPI_PARTIAL);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        return launch_splitk_reduce(a, splits, s);
    }
    switch (a.epilogue) {
    case EPI_NONE: LAUNCH(EPI_NONE); break;
    case EPI_RESIDUAL: LAUNCH(EPI_RESIDUAL); break;
    default: LAUNCH(EPI_SWIGLU); break;
    }
#undef LAUNCH
    return hipGetLastError();
}

// Split count for decode-sized problems: about one workgroup per CU (measured: more splits lose
// to the fp32 partial traffic, fewer leave CUs without a weight stream), at least 4 k-tiles per
// split, partials (written and read back) below about the weight bytes, and they must fit the
// scratch buffer.
static int choose_splits(const GemmArgs &a, int BM, int BN)
{
    if (!a.splitk_ws || a.N % 4 != 0 || a.ldc % 4 != 0 || (a.epilogue == EPI_RESIDUAL && a.ldr % 4 != 0))
        return 1;
    const int n_cols = a.epilogue == EPI_SWIGLU ? 2 * a.N : a.N;
    // row tiles that do work: for a grouped problem at most one per group and per row (rows are few here)
    int row_tiles = (a.M + BM - 1) / BM;
    if (a.group_offsets) row_tiles = a.M < a.n_groups ? a.M : a.n_groups;
    const int tiles = row_tiles * ((n_cols + BN - 1) / BN);
    const int nk = a.K / BK;
    int splits = 256 / tiles;                      // never more workgroups than CUs: a second, nearly
    if (splits > nk / 4) splits = nk / 4;          // empty round costs more than the idle CUs
    const int cap = a.K / (4 * a.M) > 1 ? a.K / (4 * a.M) : 1;
    if (splits > cap) splits = cap;
    while (splits > 1 && (size_t)splits * a.M * n_cols > a.splitk_ws_elems) --splits;
    return splits < 1 ? 1 : splits;
}

// Split count for chunk-sized problems (a few hundred to a few thousand rows): these are bound by
// the matrix pipe, but 256 x 256 tiles alone leave most CUs idle, so K is split until about one
// workgroup per CU exists (at least 8 k-tiles per split; the fp32 partials must fit the scratch).
static int choose_splits_mid(const GemmArgs &a)
{
    if (!a.splitk_ws || a.group_offsets || a.a_gather || a.N % 4 != 0 || a.ldc % 4 != 0 ||
        (a.epilogue == EPI_RESIDUAL && a.ldr % 4 != 0))
        return 1;
    const int n_cols = a.epilogue == EPI_SWIGLU ? 2 * a.N : a.N;
    const int tiles = ((a.M + 255) / 256) * ((n_cols + 255) / 256);
    if (tiles >= 192) return 1;
    int splits = (256 + tiles / 2) / tiles;
    const int nk = a.K / BK;
    if (splits > nk / 8) splits = nk / 8;
    while (splits > 1 && (size_t)splits * a.M * n_cols > a.splitk_ws_elems) --splits;
    return splits < 1 ? 1 : splits;
}

// 8-bit operands (see the kernel): a.A are E4M3 codes [M, 2 K] with a.a_scale per row, a.B the codes in
// the pack of the halved view with a.b_scale per packed row; a.K, a.lda, a.ldb count code pairs.
bool gemm_mfma_f8_supported(const GemmArgs &a)
{
    return gemm_mfma_supported(a) && a.a_scale && a.b_scale;
}

hipError_t launch_gemm_mfma_f8(const GemmArgs &a, hipStream_t s)
{
    // a decode batch of a few hundred rows is bound by the weight stream, not by the matrix pipe: for the
    // products with few columns narrow column tiles and K split over workgroups, as for bf16 (measured
    // at 448 rows: QKV 44 -> 26 us, O 46 -> 34, down 68 -> 57; the wide gate / up product is faster on
    // the large tiles, 65 against 74 us)
    if (a.M <= 512 && !a.group_offsets && (a.epilogue == EPI_SWIGLU ? 2 * a.N : a.N) < 16384)
        return launch_cfg<256, 64, 8, 1, 3, true>(a, s, choose_splits(a, 256, 64));
    // as for bf16: 16 waves for the short-K products (a.K counts code pairs)
    if (a.K <= 2048 && a.epilogue != EPI_SWIGLU && !a.group_offsets)
        return launch_cfg<256, 256, 4, 4, 2, true>(a, s, choose_splits_mid(a));
    return launch_cfg<256, 256, 2, 4, 2, true>(a, s, choose_splits_mid(a));
}

hipError_t launch_gemm_mfma(const GemmArgs &a, hipStream_t s)
{
    // rows that share a weight matrix: for a grouped problem the mean group size picks the tile
    // (larger groups take several row tiles)
    const int rows = a.group_offsets ? (a.M + a.n_groups - 1) / a.n_groups : a.M;
    if (rows > 256) {
        // 8 waves (two per SIMD hide each other's stalls); short-K problems spend relatively more time in
        // the prologue / epilogue, where 16 waves measured 5-8 % faster
        const int splits = choose_splits_mid(a);
        if (a.K <= 4096 && a.epilogue != EPI_SWIGLU && !a.group_offsets) return launch_cfg<256, 256, 4, 4, 2>(a, s, splits);
        return launch_cfg<256, 256, 2, 4, 2>(a, s, splits);
    }
    const int n_cols = a.epilogue == EPI_SWIGLU ? 2 * a.N : a.N;
    const bool wide = n_cols >= 16384;                            // enough column tiles without splitting K
    if (rows > 128) {
        if (wide) return launch_cfg<256, 128, 4, 2, 3>(a, s, 1);
        return launch_cfg<256, 64, 8, 1, 3>(a, s, choose_splits(a, 256, 64));
    }
    if (rows > 64) {
        if (wide) return launch_cfg<128, 128, 2, 2, 3>(a, s, 1);     // measured 52 vs 62 us on the gate/up shape
        return launch_cfg<128, 64, 4, 1, 4>(a, s, choose_splits(a, 128, 64));
    }
    return launch_cfg<64, 128, 2, 2, 4>(a, s, wide ? 1 : choose_splits(a, 64, 128));
}

}  // namespace pd
