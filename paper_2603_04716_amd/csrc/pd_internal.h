// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "pd.h"

namespace pd {

// bf16 storage element (raw bits); conversions are round-to-nearest-even.
struct bf16_t {
    uint16_t x;
};

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((uint32_t)v.x) << 16); }
__device__ __forceinline__ float bfbits2f(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
// fp32 -> bf16, round to nearest even: the hardware conversion of gfx950 (v_cvt_pk_bf16_f32)
typedef __bf16 pd_bf16x2 __attribute__((ext_vector_type(2)));
typedef float pd_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack2bf(float lo, float hi)
{
    pd_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, pd_bf16x2));
}
__device__ __forceinline__ bf16_t f2bf(float f)
{
    bf16_t r;
    r.x = (uint16_t)(pack2bf(f, 0.f) & 0xffffu);
    return r;
}

template <typename T>
struct Elem;
template <>
struct Elem<float> {
    static __device__ __forceinline__ float ld(const float *p) { return *p; }
    static __device__ __forceinline__ void st(float *p, float v) { *p = v; }
};
template <>
struct Elem<bf16_t> {
    static __device__ __forceinline__ float ld(const bf16_t *p) { return bf2f(*p); }
    static __device__ __forceinline__ void st(bf16_t *p, float v) { *p = f2bf(v); }
};

// Blocked bf16 / head_dim-128 cache layout used by the matrix-core decode attention.  Offsets are
// in elements inside one (slot, kv head) plane of max_len_pad * 128 elements (max_len_pad is a
// multiple of 64).
//   keys:   blocks of 16 positions; inside a block [channel/32][position%16][channel%32], so the
//           16 rows x 64 bytes that one MFMA A-operand load touches are 1 KB contiguous.
//   values: blocks of 32 positions stored transposed, [channel][sigma(position%32)], where
//           sigma(16a + 4q + j) = 8q + 4a + j is the key order in which the exp'd scores leave the
//           S^T accumulators; again every operand load is 1 KB contiguous.
__host__ __device__ __forceinline__ size_t kblk_off(int pos, int c)
{
    return (size_t)(pos >> 4) * 2048 + (size_t)(c >> 5) * 512 + (pos & 15) * 32 + (c & 31);
}
__host__ __device__ __forceinline__ size_t vblk_off(int pos, int d)
{
    const int pp = pos & 31;
    return (size_t)(pos >> 5) * 4096 + (size_t)d * 32 + 8 * ((pp >> 2) & 3) + 4 * (pp >> 4) + (pp & 3);
}

// The same cache held as 8-bit E4M3 codes (one byte per element, byte offsets inside a plane of
// max_len_pad * 128 bytes).  A 16-byte-per-lane load still fills whole operand registers:
//   keys:   blocks of 16 positions (2 KB) = two 1 KB halves t; lane 16*kg + position%16 of half t
//           holds channels 64t + 8kg .. +7 (bytes 0-7) and 64t + 32 + 8kg .. +7 (bytes 8-15), i.e.
//           its A operands of k-steps 2t and 2t+1.
//   values: blocks of 64 positions (8 KB) = eight 1 KB groups of 16 channels; lane 16*kg + channel%16
//           holds the 8 keys sigma^-1(8kg .. 8kg+7) of the first 32 positions (bytes 0-7) and of the
//           second 32 positions (bytes 8-15).
__host__ __device__ __forceinline__ size_t kblk8_off(int pos, int c)
{
    return (size_t)(pos >> 4) * 2048 + (size_t)(c >> 6) * 1024 + ((c >> 3) & 3) * 256 + (pos & 15) * 16 +
           ((c >> 5) & 1) * 8 + (c & 7);
}
__host__ __device__ __forceinline__ size_t vblk8_off(int pos, int d)
{
    const int pp = pos & 31;
    const int sg = 8 * ((pp >> 2) & 3) + 4 * (pp >> 4) + (pp & 3);
    return (size_t)(pos >> 6) * 8192 + (size_t)(d >> 4) * 1024 + (sg >> 3) * 256 + (d & 15) * 16 +
           ((pos >> 5) & 1) * 8 + (sg & 7);
}

// OCP FP8 E4M3 ("fn": no infinities, NaN = 0x7F / 0xFF, largest finite 448): nearest code of q,
// ties to the even mantissa, saturating.  Works on the bit pattern of the double: the 53-bit
// significand is cut at the quantum 2^(max(exponent, -6) - 3) and rounded on the discarded bits;
// a carry out of the mantissa lands in the exponent field by plain addition.
__device__ __forceinline__ uint32_t e4m3_encode(double q)
{
    uint64_t b = (uint64_t)__double_as_longlong(q);
    const uint32_t sign = (uint32_t)(b >> 56) & 0x80u;
    b &= 0x7FFFFFFFFFFFFFFFull;
    if (b > 0x7FF0000000000000ull) return sign | 0x7Fu;        // NaN
    if (b >= 0x407C000000000000ull) return sign | 0x7Eu;        // |q| >= 448
    const int ex = (int)(b >> 52) - 1023;
    if (ex < -10) return sign;                                  // below half the smallest subnormal
    const uint64_t mant = (b & 0x000FFFFFFFFFFFFFull) | 0x0010000000000000ull;
    const int E = ex < -6 ? -6 : ex;
    const int sh = 49 + (E - ex);                               // 49 .. 53
    uint32_t n = (uint32_t)(mant >> sh);
    const uint64_t rem = mant & ((1ull << sh) - 1), half = 1ull << (sh - 1);
    if (rem > half || (rem == half && (n & 1u))) ++n;
    return sign | (uint32_t)(((E + 7) << 3) + (int)n - 8);
}
// value of one code (hardware conversion; exact for every code)
__device__ __forceinline__ float e4m3_decode(uint32_t code)
{
    return __builtin_amdgcn_cvt_pk_f32_fp8((int)code, false)[0];
}

// Packed weight layout of the matrix-core kernels.  A [N, K] matrix is cut into blocks of 16 rows x
// 32 k (1 KB); inside a block the order is [k/8][row][k%8], i.e. exactly the register image of one
// v_mfma_f32_16x16x32_bf16 A operand (lane = 16*(k/8) + row holds 8 consecutive k), so a wave reads
// a block with one fully contiguous 16-byte-per-lane load.  Blocks are ordered [N/16][K/32].  For
// the SwiGLU pack the rows are first interleaved in 32-row blocks: gate[j..j+31], up[j..j+31], ...
__host__ __device__ __forceinline__ size_t wpack_off(int n, int k, int K)
{
    return ((size_t)(n >> 4) * (K >> 5) + (k >> 5)) * 512 + ((k >> 3) & 3) * 128 + (n & 15) * 8 + (k & 7);
}

// 8-bit packed weights: blocks of 16 rows x 64 k (1 KB), ordered [N/16][K/64]; lane 16*(k/8 % 4) + row
// of a block owns 16 bytes: k = 64b + 8kg .. +7 (bytes 0-7) and 64b + 32 + 8kg .. +7 (bytes 8-15), its
// A operands of two consecutive 32-wide k-steps.  Byte offset of element (n, k):
__host__ __device__ __forceinline__ size_t w8pack_off(int n, int k, int K)
{
    return ((size_t)(n >> 4) * (K >> 6) + (k >> 6)) * 1024 + ((k >> 3) & 3) * 256 + (n & 15) * 16 +
           ((k >> 5) & 1) * 8 + (k & 7);
}

// RMSNorm of one bf16 row of 8 * d8 elements by one workgroup of 256 threads: 16-byte loads and stores,
// statistics in fp32.  red: 4 floats of LDS.
__device__ __forceinline__ void rmsnorm_bf16_row(const uint4 *__restrict__ xr, const uint4 *__restrict__ g,
                                                 uint4 *__restrict__ yr, int d8, float d_inv, float eps, float *red)
{
    float ss = 0.f;
    for (int i = threadIdx.x; i < d8; i += 256) {
        uint4 v = xr[i];
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float a = bfbits2f(w[j] & 0xffffu), b = bfbits2f(w[j] >> 16);
            ss += a * a + b * b;
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    float inv = rsqrtf((red[0] + red[1] + red[2] + red[3]) * d_inv + eps);
    for (int i = threadIdx.x; i < d8; i += 256) {
        uint4 v = xr[i], gg = g[i];
        uint32_t w[4] = {v.x, v.y, v.z, v.w}, gw[4] = {gg.x, gg.y, gg.z, gg.w}, o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float a = bfbits2f(w[j] & 0xffffu) * inv * bfbits2f(gw[j] & 0xffffu);
            float b = bfbits2f(w[j] >> 16) * inv * bfbits2f(gw[j] >> 16);
            o[j] = pack2bf(a, b);
        }
        yr[i] = make_uint4(o[0], o[1], o[2], o[3]);
    }
}

constexpr int kMetaChunk = 255;  // ints carried by value per meta-kernel launch (+1 for cu_seqlens)
struct IntChunk {
    int32_t v[256];
};
struct IntDst4 {
    int32_t *dst[4];
    int32_t start[5];   // array k is v[start[k] .. start[k + 1])
};

struct RopeArgs;

enum Epilogue { EPI_NONE = 0, EPI_RESIDUAL = 1, EPI_SWIGLU = 2, EPI_PARTIAL = 3 /* internal: fp32 split-K partials */ };

// C[M,N] = epilogue(A[M,K] * B[N,K]^T).  All matrices row-major with leading dimensions in
// elements.  a_gather (optional): logical row i of A is physical row a_gather[i].  Groups
// (optional): rows [group_offsets[g], group_offsets[g+1]) multiply B + g*b_group_stride.
struct GemmArgs {
    const void *A;
    const void *B;        // weights; EPI_SWIGLU: gate rows (plain) or the gate/up pack (packed)
    const void *B1;       // EPI_SWIGLU with plain layout: up rows; else unused
    void *C;
    const void *R;        // EPI_RESIDUAL: residual [M,N]
    const int32_t *a_gather;
    const int32_t *group_offsets;  // device [n_groups+1] or nullptr
    int64_t b_group_stride;        // elements
    int32_t n_groups;
    int32_t M, N, K;               // N = output columns (for SWIGLU: F)
    int32_t lda, ldb, ldc, ldr;
    int32_t epilogue;
    int32_t packed;                // B is in the MFMA block layout below (matrix-core kernels only)
    float *splitk_ws;              // optional scratch for split-K partials (decode-sized M)
    size_t splitk_ws_elems;
    // 8-bit twin of the packed weights (skinny and wide decode kernels only; null = none): E4M3 codes in the layout
    // of w8pack_off, and one power-of-two scale per packed weight row; weight = scale * value(code).
    // Groups are b_group_stride codes and (2N for SwiGLU, else N) scales apart.
    const void *B8;
    const float *b_scale;
    // 8-bit activations (tiled kernel, F8 form): one scale per row of A; A and B then hold E4M3 codes
    const float *a_scale;
    // Optional work for the launch that adds split-K partials of an EPI_RESIDUAL product (N a multiple of
    // 8, at most 8192): the RMSNorm of the rows it has just formed, y = rmsnorm(C; fuse_g, fuse_eps) into
    // fuse_y [M, N] (leading dimension N), and, if fuse_append is set, the cache append of a decode
    // step (see launch_rmsnorm_append).  A launcher that does so sets *fuse_done = 1; otherwise (no split,
    // another kernel) the caller runs the norm itself.
    const void *fuse_g;
    void *fuse_y;
    float fuse_eps;
    const RopeArgs *fuse_append;
    int *fuse_done;
};

// ---- launchers (each returns hipGetLastError() after the launch) ------------------------------
hipError_t launch_rmsnorm(int dtype, const void *x, const void *g, void *y, int T, int d, float eps,
                          hipStream_t s);
hipError_t launch_gemm_generic(int dtype, const GemmArgs &a, hipStream_t s);
bool gemm_mfma_supported(const GemmArgs &a);
hipError_t launch_gemm_mfma(const GemmArgs &a, hipStream_t s);   // bf16 only
bool gemm_mfma_f8_supported(const GemmArgs &a);                   // E4M3 x E4M3, dense
hipError_t launch_gemm_mfma_f8(const GemmArgs &a, hipStream_t s);
// per row of x [T, K] (bf16, row stride ldx): scale = smallest power of two with max|x| / scale <= 448
// (1 for a zero row), codes = E4M3(x / scale), round to nearest even, saturating; codes [T, K] bytes
hipError_t launch_quant_rows_e4m3(const void *x, int ldx, int T, int K, void *codes, float *scales, hipStream_t s);
// the two in one pass for bf16 rows of up to 8192 elements (the normalised bf16 row is not stored)
bool rmsnorm_quant_supported(int d);
hipError_t launch_rmsnorm_quant_e4m3(const void *x, const void *g, int T, int d, float eps, void *codes,
                                     float *scales, hipStream_t s);
// codes in the layout of w8pack_off -> the bf16 block pack of the same matrix seen as [n_rows, K / 2] code pairs
hipError_t launch_repack_w8_tiles(const void *src8, void *dst, int n_rows, int K, hipStream_t s);
hipError_t launch_pack_rows_e4m3_tiles(const void *src, void *dst, int n_rows, int K, hipStream_t s);   // from row-major codes
// sums the fp32 partials [splits][M][N or 2N packed] in a.splitk_ws in a fixed order and applies a.epilogue
hipError_t launch_splitk_reduce(const GemmArgs &a, int splits, hipStream_t s);
bool wgemm_mfma_supported(const GemmArgs &a);                    // 16 < M <= 128 (8-bit weights) or 32 (bf16)
hipError_t launch_wgemm_mfma(const GemmArgs &a, hipStream_t s);
bool gemv_mfma_supported(const GemmArgs &a);                      // bf16, M <= 16
hipError_t launch_gemv_mfma(const GemmArgs &a, hipStream_t s);
// per token row: its sequence, its position inside it and (if d_slots) its cache slot
// d_prefix (optional, [n_seqs]): positions start at d_prefix[seq] instead of 0
hipError_t launch_token_meta(const int32_t *d_cu, const int32_t *d_slots, const int32_t *d_prefix,
                             int n_seqs, int T, int32_t *tok_seq, int32_t *tok_pos, int32_t *tok_slot,
                             hipStream_t s);
hipError_t launch_write_ints(int32_t *dst, const int32_t *host_src, int n, hipStream_t s);
// Up to four arrays (n[k] may be 0) in one launch when they hold 256 ints or fewer together.
hipError_t launch_write_ints4(int32_t *const dst[4], const int32_t *const host_src[4], const int n[4],
                              hipStream_t s);
// The same four arrays of a prefill call (0 = sequence starts [n_seqs + 1], 1 = padded starts, 2 = slots
// or none, 3 = prefixes or none) together with the per-token sequence index / position / slot.
hipError_t launch_prefill_meta(int32_t *const dst[4], const int32_t *const host_src[4], const int n[4],
                               int n_seqs, int T, int32_t *tok_seq, int32_t *tok_pos, int32_t *tok_slot,
                               hipStream_t s);
// dst[idx[i]] = val[i] for i < n (host arrays, carried by value in the kernel arguments)
hipError_t launch_scatter_ints(int32_t *dst, const int32_t *host_idx, const int32_t *host_val, int n,
                               hipStream_t s);
// decode meta: for b in [0,B): pos[b] = len[slot[b]]; len[slot[b]] += 1
hipError_t launch_decode_meta(const int32_t *d_slots, int B, int32_t *d_len, int32_t *d_pos,
                              hipStream_t s);
// prefill: len[slot[s]] = cu[s+1]-cu[s]  (add != 0: += instead of =)
hipError_t launch_prefill_set_len(const int32_t *d_slots, const int32_t *d_cu, int n_seqs,
                                  int32_t *d_len, int add, hipStream_t s);

struct RopeArgs {
    void *qkv;               // [T, (Hq+2Hkv)*hd]; q and k rotated in place
    int32_t ld;              // row stride of qkv (elements)
    int32_t T, Hq, Hkv, hd;
    const int32_t *tok_pos;  // [T] position of each row inside its sequence
    const int32_t *tok_slot; // [T] cache slot of each row, or nullptr = no cache write
    void *k_cache, *v_cache; // [slots][Hkv][max_len][hd], or the blocked layout above
    int32_t max_len;         // plane length in positions (padded length for the blocked layout)
    int32_t blocked;
    int32_t fp8;             // blocked cache of E4M3 codes: element stored = code of x / scale
    double k_scale, v_scale;
    const double *inv_freq;  // [hd/2] rope_base^(-2i/hd)
    const float2 *table;     // optional [table_len][hd/2] (cos, sin) of pos * inv_freq, made in double
    int32_t table_len;
};
// The cache append of decode row t (bf16 layer, head_dim up to 256, blocked bf16 or 8-bit cache) by one
// workgroup (all of its threads take part): the key of every kv head rotated at tok_pos[t] in fp32 and stored, the value
// stored; the qkv buffer is only read.  cs, sn: 128 floats of LDS each.
__device__ __forceinline__ void append_token_body(const RopeArgs &a, int t, float *cs, float *sn)
{
    const int half = a.hd >> 1, nt = blockDim.x;
    const int pos = a.tok_pos[t], slot = a.tok_slot[t];
    for (int i = threadIdx.x; i < half; i += nt) {
        if (pos < a.table_len) {
            float2 f = a.table[(size_t)pos * half + i];
            cs[i] = f.x;
            sn[i] = f.y;
        } else {
            double sv, cv;
            sincos((double)pos * a.inv_freq[i], &sv, &cv);
            cs[i] = (float)cv;
            sn[i] = (float)sv;
        }
    }
    __syncthreads();
    const uint16_t *row = (const uint16_t *)a.qkv + (size_t)t * a.ld;
    const size_t plane_elems = (size_t)a.max_len * a.hd;
    for (int idx = threadIdx.x; idx < a.Hkv * half; idx += nt) {
        const int gk = idx / half, i = idx - gk * half;
        const uint16_t *kv = row + (size_t)(a.Hq + gk) * a.hd;
        const float x0 = bfbits2f(kv[i]), x1 = bfbits2f(kv[i + half]);
        const float y0 = x0 * cs[i] - x1 * sn[i], y1 = x1 * cs[i] + x0 * sn[i];
        const size_t plane = ((size_t)slot * a.Hkv + gk) * plane_elems;
        if (a.fp8) {
            uint8_t *p8 = (uint8_t *)a.k_cache + plane;
            p8[kblk8_off(pos, i)] = (uint8_t)e4m3_encode((double)y0 / a.k_scale);
            p8[kblk8_off(pos, i + half)] = (uint8_t)e4m3_encode((double)y1 / a.k_scale);
        } else {
            uint16_t *pk = (uint16_t *)a.k_cache + plane;
            pk[kblk_off(pos, i)] = f2bf(y0).x;
            pk[kblk_off(pos, i + half)] = f2bf(y1).x;
        }
    }
    const uint16_t *vsrc = row + (size_t)(a.Hq + a.Hkv) * a.hd;
    for (int idx = threadIdx.x; idx < a.Hkv * a.hd; idx += nt) {
        const int gv = idx / a.hd, i = idx - gv * a.hd;
        const size_t plane = ((size_t)slot * a.Hkv + gv) * plane_elems;
        if (a.fp8)
            ((uint8_t *)a.v_cache)[plane + vblk8_off(pos, i)] = (uint8_t)e4m3_encode((double)bfbits2f(vsrc[idx]) / a.v_scale);
        else
            ((uint16_t *)a.v_cache)[plane + vblk_off(pos, i)] = vsrc[idx];
    }
}

hipError_t launch_rope_table(float2 *table, int table_len, int half, const double *inv_freq, hipStream_t s);
hipError_t launch_rope_kv(int dtype, const RopeArgs &a, hipStream_t s);
// RMSNorm of n_rows bf16 rows (d a multiple of 8) and, in the same launch, the cache append of a decode
// step: for each of the a.T rows of a.qkv the key is rotated (qkv itself is left unrotated) and stored
// with the value at a.tok_pos / a.tok_slot of the blocked bf16 or 8-bit cache.  The two halves are
// independent; together they cost one launch.
hipError_t launch_rmsnorm_append(const RopeArgs &a, const void *x, const void *g, void *y, int n_rows, int d,
                                 float eps, hipStream_t s);

struct AttnArgs {
    const void *qkv;         // rotated q (and, for prefill, k and v) rows
    int32_t ld;
    void *o;                 // [T, Hq*hd]
    int32_t T, Hq, Hkv, hd;
    float scale;
    // prefill: keys of row t are rows (t - tok_pos[t]) .. t of qkv
    const int32_t *tok_pos;
    // decode: keys of row b are cache positions 0 .. tok_pos[b] of slot tok_slot[b]
    const int32_t *tok_slot;
    const void *k_cache, *v_cache;
    int32_t max_len;
    int32_t decode;
    // prefill tiling helpers
    const int32_t *d_cu;     // [n_seqs+1]
    int32_t n_seqs, max_seq_len;
    // chunked prefill on the matrix-core kernel (all null / 0 for an ordinary prefill): the keys of
    // sequence s are rows k_cu[s] .. k_cu[s] + prefix[s] + L_s - 1 of the plain key buffer kx
    // ([rows][Hkv*128], row stride kx_ld), and query i of the sequence sees keys 0 .. prefix[s] + i
    const void *kx;
    int32_t kx_ld;
    const int32_t *k_cu;     // [n_seqs+1]
    const int32_t *prefix;   // [n_seqs]
    // chunked prefill source is the 8-bit E4M3 blocked cache: gathered values are code * scale
    int32_t kv_fp8;
    float k_scale, v_scale;
};
hipError_t launch_attn_generic(int dtype, const AttnArgs &a, hipStream_t s);
bool attn_prefill_mfma_supported(const AttnArgs &a);
// bf16, hd = 128.  vt: scratch for V transposed, [Hkv][128][vt_ld] with vt_ld = padded token count
// (each sequence start rounded up to a multiple of 64); pad_cu: device [n_seqs+1] padded starts.
hipError_t launch_attn_prefill_mfma(const AttnArgs &a, uint16_t *vt, int vt_ld, const int32_t *pad_cu,
                                    hipStream_t s);
// Chunked prefill over a blocked cache: copies the keys (as plain rows kx[pad_cu[s] + pos][Hkv*128])
// and the values (transposed, vt[g][d][pad_cu[s] + pos], zero past the end) of positions
// 0 .. prefix[s] + L_s - 1 of every sequence's slot out of the cache, then runs the prefill kernel
// with the prefix offsets.  pad_cu: padded key-row starts (multiples of 64) of the sequences.
// n_split >= 2 divides every query block's keys over that many workgroups (fp32 partial results in
// part, attn_chunk_split_bytes(a, n_split) bytes, merged by a second kernel); attn_chunk_splits
// picks the count for the call's grid and its longest key range.
hipError_t launch_attn_chunk_mfma(const AttnArgs &a, const int32_t *d_slots, uint16_t *kx, uint16_t *vt,
                                  int vt_ld, const int32_t *pad_cu, int n_split, float *part, hipStream_t s);
int attn_chunk_splits(const AttnArgs &a, int max_keys);
size_t attn_chunk_split_bytes(const AttnArgs &a, int n_split);

hipError_t launch_stream_copy(void *dst, const void *src, size_t n_vec16, hipStream_t s);
hipError_t launch_mfma_probe(float *sink, const void *a_vals, const void *b_vals, int n_workgroups, int iters, hipStream_t s);
// out[t, :] = table[ids[t], :] (rows of row_bytes bytes, a multiple of 4); ids outside 0 .. n_rows-1 give zeros
hipError_t launch_embed_rows(void *out, const void *table, const int32_t *ids, int T, int n_rows,
                             size_t row_bytes, hipStream_t s);
hipError_t launch_kv_copy(int dtype, void *cache_k, void *cache_v, const void *k, const void *v,
                          int slot, int Hkv, int len, int hd, int max_len, int blocked, int to_cache,
                          hipStream_t s);
// the same for the 8-bit E4M3 blocked cache (bf16 tensors outside, head_dim 128)
hipError_t launch_kv_copy_fp8(void *cache_k, void *cache_v, const void *k, const void *v, int slot, int Hkv,
                              int len, int max_len_pad, double k_scale, double v_scale, int to_cache,
                              hipStream_t s);

// ---- matrix-core decode attention over the blocked cache (bf16, head_dim 128, group <= 16) ---------
struct DecodeAttnArgs {
    const void *qkv;           // [B, ld] rotated q rows
    int32_t ld;
    void *o;                   // [B, Hq*128] bf16
    int32_t B, Hq, Hkv;
    float scale;
    const int32_t *slots;      // [B]
    const int32_t *pos;        // [B] position of the new token = keys - 1
    const int32_t *chunk_cu;   // [B+1] prefix sum of key chunks per sequence
    const int32_t *chunk_seq;  // [total_chunks] sequence of every chunk, or nullptr (then found by bisection of chunk_cu)
    int32_t chunk_keys;        // keys per chunk (multiple of 64)
    int32_t total_chunks;
    const void *k_cache, *v_cache;
    int32_t max_len_pad;
    float *part_o;             // [total_chunks][Hq][128]
    float *part_ml;            // [total_chunks][Hq][2]
    // Multi-token form (all null for the one-token step): "sequence" b is a unit of u_ntok[b] <= 16/group
    // consecutive new tokens of one cache slot; token i of the unit is row u_row0[b] + i of qkv / o,
    // sits at position pos[b] + i and sees keys 0 .. pos[b] + i.  The 16 MFMA columns are
    // (token, head of the group) pairs; partials are then [total_chunks][Hkv][16][128] / [..][2].
    const int32_t *u_row0;
    const int32_t *u_ntok;
    // E4M3 cache (the 8-bit blocked layout): value = code * scale
    int32_t fp8;
    float k_scale, v_scale;
    // Fused rotary embedding (one-token step only; rope_table null = off): the q and k rows of qkv arrive
    // unrotated, every worker rotates its query rows at position pos[b], and the worker that owns the last
    // chunk of a (sequence, kv head) adds the new token (position pos[b], not yet in the cache: the chunks
    // cover positions below it) from registers, its key rotated and rounded as the cache will hold it
    // (bf16, or the value of the E4M3 code of x / scale).  The caller appends it to the cache afterwards.
    const float2 *rope_table;  // [rope_table_len][64] (cos, sin) of pos * inv_freq[i]
    int32_t rope_table_len;
    const double *inv_freq;    // [64], for positions beyond the table
    double k_scale_d, v_scale_d;
};
hipError_t launch_decode_attn_mfma(const DecodeAttnArgs &a, hipStream_t s);
// pos[b] = len[slot[b]]; len[slot[b]] += 1; chunk_cu = prefix sum of ceil((pos+1)/chunk_keys);
// chunk_seq[c] = b for the chunks c of sequence b
hipError_t launch_decode_meta_chunks(const int32_t *d_slots, int B, int32_t *d_len, int32_t *d_pos,
                                     int32_t *chunk_cu, int32_t *chunk_seq, int chunk_keys, hipStream_t s);
// the same for B <= 256 with the slots taken from the host array (and stored to d_slots): one launch
hipError_t launch_decode_meta_chunks_upload(const int32_t *host_slots, int32_t *d_slots, int B, int32_t *d_len,
                                            int32_t *d_pos, int32_t *chunk_cu, int32_t *chunk_seq, int chunk_keys,
                                            hipStream_t s);
// that and the RMSNorm of the step's B bf16 rows (d a multiple of 8) in one launch: blocks 0 .. B-1
// normalise a row each, block B does the bookkeeping
hipError_t launch_decode_meta_norm(const int32_t *host_slots, int32_t *d_slots, int B, int32_t *d_len, int32_t *d_pos,
                                   int32_t *chunk_cu, int32_t *chunk_seq, int chunk_keys, const void *x, const void *g,
                                   void *y, int d, float eps, hipStream_t s);

// ---- MoE -----------------------------------------------------------------------------------------
struct MoeRouteArgs {
    const float *logits;   // [T, E]
    int32_t T, E, top_k;
    int32_t *expert_idx;   // [T, top_k]
    float *expert_w;       // [T, top_k]
    int32_t *sorted_token; // [T*top_k] token of each (token, expert) pair, ordered by expert
    int32_t *pair_pos;     // [T, top_k] position of each pair in the sorted order
    int32_t *offsets;      // [E+1]
    int32_t *block_hist;   // scratch [ceil(T*top_k / 256)][E], or nullptr (then one block sorts alone)
};
hipError_t launch_moe_route(const MoeRouteArgs &a, hipStream_t s);
hipError_t launch_router_logits(int dtype, const void *y, const void *w_router, float *logits,
                                int T, int d, int E, hipStream_t s);
hipError_t launch_moe_combine(int dtype, const void *h, const void *expert_out,
                              const int32_t *pair_pos, const float *expert_w, void *out, int T,
                              int d, int top_k, hipStream_t s);

void set_error(const char *fmt, ...);

// "Done once per device" flag for per-kernel attributes (hipFuncSetAttribute applies to the current
// device only).  Threads that race on the first call of a device both do the work, which is harmless.
struct OncePerDevice {
    std::atomic<uint64_t> done{0};
    // true if the caller has to do the work for the current device (devices beyond 63: every time)
    bool need(int *dev_out)
    {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess) dev = 64;
        *dev_out = dev;
        return dev >= 64 || !((done.load(std::memory_order_acquire) >> dev) & 1u);
    }
    void mark(int dev)
    {
        if (dev < 64) done.fetch_or(1ull << dev, std::memory_order_release);
    }
};

}  // namespace pd
