// Shape-generic kernels (fp32 or bf16 storage, fp32 arithmetic): RMSNorm, a tiled FMA GEMM with
// fused epilogues, rotary embedding + KV-cache write, wave-per-row attention, and the small
// metadata kernels.  These carry the fp32 parity configuration and any bf16 shape the MFMA
// kernels do not cover.
#include "pd_internal.h"

namespace pd {

// ---------------------------------------------------------------------------------------------
// RMSNorm: y = x * rsqrt(mean(x^2) + eps) * g.  One 256-thread block per row.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const T *__restrict__ x,
                                                      const T *__restrict__ g, T *__restrict__ y,
                                                      int d, float eps)
{
    __shared__ float red[4];
    const T *xr = x + (size_t)blockIdx.x * d;
    T *yr = y + (size_t)blockIdx.x * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += 256) {
        float v = Elem<T>::ld(xr + i);
        ss += v * v;
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = red[0] + red[1] + red[2] + red[3];
    float inv = rsqrtf(tot / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += 256)
        Elem<T>::st(yr + i, Elem<T>::ld(xr + i) * inv * Elem<T>::ld(g + i));
}

// bf16 rows with d % 8 == 0: 16-byte loads and stores (the row routine is rmsnorm_bf16_row of pd_internal.h).
__global__ __launch_bounds__(256) void rmsnorm_bf16_vec_kernel(const uint4 *__restrict__ x,
                                                               const uint4 *__restrict__ g,
                                                               uint4 *__restrict__ y, int d8,
                                                               float d_inv, float eps)
{
    __shared__ float red[4];
    rmsnorm_bf16_row(x + (size_t)blockIdx.x * d8, g, y + (size_t)blockIdx.x * d8, d8, d_inv, eps, red);
}

hipError_t launch_rmsnorm(int dtype, const void *x, const void *g, void *y, int T, int d, float eps,
                          hipStream_t s)
{
    if (T <= 0) return hipSuccess;
    if (dtype == PD_F32) {
        rmsnorm_kernel<float><<<T, 256, 0, s>>>((const float *)x, (const float *)g, (float *)y, d, eps);
    } else if (d % 8 == 0) {
        rmsnorm_bf16_vec_kernel<<<T, 256, 0, s>>>((const uint4 *)x, (const uint4 *)g, (uint4 *)y,
                                                  d / 8, 1.0f / (float)d, eps);
    } else {
        rmsnorm_kernel<bf16_t><<<T, 256, 0, s>>>((const bf16_t *)x, (const bf16_t *)g, (bf16_t *)y, d, eps);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Generic GEMM: 64x64 tile, K step 16, 256 threads, 4x4 outputs per thread, fp32 accumulate.
// ---------------------------------------------------------------------------------------------
constexpr int GT = 64, GK = 16;

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + expf(-z)); }

template <typename T, int EPI>
__global__ __launch_bounds__(256) void gemm_generic_kernel(GemmArgs a)
{
    __shared__ float As[GK][GT + 1];
    __shared__ float Bs[GK][GT + 1];
    __shared__ float B1s[EPI == EPI_SWIGLU ? GK : 1][GT + 1];

    // locate this block's group and row range
    int row0, row_end, group = 0;
    {
        int vt = blockIdx.y;
        if (a.group_offsets) {
            int acc = 0;
            row0 = -1;
            row_end = 0;
            for (int g = 0; g < a.n_groups; ++g) {
                int lo = a.group_offsets[g], hi = a.group_offsets[g + 1];
                int nt = (hi - lo + GT - 1) / GT;
                if (vt < acc + nt) {
                    group = g;
                    row0 = lo + (vt - acc) * GT;
                    row_end = hi;
                    break;
                }
                acc += nt;
            }
            if (row0 < 0) return;
        } else {
            row0 = vt * GT;
            row_end = a.M;
            if (row0 >= a.M) return;
        }
    }
    const int col0 = blockIdx.x * GT;
    const T *A = (const T *)a.A;
    const T *B = (const T *)a.B + (size_t)group * a.b_group_stride;
    const T *B1 = EPI == EPI_SWIGLU ? (const T *)a.B1 + (size_t)group * a.b_group_stride : nullptr;

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    float acc[4][4] = {}, acc1[4][4] = {};

    // loader mapping: 64 rows x 16 k = 1024 elements, 4 per thread
    const int lr = tid >> 2;          // 0..63 row in tile
    const int lk = (tid & 3) * 4;     // 0,4,8,12
    int arow = row0 + lr;
    const bool arow_ok = arow < row_end;
    size_t a_off = 0;
    if (arow_ok) a_off = (size_t)(a.a_gather ? a.a_gather[arow] : arow) * a.lda;
    const int bcol = col0 + lr;
    const bool bcol_ok = bcol < a.N;
    size_t b_off = 0, b1_off = 0;
    if (bcol_ok) {
        b_off = (size_t)bcol * a.ldb;
        b1_off = b_off;
    }

    for (int k0 = 0; k0 < a.K; k0 += GK) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int k = k0 + lk + j;
            bool kok = k < a.K;
            As[lk + j][lr] = (arow_ok && kok) ? Elem<T>::ld(A + a_off + k) : 0.f;
            Bs[lk + j][lr] = (bcol_ok && kok) ? Elem<T>::ld(B + b_off + k) : 0.f;
            if (EPI == EPI_SWIGLU) B1s[lk + j][lr] = (bcol_ok && kok) ? Elem<T>::ld(B1 + b1_off + k) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < GK; ++k) {
            float av[4], bv[4], b1v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                av[i] = As[k][ty * 4 + i];
                bv[i] = Bs[k][tx * 4 + i];
                if (EPI == EPI_SWIGLU) b1v[i] = B1s[k][tx * 4 + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
                    if (EPI == EPI_SWIGLU) acc1[i][j] = fmaf(av[i], b1v[j], acc1[i][j]);
                }
        }
        __syncthreads();
    }

    T *C = (T *)a.C;
    const T *R = (const T *)a.R;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int r = row0 + ty * 4 + i;
        if (r >= row_end) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int c = col0 + tx * 4 + j;
            if (c >= a.N) continue;
            float v = acc[i][j];
            if (EPI == EPI_RESIDUAL) v += Elem<T>::ld(R + (size_t)r * a.ldr + c);
            if (EPI == EPI_SWIGLU) v = silu_f(v) * acc1[i][j];
            Elem<T>::st(C + (size_t)r * a.ldc + c, v);
        }
    }
}

template <typename T>
static hipError_t launch_gemm_generic_t(const GemmArgs &a, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    int mt = (a.M + GT - 1) / GT + (a.group_offsets ? a.n_groups : 0);
    dim3 grid((a.N + GT - 1) / GT, mt);
    switch (a.epilogue) {
    case EPI_NONE: gemm_generic_kernel<T, EPI_NONE><<<grid, 256, 0, s>>>(a); break;
    case EPI_RESIDUAL: gemm_generic_kernel<T, EPI_RESIDUAL><<<grid, 256, 0, s>>>(a); break;
    default: gemm_generic_kernel<T, EPI_SWIGLU><<<grid, 256, 0, s>>>(a); break;
    }
    return hipGetLastError();
}

hipError_t launch_gemm_generic(int dtype, const GemmArgs &a, hipStream_t s)
{
    return dtype == PD_F32 ? launch_gemm_generic_t<float>(a, s) : launch_gemm_generic_t<bf16_t>(a, s);
}

// ---------------------------------------------------------------------------------------------
// Metadata kernels.
// ---------------------------------------------------------------------------------------------
__global__ void write_ints_kernel(int32_t *dst, IntChunk c, int n)
{
    int i = threadIdx.x;
    if (i < n) dst[i] = c.v[i];
}

hipError_t launch_write_ints(int32_t *dst, const int32_t *host_src, int n, hipStream_t s)
{
    for (int off = 0; off < n; off += 256) {
        IntChunk c;
        int m = n - off < 256 ? n - off : 256;
        for (int i = 0; i < m; ++i) c.v[i] = host_src[off + i];
        write_ints_kernel<<<1, 256, 0, s>>>(dst + off, c, m);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Up to four short arrays in one launch: array k takes c.v[start[k] .. start[k + 1]).
__global__ void write_ints4_kernel(IntDst4 d, IntChunk c)
{
    const int i = threadIdx.x;
    if (i >= d.start[4]) return;
    const int k = (i >= d.start[1]) + (i >= d.start[2]) + (i >= d.start[3]);
    d.dst[k][i - d.start[k]] = c.v[i];
}

hipError_t launch_write_ints4(int32_t *const dst[4], const int32_t *const host_src[4], const int n[4],
                              hipStream_t s)
{
    const int total = n[0] + n[1] + n[2] + n[3];
    if (total > 256) {                             // too long for one launch: one array at a time
        for (int k = 0; k < 4; ++k) {
            if (n[k] == 0) continue;
            hipError_t e = launch_write_ints(dst[k], host_src[k], n[k], s);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    if (total == 0) return hipSuccess;
    IntDst4 d;
    IntChunk c;
    int at = 0;
    for (int k = 0; k < 4; ++k) {
        d.dst[k] = dst[k];
        d.start[k] = at;
        for (int i = 0; i < n[k]; ++i) c.v[at + i] = host_src[k][i];
        at += n[k];
    }
    d.start[4] = at;
    write_ints4_kernel<<<1, 256, 0, s>>>(d, c);
    return hipGetLastError();
}

__global__ void scatter_ints_kernel(int32_t *dst, IntChunk c, int n)
{
    int i = threadIdx.x;
    if (i < n) dst[c.v[i]] = c.v[128 + i];
}

hipError_t launch_scatter_ints(int32_t *dst, const int32_t *host_idx, const int32_t *host_val, int n,
                               hipStream_t s)
{
    for (int off = 0; off < n; off += 128) {
        IntChunk c;
        int m = n - off < 128 ? n - off : 128;
        for (int i = 0; i < m; ++i) {
            c.v[i] = host_idx[off + i];
            c.v[128 + i] = host_val[off + i];
        }
        scatter_ints_kernel<<<1, 128, 0, s>>>(dst, c, m);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

__global__ void token_meta_kernel(const int32_t *__restrict__ cu, const int32_t *__restrict__ slots,
                                  const int32_t *__restrict__ prefix, int n_seqs, int T,
                                  int32_t *__restrict__ tok_seq,
                                  int32_t *__restrict__ tok_pos, int32_t *__restrict__ tok_slot)
{
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    int lo = 0, hi = n_seqs;  // largest s with cu[s] <= t
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (cu[mid] <= t) lo = mid; else hi = mid;
    }
    tok_seq[t] = lo;
    tok_pos[t] = t - cu[lo] + (prefix ? prefix[lo] : 0);
    if (slots) tok_slot[t] = slots[lo];
}

hipError_t launch_token_meta(const int32_t *d_cu, const int32_t *d_slots, const int32_t *d_prefix,
                             int n_seqs, int T, int32_t *tok_seq, int32_t *tok_pos, int32_t *tok_slot,
                             hipStream_t s)
{
    if (T <= 0) return hipSuccess;
    token_meta_kernel<<<(T + 255) / 256, 256, 0, s>>>(d_cu, d_slots, d_prefix, n_seqs, T, tok_seq,
                                                      tok_pos, tok_slot);
    return hipGetLastError();
}

// The sequence arrays of a prefill call and the per-token metadata in one launch: block 0 stores
// the arrays like write_ints4_kernel (0 = sequence starts, 1 = padded starts, 2 = slots or empty,
// 3 = prefixes or empty), and every thread derives its token's entries from the copy of the arrays in
// the kernel arguments, so nothing waits for those stores.
__global__ void prefill_meta_kernel(IntDst4 d, IntChunk c, int n_seqs, int T, int32_t *__restrict__ tok_seq,
                                    int32_t *__restrict__ tok_pos, int32_t *__restrict__ tok_slot)
{
    if (blockIdx.x == 0) {
        const int i = threadIdx.x;
        if (i < d.start[4]) {
            const int k = (i >= d.start[1]) + (i >= d.start[2]) + (i >= d.start[3]);
            d.dst[k][i - d.start[k]] = c.v[i];
        }
    }
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    int lo = 0, hi = n_seqs;  // largest s with cu[s] <= t; cu = c.v[0 .. n_seqs]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (c.v[mid] <= t) lo = mid; else hi = mid;
    }
    const bool has_slots = d.start[3] > d.start[2], has_prefix = d.start[4] > d.start[3];
    tok_seq[t] = lo;
    tok_pos[t] = t - c.v[lo] + (has_prefix ? c.v[d.start[3] + lo] : 0);
    if (has_slots) tok_slot[t] = c.v[d.start[2] + lo];
}

hipError_t launch_prefill_meta(int32_t *const dst[4], const int32_t *const host_src[4], const int n[4],
                               int n_seqs, int T, int32_t *tok_seq, int32_t *tok_pos, int32_t *tok_slot,
                               hipStream_t s)
{
    const int total = n[0] + n[1] + n[2] + n[3];
    if (total > 256 || T <= 0) {                   // too many sequences for the kernel arguments: separate launches
        hipError_t e = launch_write_ints4(dst, host_src, n, s);
        if (e != hipSuccess) return e;
        return launch_token_meta(dst[0], n[2] ? dst[2] : nullptr, n[3] ? dst[3] : nullptr, n_seqs, T, tok_seq,
                                 tok_pos, tok_slot, s);
    }
    IntDst4 d;
    IntChunk c;
    int at = 0;
    for (int k = 0; k < 4; ++k) {
        d.dst[k] = dst[k];
        d.start[k] = at;
        for (int i = 0; i < n[k]; ++i) c.v[at + i] = host_src[k][i];
        at += n[k];
    }
    d.start[4] = at;
    prefill_meta_kernel<<<(T + 255) / 256, 256, 0, s>>>(d, c, n_seqs, T, tok_seq, tok_pos, tok_slot);
    return hipGetLastError();
}

__global__ void decode_meta_kernel(const int32_t *__restrict__ slots, int B, int32_t *len,
                                   int32_t *pos)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int s = slots[b];
    int p = len[s];
    pos[b] = p;
    len[s] = p + 1;  // slots are distinct
}

hipError_t launch_decode_meta(const int32_t *d_slots, int B, int32_t *d_len, int32_t *d_pos,
                              hipStream_t s)
{
    decode_meta_kernel<<<(B + 255) / 256, 256, 0, s>>>(d_slots, B, d_len, d_pos);
    return hipGetLastError();
}

__global__ void prefill_set_len_kernel(const int32_t *__restrict__ slots,
                                       const int32_t *__restrict__ cu, int n, int32_t *len, int add)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) len[slots[i]] = (add ? len[slots[i]] : 0) + cu[i + 1] - cu[i];   // slots are distinct
}

hipError_t launch_prefill_set_len(const int32_t *d_slots, const int32_t *d_cu, int n_seqs,
                                  int32_t *d_len, int add, hipStream_t s)
{
    prefill_set_len_kernel<<<(n_seqs + 255) / 256, 256, 0, s>>>(d_slots, d_cu, n_seqs, d_len, add);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Rotary embedding (rotate-half pairing) of q and k in place + write of k, v into the cache.
// blockIdx.x is the token row; the gridDim.y blocks of a row share its (head, pair) and value
// elements round-robin, so that no thread has more than a few dependent memory round trips (a
// lone block per row spent most of a decode step's rope time waiting).  The angle pos *
// inv_freq[i] and its sine / cosine are evaluated in
// double so that the fp32 configuration stays inside its 1e-5 budget at any position.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void rope_kv_kernel(RopeArgs a)
{
    __shared__ float cs[128], sn[128];
    const int t = blockIdx.x;
    const int half = a.hd >> 1;
    const int pos = a.tok_pos[t];
    for (int i = threadIdx.x; i < half; i += 256) {
        if (pos < a.table_len) {
            float2 t = a.table[(size_t)pos * half + i];
            cs[i] = t.x;
            sn[i] = t.y;
        } else {
            double ang = (double)pos * a.inv_freq[i];
            double sv, cv;
            sincos(ang, &sv, &cv);
            cs[i] = (float)cv;
            sn[i] = (float)sv;
        }
    }
    __syncthreads();
    T *row = (T *)a.qkv + (size_t)t * a.ld;
    const int slot = a.tok_slot ? a.tok_slot[t] : -1;
    const int n_rot = (a.Hq + a.Hkv) * half;
    const int part = blockIdx.y * 256 + threadIdx.x, stride = gridDim.y * 256;
    for (int idx = part; idx < n_rot; idx += stride) {
        int h = idx / half, i = idx - h * half;
        T *v = row + (size_t)h * a.hd;
        float x0 = Elem<T>::ld(v + i), x1 = Elem<T>::ld(v + i + half);
        float y0 = x0 * cs[i] - x1 * sn[i];
        float y1 = x1 * cs[i] + x0 * sn[i];
        Elem<T>::st(v + i, y0);
        Elem<T>::st(v + i + half, y1);
        if (slot >= 0 && h >= a.Hq) {
            int g = h - a.Hq;
            T *plane = (T *)a.k_cache + ((size_t)slot * a.Hkv + g) * a.max_len * a.hd;
            if (a.fp8) {
                uint8_t *p8 = (uint8_t *)a.k_cache + ((size_t)slot * a.Hkv + g) * a.max_len * a.hd;
                p8[kblk8_off(pos, i)] = (uint8_t)e4m3_encode((double)y0 / a.k_scale);
                p8[kblk8_off(pos, i + half)] = (uint8_t)e4m3_encode((double)y1 / a.k_scale);
            } else if (a.blocked) {
                Elem<T>::st(plane + kblk_off(pos, i), y0);
                Elem<T>::st(plane + kblk_off(pos, i + half), y1);
            } else {
                Elem<T>::st(plane + (size_t)pos * a.hd + i, y0);
                Elem<T>::st(plane + (size_t)pos * a.hd + i + half, y1);
            }
        }
    }
    if (slot >= 0) {
        const T *vsrc = row + (size_t)(a.Hq + a.Hkv) * a.hd;
        for (int idx = part; idx < a.Hkv * a.hd; idx += stride) {
            int g = idx / a.hd, i = idx - g * a.hd;
            T *plane = (T *)a.v_cache + ((size_t)slot * a.Hkv + g) * a.max_len * a.hd;
            if (a.fp8)
                ((uint8_t *)a.v_cache)[((size_t)slot * a.Hkv + g) * a.max_len * a.hd + vblk8_off(pos, i)] =
                    (uint8_t)e4m3_encode((double)Elem<T>::ld(vsrc + idx) / a.v_scale);
            else if (a.blocked) plane[vblk_off(pos, i)] = vsrc[idx];
            else plane[(size_t)pos * a.hd + i] = vsrc[idx];
        }
    }
}

// (cos, sin) of pos * inv_freq[i], evaluated in double, for pos < table_len.
__global__ void rope_table_kernel(float2 *table, int table_len, int half, const double *inv_freq)
{
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)table_len * half) return;
    int pos = (int)(idx / half), i = (int)(idx % half);
    double sv, cv;
    sincos((double)pos * inv_freq[i], &sv, &cv);
    table[idx] = make_float2((float)cv, (float)sv);
}

hipError_t launch_rope_table(float2 *table, int table_len, int half, const double *inv_freq, hipStream_t s)
{
    size_t n = (size_t)table_len * half;
    rope_table_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(table, table_len, half, inv_freq);
    return hipGetLastError();
}

// Blocks 0 .. n_rows-1: RMSNorm of one bf16 row each.  Blocks n_rows .. n_rows + a.T - 1: the cache append
// of decode row t = block - n_rows (bf16, blocked or 8-bit cache): key rotated at tok_pos[t] in fp32 and
// stored, value stored; the qkv buffer is only read.
__global__ __launch_bounds__(256) void rmsnorm_append_kernel(RopeArgs a, const uint4 *__restrict__ x,
                                                             const uint4 *__restrict__ g, uint4 *__restrict__ y,
                                                             int n_rows, int d8, float d_inv, float eps)
{
    __shared__ float red[4];
    __shared__ float cs[128], sn[128];
    if ((int)blockIdx.x < n_rows) {
        rmsnorm_bf16_row(x + (size_t)blockIdx.x * d8, g, y + (size_t)blockIdx.x * d8, d8, d_inv, eps, red);
        return;
    }
    append_token_body(a, blockIdx.x - n_rows, cs, sn);
}

hipError_t launch_rmsnorm_append(const RopeArgs &a, const void *x, const void *g, void *y, int n_rows, int d,
                                 float eps, hipStream_t s)
{
    if (d % 8 != 0 || a.hd != 128 || !a.blocked || !a.tok_slot || n_rows < 0 || a.T < 0) return hipErrorInvalidValue;
    if (n_rows + a.T == 0) return hipSuccess;
    rmsnorm_append_kernel<<<n_rows + a.T, 256, 0, s>>>(a, (const uint4 *)x, (const uint4 *)g, (uint4 *)y, n_rows, d / 8,
                                                       1.0f / (float)d, eps);
    return hipGetLastError();
}

hipError_t launch_rope_kv(int dtype, const RopeArgs &a, hipStream_t s)
{
    if (a.T <= 0) return hipSuccess;
    // about two (head, pair) elements per thread for the few rows of a decode step; a prefill has
    // rows enough to fill the chip with one block each (measured faster there)
    const int n_rot = (a.Hq + a.Hkv) * (a.hd / 2);
    int slices = a.T >= 1024 ? 1 : (n_rot + 511) / 512;
    if (slices < 1) slices = 1;
    const dim3 grid((unsigned)a.T, (unsigned)slices);
    if (dtype == PD_F32) rope_kv_kernel<float><<<grid, 256, 0, s>>>(a);
    else rope_kv_kernel<bf16_t><<<grid, 256, 0, s>>>(a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Generic attention: one wavefront per (row, query head).  Lanes split the keys of a 64-key
// chunk for the scores and split head_dim for the weighted sum of values; online softmax across
// chunks.  head_dim <= 256.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void attn_generic_kernel(AttnArgs a)
{
    __shared__ float qs[4][256];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long item = (long long)blockIdx.x * 4 + wave;
    const long long n_items = (long long)a.T * a.Hq;
    const bool active = item < n_items;
    const int t = active ? (int)(item / a.Hq) : 0;
    const int h = active ? (int)(item - (long long)t * a.Hq) : 0;
    const int g = h / (a.Hq / a.Hkv);
    const int hd = a.hd;
    const T *q = (const T *)a.qkv + (size_t)t * a.ld + (size_t)h * hd;
    for (int i = lane; i < hd; i += 64) qs[wave][i] = active ? Elem<T>::ld(q + i) * a.scale : 0.f;
    __syncthreads();
    if (!active) return;

    const int pos = a.tok_pos[t];
    const int n_keys = pos + 1;
    const T *Kb, *Vb;
    size_t stride;
    if (a.decode) {
        size_t base = (((size_t)a.tok_slot[t] * a.Hkv + g) * a.max_len) * hd;
        Kb = (const T *)a.k_cache + base;
        Vb = (const T *)a.v_cache + base;
        stride = (size_t)hd;
    } else {
        const T *first = (const T *)a.qkv + (size_t)(t - pos) * a.ld;
        Kb = first + (size_t)(a.Hq + g) * hd;
        Vb = first + (size_t)(a.Hq + a.Hkv + g) * hd;
        stride = (size_t)a.ld;
    }

    float m = -INFINITY, l = 0.f;
    float o[4] = {0.f, 0.f, 0.f, 0.f};
    for (int c0 = 0; c0 < n_keys; c0 += 64) {
        int s = c0 + lane;
        float sc = -INFINITY;
        if (s < n_keys) {
            const T *kr = Kb + (size_t)s * stride;
            float acc = 0.f;
            for (int i = 0; i < hd; ++i) acc = fmaf(qs[wave][i], Elem<T>::ld(kr + i), acc);
            sc = acc;
        }
        float m_new = fmaxf(m, wave_max(sc));
        float p = (s < n_keys) ? expf(sc - m_new) : 0.f;
        float corr = expf(m - m_new);   // m = -inf on the first chunk -> 0
        l = l * corr + wave_sum(p);
        m = m_new;
        int cnt = n_keys - c0 < 64 ? n_keys - c0 : 64;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] *= corr;
        for (int j = 0; j < cnt; ++j) {
            float pj = __shfl(p, j, 64);
            const T *vr = Vb + (size_t)(c0 + j) * stride;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                int i = lane + 64 * e;
                if (i < hd) o[e] = fmaf(pj, Elem<T>::ld(vr + i), o[e]);
            }
        }
    }
    T *orow = (T *)a.o + (size_t)t * a.Hq * hd + (size_t)h * hd;
    float inv = 1.0f / l;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        int i = lane + 64 * e;
        if (i < hd) Elem<T>::st(orow + i, o[e] * inv);
    }
}

hipError_t launch_attn_generic(int dtype, const AttnArgs &a, hipStream_t s)
{
    long long items = (long long)a.T * a.Hq;
    if (items <= 0) return hipSuccess;
    unsigned grid = (unsigned)((items + 3) / 4);
    if (dtype == PD_F32) attn_generic_kernel<float><<<grid, 256, 0, s>>>(a);
    else attn_generic_kernel<bf16_t><<<grid, 256, 0, s>>>(a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Cache fill / read-back: [Hkv, len, hd] tensor <-> one slot of the cache.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void kv_copy_kernel(T *ck, T *cv, T *k, T *v, int slot, int Hkv, int len, int hd,
                               int max_len, int blocked, int to_cache)
{
    size_t n = (size_t)Hkv * len * hd;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n;
         idx += (size_t)gridDim.x * blockDim.x) {
        int i = (int)(idx % hd);
        size_t r = idx / hd;
        int p = (int)(r % len);
        int g = (int)(r / len);
        size_t plane = ((size_t)slot * Hkv + g) * max_len * hd;
        size_t c = plane + (blocked ? kblk_off(p, i) : (size_t)p * hd + i);
        size_t cvo = plane + (blocked ? vblk_off(p, i) : (size_t)p * hd + i);
        if (to_cache) {
            ck[c] = k[idx];
            cv[cvo] = v[idx];
        } else {
            k[idx] = ck[c];
            v[idx] = cv[cvo];
        }
    }
}

hipError_t launch_kv_copy(int dtype, void *cache_k, void *cache_v, const void *k, const void *v,
                          int slot, int Hkv, int len, int hd, int max_len, int blocked, int to_cache,
                          hipStream_t s)
{
    size_t n = (size_t)Hkv * len * hd;
    if (n == 0) return hipSuccess;
    unsigned grid = (unsigned)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    if (dtype == PD_F32)
        kv_copy_kernel<float><<<grid, 256, 0, s>>>((float *)cache_k, (float *)cache_v, (float *)k,
                                                   (float *)v, slot, Hkv, len, hd, max_len, blocked, to_cache);
    else
        kv_copy_kernel<uint16_t><<<grid, 256, 0, s>>>((uint16_t *)cache_k, (uint16_t *)cache_v,
                                                      (uint16_t *)k, (uint16_t *)v, slot, Hkv, len,
                                                      hd, max_len, blocked, to_cache);
    return hipGetLastError();
}

// [Hkv, len, 128] bf16 tensor <-> one slot of the 8-bit E4M3 blocked cache.  Into the cache: the
// code of x / scale; out of it: scale * value(code), formed in double and rounded once to float
// and once to bf16.
__global__ void kv_copy_fp8_kernel(uint8_t *ck, uint8_t *cv, bf16_t *k, bf16_t *v, int slot, int Hkv,
                                   int len, int max_len_pad, double k_scale, double v_scale, int to_cache)
{
    size_t n = (size_t)Hkv * len * 128;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < n;
         idx += (size_t)gridDim.x * blockDim.x) {
        int i = (int)(idx & 127);
        size_t r = idx >> 7;
        int p = (int)(r % len);
        int g = (int)(r / len);
        size_t plane = ((size_t)slot * Hkv + g) * max_len_pad * 128;
        size_t c = plane + kblk8_off(p, i), cvo = plane + vblk8_off(p, i);
        if (to_cache) {
            ck[c] = (uint8_t)e4m3_encode((double)bf2f(k[idx]) / k_scale);
            cv[cvo] = (uint8_t)e4m3_encode((double)bf2f(v[idx]) / v_scale);
        } else {
            k[idx] = f2bf((float)(k_scale * (double)e4m3_decode(ck[c])));
            v[idx] = f2bf((float)(v_scale * (double)e4m3_decode(cv[cvo])));
        }
    }
}

hipError_t launch_kv_copy_fp8(void *cache_k, void *cache_v, const void *k, const void *v, int slot, int Hkv,
                              int len, int max_len_pad, double k_scale, double v_scale, int to_cache,
                              hipStream_t s)
{
    size_t n = (size_t)Hkv * len * 128;
    if (n == 0) return hipSuccess;
    unsigned grid = (unsigned)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    kv_copy_fp8_kernel<<<grid, 256, 0, s>>>((uint8_t *)cache_k, (uint8_t *)cache_v, (bf16_t *)k, (bf16_t *)v,
                                            slot, Hkv, len, max_len_pad, k_scale, v_scale, to_cache);
    return hipGetLastError();
}

// ---- embedding: one block per token row, 4-byte words ----------------------------------------------
__global__ __launch_bounds__(256) void embed_rows_kernel(uint32_t *__restrict__ out, const uint32_t *__restrict__ table,
                                                         const int32_t *__restrict__ ids, int n_rows, int row_words)
{
    const int t = blockIdx.x;
    const int id = ids[t];
    const bool ok = id >= 0 && id < n_rows;
    const uint32_t *src = table + (size_t)(ok ? id : 0) * row_words;
    uint32_t *dst = out + (size_t)t * row_words;
    for (int i = threadIdx.x; i < row_words; i += 256) dst[i] = ok ? src[i] : 0u;
}

hipError_t launch_embed_rows(void *out, const void *table, const int32_t *ids, int T, int n_rows,
                             size_t row_bytes, hipStream_t s)
{
    if (T <= 0) return hipSuccess;
    embed_rows_kernel<<<T, 256, 0, s>>>((uint32_t *)out, (const uint32_t *)table, ids, n_rows, (int)(row_bytes / 4));
    return hipGetLastError();
}

// ---- 8-bit activations: per-row power-of-two scale and E4M3 codes -----------------------------------
// One workgroup per row of x [T, K] (bf16).  The scale is the smallest power of two s with
// max|x_row| / s <= 448 (1 for a row of zeros or with an infinity); x / s is exact, the hardware
// conversion rounds to nearest even and is given only values inside +-448, so the codes are those of
// a saturating round-to-nearest-even encoder.
__global__ __launch_bounds__(256) void quant_rows_e4m3_kernel(const uint16_t *__restrict__ x, int ldx, int K,
                                                              uint8_t *__restrict__ codes, float *__restrict__ scales)
{
    __shared__ float red[4];
    __shared__ float inv_s;
    const int row = blockIdx.x, tid = threadIdx.x;
    const uint4 *p = (const uint4 *)(x + (size_t)row * ldx);
    const int n8 = K >> 3;
    float m = 0.f;
    for (int i = tid; i < n8; i += 256) {
        const uint4 v = p[i];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            m = fmaxf(m, fabsf(bfbits2f(w[j] & 0xffffu)));
            m = fmaxf(m, fabsf(bfbits2f(w[j] >> 16)));
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if ((tid & 63) == 0) red[tid >> 6] = m;
    __syncthreads();
    if (tid == 0) {
        m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        float s = 1.f;
        if (m > 0.f && m < INFINITY) {
            int e;
            const double f = frexp((double)m / 448.0, &e);    // m / 448 = f * 2^e, f in [0.5, 1)
            s = (float)ldexp(1.0, f == 0.5 ? e - 1 : e);
        }
        scales[row] = s;
        inv_s = 1.0f / s;
    }
    __syncthreads();
    const float inv = inv_s;
    uint2 *q = (uint2 *)(codes + (size_t)row * K);
    for (int i = tid; i < n8; i += 256) {
        const uint4 v = p[i];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
        float f[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f[2 * j] = bfbits2f(w[j] & 0xffffu) * inv;
            f[2 * j + 1] = bfbits2f(w[j] >> 16) * inv;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (f[j] == f[j]) f[j] = fminf(fmaxf(f[j], -448.f), 448.f);
        int lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], 0, false);
        lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], lo, true);
        int hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[4], f[5], 0, false);
        hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[6], f[7], hi, true);
        q[i] = make_uint2((uint32_t)lo, (uint32_t)hi);
    }
}

// RMSNorm and row quantisation in one pass for rows of up to 8192 bf16 elements: the normalised row is
// rounded to bf16 exactly as rmsnorm_bf16_vec_kernel rounds it, kept in registers, and encoded like
// quant_rows_e4m3_kernel encodes a stored row; the bf16 row itself is not written.
__global__ __launch_bounds__(256) void rmsnorm_quant_e4m3_kernel(const uint4 *__restrict__ x, const uint4 *__restrict__ g,
                                                                 int d8, float d_inv, float eps,
                                                                 uint8_t *__restrict__ codes, float *__restrict__ scales)
{
    __shared__ float red[4], redm[4];
    __shared__ float inv_s;
    const int tid = threadIdx.x;
    const uint4 *xr = x + (size_t)blockIdx.x * d8;
    uint4 xv[4];
    float ss = 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = tid + u * 256;
        xv[u] = i < d8 ? xr[i] : make_uint4(0u, 0u, 0u, 0u);
        const uint32_t w[4] = {xv[u].x, xv[u].y, xv[u].z, xv[u].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float a = bfbits2f(w[j] & 0xffffu), b = bfbits2f(w[j] >> 16);
            ss += a * a + b * b;
        }
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    const float inv = rsqrtf((red[0] + red[1] + red[2] + red[3]) * d_inv + eps);
    uint32_t y[4][4];
    float m = 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = tid + u * 256;
        const uint4 gg = i < d8 ? g[i] : make_uint4(0u, 0u, 0u, 0u);
        const uint32_t w[4] = {xv[u].x, xv[u].y, xv[u].z, xv[u].w}, gw[4] = {gg.x, gg.y, gg.z, gg.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float a = bfbits2f(w[j] & 0xffffu) * inv * bfbits2f(gw[j] & 0xffffu);
            float b = bfbits2f(w[j] >> 16) * inv * bfbits2f(gw[j] >> 16);
            y[u][j] = pack2bf(a, b);
            m = fmaxf(m, fmaxf(fabsf(bfbits2f(y[u][j] & 0xffffu)), fabsf(bfbits2f(y[u][j] >> 16))));
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if ((tid & 63) == 0) redm[tid >> 6] = m;
    __syncthreads();
    if (tid == 0) {
        m = fmaxf(fmaxf(redm[0], redm[1]), fmaxf(redm[2], redm[3]));
        float s = 1.f;
        if (m > 0.f && m < INFINITY) {
            int e;
            const double f = frexp((double)m / 448.0, &e);
            s = (float)ldexp(1.0, f == 0.5 ? e - 1 : e);
        }
        scales[blockIdx.x] = s;
        inv_s = 1.0f / s;
    }
    __syncthreads();
    const float is = inv_s;
    uint2 *q = (uint2 *)(codes + (size_t)blockIdx.x * d8 * 8);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = tid + u * 256;
        if (i >= d8) continue;
        float f[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f[2 * j] = bfbits2f(y[u][j] & 0xffffu) * is;
            f[2 * j + 1] = bfbits2f(y[u][j] >> 16) * is;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (f[j] == f[j]) f[j] = fminf(fmaxf(f[j], -448.f), 448.f);
        int lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], 0, false);
        lo = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], lo, true);
        int hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[4], f[5], 0, false);
        hi = __builtin_amdgcn_cvt_pk_fp8_f32(f[6], f[7], hi, true);
        q[i] = make_uint2((uint32_t)lo, (uint32_t)hi);
    }
}

bool rmsnorm_quant_supported(int d) { return d % 8 == 0 && d <= 8192; }

hipError_t launch_rmsnorm_quant_e4m3(const void *x, const void *g, int T, int d, float eps, void *codes,
                                     float *scales, hipStream_t s)
{
    if (T <= 0) return hipSuccess;
    if (!rmsnorm_quant_supported(d)) return hipErrorInvalidValue;
    rmsnorm_quant_e4m3_kernel<<<T, 256, 0, s>>>((const uint4 *)x, (const uint4 *)g, d / 8, 1.0f / (float)d, eps,
                                                (uint8_t *)codes, scales);
    return hipGetLastError();
}

hipError_t launch_quant_rows_e4m3(const void *x, int ldx, int T, int K, void *codes, float *scales, hipStream_t s)
{
    if (T <= 0) return hipSuccess;
    if (K % 8 != 0 || ldx % 8 != 0) return hipErrorInvalidValue;
    quant_rows_e4m3_kernel<<<T, 256, 0, s>>>((const uint16_t *)x, ldx, K, (uint8_t *)codes, scales);
    return hipGetLastError();
}

// 8-bit weight codes from the skinny kernels' layout into the tiled kernel's: the matrix seen as
// [n_rows, K / 2] two-byte elements in the block pack of wpack_off; 16 codes per thread step.
__global__ __launch_bounds__(256) void repack_w8_tiles_kernel(const uint8_t *__restrict__ src, uint8_t *__restrict__ dst,
                                                              int n_rows, int K)
{
    const size_t n_items = (size_t)n_rows * (K >> 4);
    for (size_t it = (size_t)blockIdx.x * 256 + threadIdx.x; it < n_items; it += (size_t)gridDim.x * 256) {
        const int n = (int)(it / (K >> 4)), k = (int)(it % (K >> 4)) << 4;
        const uint2 a = *(const uint2 *)(src + w8pack_off(n, k, K));
        const uint2 b = *(const uint2 *)(src + w8pack_off(n, k + 8, K));
        *(uint4 *)(dst + 2 * wpack_off(n, k >> 1, K >> 1)) = make_uint4(a.x, a.y, b.x, b.y);
    }
}

// the same from plain row-major codes [n_rows, K]
__global__ __launch_bounds__(256) void pack_rows_e4m3_tiles_kernel(const uint8_t *__restrict__ src, uint8_t *__restrict__ dst,
                                                                   int n_rows, int K)
{
    const size_t n_items = (size_t)n_rows * (K >> 4);
    for (size_t it = (size_t)blockIdx.x * 256 + threadIdx.x; it < n_items; it += (size_t)gridDim.x * 256) {
        const int n = (int)(it / (K >> 4)), k = (int)(it % (K >> 4)) << 4;
        *(uint4 *)(dst + 2 * wpack_off(n, k >> 1, K >> 1)) = *(const uint4 *)(src + (size_t)n * K + k);
    }
}

hipError_t launch_pack_rows_e4m3_tiles(const void *src, void *dst, int n_rows, int K, hipStream_t s)
{
    if (K % 64 != 0 || n_rows % 16 != 0) return hipErrorInvalidValue;
    pack_rows_e4m3_tiles_kernel<<<2048, 256, 0, s>>>((const uint8_t *)src, (uint8_t *)dst, n_rows, K);
    return hipGetLastError();
}

hipError_t launch_repack_w8_tiles(const void *src8, void *dst, int n_rows, int K, hipStream_t s)
{
    if (K % 64 != 0 || n_rows % 16 != 0) return hipErrorInvalidValue;
    repack_w8_tiles_kernel<<<2048, 256, 0, s>>>((const uint8_t *)src8, (uint8_t *)dst, n_rows, K);
    return hipGetLastError();
}

// ---- plain copy (traffic-counter calibration) -----------------------------------------------------
__global__ __launch_bounds__(256) void stream_copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src,
                                                          size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

hipError_t launch_stream_copy(void *dst, const void *src, size_t n_vec16, hipStream_t s)
{
    const size_t want = (n_vec16 + 255) / 256;
    const unsigned grid = (unsigned)(want < 256 * 16 ? (want ? want : 1) : 256 * 16);
    stream_copy_kernel<<<grid, 256, 0, s>>>((uint4 *)dst, (const uint4 *)src, n_vec16);
    return hipGetLastError();
}

// ---- matrix-core loop on register operands (ceiling of the matrix pipe for given operand values) -----
typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_f32x16 __attribute__((ext_vector_type(16)));

// Each of the 512 lanes of a workgroup loads four A fragments and two B fragments (8 bf16 each) once and
// then issues nothing but v_mfma_f32_32x32x16_bf16 on them: iters x 8 instructions per wave, 8 independent
// accumulator blocks, no memory traffic inside the loop.
__global__ __launch_bounds__(512) void mfma_probe_kernel(float *__restrict__ sink, const uint4 *__restrict__ a_vals,
                                                         const uint4 *__restrict__ b_vals, int iters)
{
    probe_bf16x8 fa[4], fb[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[i] = __builtin_bit_cast(probe_bf16x8, a_vals[threadIdx.x * 4 + i]);
#pragma unroll
    for (int i = 0; i < 2; ++i) fb[i] = __builtin_bit_cast(probe_bf16x8, b_vals[threadIdx.x * 2 + i]);
    probe_f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) t += acc[i][j][r];
    sink[(size_t)blockIdx.x * 512 + threadIdx.x] = t;
}

hipError_t launch_mfma_probe(float *sink, const void *a_vals, const void *b_vals, int n_workgroups, int iters, hipStream_t s)
{
    mfma_probe_kernel<<<n_workgroups, 512, 0, s>>>(sink, (const uint4 *)a_vals, (const uint4 *)b_vals, iters);
    return hipGetLastError();
}

}  // namespace pd
