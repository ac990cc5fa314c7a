// Block mean-pooling of Q, K, V (Sec. 3.2 "Compression Branch": non-overlapping average
// pooling, here over runs of B consecutive tokens) fused with the re-layout of K and V into
// per-(head, block) MFMA operand tiles for the selection kernel.  One pass over Q, K, V: the
// kernel is HBM-bandwidth bound (reads 3 * n_tok * heads * 64 elements once).
#include "s3r_device.h"
#include "s3r_kernels.h"

namespace s3r {

template <typename T> struct Load8;
template <> struct Load8<bf16_t> {
    static __device__ __forceinline__ void run(const bf16_t *p, float (&f)[8], bf16x8 &raw)
    {
        raw = *reinterpret_cast<const bf16x8 *>(p);
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = static_cast<float>(raw[i]);
    }
};
template <> struct Load8<float> {
    static __device__ __forceinline__ void run(const float *p, float (&f)[8], bf16x8 &raw)
    {
        const floatx4 a = *reinterpret_cast<const floatx4 *>(p);
        const floatx4 b = *reinterpret_cast<const floatx4 *>(p + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) { f[i] = a[i]; f[4 + i] = b[i]; }
#pragma unroll
        for (int i = 0; i < 8; ++i) raw[i] = static_cast<bf16_t>(f[i]);   // the hi part of the operand pair
    }
};

// x = hi + lo + O(2^-17 |x|) with hi = bf16(x), lo = bf16(x - hi): an operand pair; with the third part
// lo2 = bf16(x - hi - lo) the sum is x itself (each residual has 8 significant bits fewer than the one before).
// V goes to the matrix pipe as a pair (its products with probabilities in [0, 1] need no more), K as a triple:
// the error of a logit enters the result through an exponential, in absolute terms, so the scores must keep
// all 24 bits of K and Q however large their entries are.
__device__ __forceinline__ bf16x8 lo_parts(const float (&f)[8], const bf16x8 &hi)
{
    bf16x8 lo;
#pragma unroll
    for (int i = 0; i < 8; ++i) lo[i] = static_cast<bf16_t>(f[i] - static_cast<float>(hi[i]));
    return lo;
}
__device__ __forceinline__ bf16x8 lo2_parts(const float (&f)[8], const bf16x8 &hi, const bf16x8 &lo)
{
    bf16x8 lo2;
#pragma unroll
    for (int i = 0; i < 8; ++i)
        lo2[i] = static_cast<bf16_t>((f[i] - static_cast<float>(hi[i])) - static_cast<float>(lo[i]));
    return lo2;
}

// grid: one workgroup per (block j, head h), head fastest; 256 threads.
// Thread (r0 = tid / 8, c = tid % 8) handles channels 8c..8c+7 of rows r0, r0 + 32, ...
template <typename T, int B, bool REPACK>
__global__ __launch_bounds__(256) void pool_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                                   const T *__restrict__ v, float *__restrict__ qc,
                                                   float *__restrict__ kc, float *__restrict__ vc,
                                                   bf16_t *__restrict__ kb, bf16_t *__restrict__ vb,
                                                   int64_t n_tok, int heads, int64_t n_blk, TokenMap map,
                                                   InStride in, int64_t lo_off)
{
    // fp32 inputs are re-laid-out as bf16 operand parts: the lo tiles lie lo_off elements after the hi ones, K's
    // third part another lo_off elements on
    constexpr bool PAIRS = REPACK && sizeof(T) == 4;
    constexpr int VS_STRIDE = 72;  // bf16 elements per staged V row (64 + pad: conflict-free columns)
    __shared__ float red[3][32][65];
    __shared__ bf16_t vs[REPACK ? B : 1][VS_STRIDE];
    __shared__ bf16_t vs_lo[PAIRS ? B : 1][VS_STRIDE];

    const int64_t bid = blockIdx.x;
    const int h = static_cast<int>(bid % heads);
    const int64_t j = bid / heads;
    const int tid = threadIdx.x;
    const int c = tid & 7, r0 = tid >> 3;
    const int64_t t0 = j * B;
    const int len = map.block_len(j, B, n_tok);
    const int64_t tile_base = (static_cast<int64_t>(h) * n_blk + j) * (B * 64);

    float acc[3][8];
#pragma unroll
    for (int x = 0; x < 3; ++x)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[x][i] = 0.f;

#pragma unroll
    for (int r = r0; r < B; r += 32) {
        float f[8];
        bf16x8 raw;
        const bool valid = r < len;
        const int64_t off = in.at(map.row(valid ? t0 + r : t0), h, heads) + c * 8;
        if (valid) {
            Load8<T>::run(q + off, f, raw);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[0][i] += f[i];
            Load8<T>::run(k + off, f, raw);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[1][i] += f[i];
        }
        if constexpr (REPACK) {
            if (!valid) {
#pragma unroll
                for (int i = 0; i < 8; ++i) { raw[i] = static_cast<bf16_t>(0.f); f[i] = 0.f; }
            }
            // 32-row tiles in operand order; a block of 16 rows is stored as the 16-row half of such a
            // tile, column chunk by column chunk, so that two of them interleave into one tile
            bf16_t *dst = (B >= 32) ? kb + tile_base + (r >> 5) * kRowTileElems + row_tile_chunk_offset(r & 31, c)
                                    : kb + tile_base + (c * 16 + r) * 8;
            *reinterpret_cast<bf16x8 *>(dst) = raw;
            if constexpr (PAIRS) {
                const bf16x8 lo = lo_parts(f, raw);
                *reinterpret_cast<bf16x8 *>(dst + lo_off) = lo;
                *reinterpret_cast<bf16x8 *>(dst + 2 * lo_off) = lo2_parts(f, raw, lo);
            }
        }
        if (valid) {
            Load8<T>::run(v + off, f, raw);
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[2][i] += f[i];
        }
        if constexpr (REPACK) {
            if (!valid) {
#pragma unroll
                for (int i = 0; i < 8; ++i) { raw[i] = static_cast<bf16_t>(0.f); f[i] = 0.f; }
            }
            *reinterpret_cast<bf16x8 *>(&vs[r][c * 8]) = raw;
            if constexpr (PAIRS) *reinterpret_cast<bf16x8 *>(&vs_lo[r][c * 8]) = lo_parts(f, raw);
        }
    }
#pragma unroll
    for (int x = 0; x < 3; ++x)
#pragma unroll
        for (int i = 0; i < 8; ++i) red[x][r0][c * 8 + i] = acc[x][i];
    __syncthreads();

    if (qc != nullptr && tid < 192) {
        const int x = tid >> 6, d = tid & 63;
        float s = 0.f;
#pragma unroll
        for (int g = 0; g < 32; ++g) s += red[x][g][d];
        float *dst = (x == 0) ? qc : (x == 1) ? kc : vc;
        dst[(static_cast<int64_t>(h) * n_blk + j) * 64 + d] = s / static_cast<float>(len);
    }

    if constexpr (REPACK) {
        // V tile, contraction (key) index made contiguous per lane: see tr_tile_key().
        for (int ci = tid; ci < B * 8; ci += 256) {
            const int l = ci & 63, dt = (ci >> 6) & 1, u = ci >> 7;
            const int d = 32 * dt + (l & 31);
            bf16x8 o;
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = vs[tr_tile_key(u, l, i)][d];
            *reinterpret_cast<bf16x8 *>(vb + tile_base + static_cast<int64_t>(ci) * 8) = o;
            if constexpr (PAIRS) {
#pragma unroll
                for (int i = 0; i < 8; ++i) o[i] = vs_lo[tr_tile_key(u, l, i)][d];
                *reinterpret_cast<bf16x8 *>(vb + lo_off + tile_base + static_cast<int64_t>(ci) * 8) = o;
            }
        }
    }
}

template <typename T, int B, bool REPACK>
static hipError_t run_pool(const void *q, const void *k, const void *v, float *qc, float *kc,
                           float *vc, void *kb, void *vb, int64_t n_tok, int heads, int64_t n_blk,
                           TokenMap map, InStride in, hipStream_t stream)
{
    const int64_t grid = n_blk * heads;
    const int64_t lo_off = static_cast<int64_t>(heads) * n_blk * B * 64;   // fp32 inputs: [hi tiles | lo tiles | K: lo2 tiles]
    hipLaunchKernelGGL((pool_kernel<T, B, REPACK>), dim3(static_cast<unsigned>(grid)), dim3(256), 0,
                       stream, static_cast<const T *>(q), static_cast<const T *>(k),
                       static_cast<const T *>(v), qc, kc, vc, static_cast<bf16_t *>(kb),
                       static_cast<bf16_t *>(vb), n_tok, heads, n_blk, map, in, lo_off);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void block_lens_kernel(TokenMap map, int block, int64_t n_tok, int64_t n_blk,
                                                         int32_t *__restrict__ blk_len)
{
    const int64_t j = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (j < n_blk) blk_len[j] = map.block_len(j, block, n_tok);
}

hipError_t launch_block_lens(TokenMap map, int block, int64_t n_tok, int64_t n_blk, int32_t *blk_len,
                             hipStream_t stream)
{
    const int64_t grid = (n_blk + 255) / 256;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(block_lens_kernel, dim3(static_cast<unsigned>(grid)), dim3(256), 0, stream, map, block, n_tok,
                       n_blk, blk_len);
    return hipGetLastError();
}

hipError_t launch_pool(const void *q, const void *k, const void *v, float *qc, float *kc, float *vc,
                       void *kb, void *vb, int64_t n_tok, int heads, int block, bool is_bf16,
                       TokenMap map, InStride in, hipStream_t stream)
{
    const int64_t n_blk = (n_tok + block - 1) / block;
    if (n_blk * heads > 0x7fffffffLL) return hipErrorInvalidValue;
    if (map.period != 0 && n_tok > 0x7fffffffLL) return hipErrorInvalidValue;
    const bool repack = kb != nullptr;
#define S3R_POOL_CASE(TT, BB, RR) \
    return run_pool<TT, BB, RR>(q, k, v, qc, kc, vc, kb, vb, n_tok, heads, n_blk, map, in, stream)
    if (is_bf16) {
        switch (block) {
        case 16: if (repack) S3R_POOL_CASE(bf16_t, 16, true); else S3R_POOL_CASE(bf16_t, 16, false);
        case 32: if (repack) S3R_POOL_CASE(bf16_t, 32, true); else S3R_POOL_CASE(bf16_t, 32, false);
        case 64: if (repack) S3R_POOL_CASE(bf16_t, 64, true); else S3R_POOL_CASE(bf16_t, 64, false);
        case 128: if (repack) S3R_POOL_CASE(bf16_t, 128, true); else S3R_POOL_CASE(bf16_t, 128, false);
        }
    } else {
        switch (block) {
        case 16: if (repack) S3R_POOL_CASE(float, 16, true); else S3R_POOL_CASE(float, 16, false);
        case 32: if (repack) S3R_POOL_CASE(float, 32, true); else S3R_POOL_CASE(float, 32, false);
        case 64: if (repack) S3R_POOL_CASE(float, 64, true); else S3R_POOL_CASE(float, 64, false);
        case 128: if (repack) S3R_POOL_CASE(float, 128, true); else S3R_POOL_CASE(float, 128, false);
        }
    }
#undef S3R_POOL_CASE
    return hipErrorInvalidValue;
}

}  // namespace s3r
