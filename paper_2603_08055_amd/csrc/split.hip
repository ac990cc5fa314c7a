// Pooled fp32 tensors -> bf16 operand tiles for the compression-branch kernel.
// Each fp32 value x is written as hi = bf16(x) and lo = bf16(x - hi), so that products of
// hi/lo pairs recover fp32-level accuracy for S_guide (eq. 4), whose ordering decides TopK.
// Tiny: touches 3 * heads * n_blk * 64 floats once.
//
// For the TopK sweeps (compress.hip) Qc and Kc are also written as single fp16 tiles, each head scaled
// by a power of two that brings its largest component into [0.5, 1) (exact, and it keeps fp16 from
// overflowing or flushing whatever the magnitude of the inputs).  pooled_stats_kernel finds those
// maxima, and the largest key norm of each head, which the sweeps turn into an error bound.
#include "s3r_device.h"
#include "s3r_kernels.h"

namespace s3r {

// grid: (tiles_padded, heads); 256 threads; one 32-row tile of Qc, Kc and Vc per workgroup.
__global__ __launch_bounds__(256) void split_kernel(const float *__restrict__ qc,
                                                    const float *__restrict__ kc,
                                                    const float *__restrict__ vc,
                                                    bf16_t *__restrict__ qs_hi, bf16_t *__restrict__ qs_lo,
                                                    bf16_t *__restrict__ ks_hi, bf16_t *__restrict__ ks_lo,
                                                    bf16_t *__restrict__ vt_hi, bf16_t *__restrict__ vt_lo,
                                                    _Float16 *__restrict__ q_f16, _Float16 *__restrict__ k_f16,
                                                    int64_t n_blk, int64_t tiles_padded,
                                                    const HeadStats *__restrict__ stats)
{
    __shared__ float vsf[32][65];
    const int tile = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
    const int r = tid >> 3, c = tid & 7;  // row in tile, 8-channel chunk
    const int64_t row = static_cast<int64_t>(tile) * 32 + r;
    const bool valid = row < n_blk;
    const int64_t src = (static_cast<int64_t>(h) * n_blk + row) * 64 + c * 8;
    const int64_t tile_base = (static_cast<int64_t>(h) * tiles_padded + tile) * kRowTileElems;

    float f[8];
    bf16x8 hi, lo;
    auto split8 = [&]() {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            hi[i] = static_cast<bf16_t>(f[i]);
            lo[i] = static_cast<bf16_t>(f[i] - static_cast<float>(hi[i]));
        }
    };
    auto load8 = [&](const float *p) {
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = valid ? p[src + i] : 0.f;
    };
    const int dst = row_tile_chunk_offset(r, c);
    typedef _Float16 half8 __attribute__((ext_vector_type(8)));
    auto store_f16 = [&](_Float16 *t, float pow2) {
        half8 hv;
#pragma unroll
        for (int i = 0; i < 8; ++i) hv[i] = static_cast<_Float16>(f[i] * pow2);
        *reinterpret_cast<half8 *>(t + tile_base + dst) = hv;
    };
    load8(qc);
    split8();
    *reinterpret_cast<bf16x8 *>(qs_hi + tile_base + dst) = hi;
    *reinterpret_cast<bf16x8 *>(qs_lo + tile_base + dst) = lo;
    if (q_f16 != nullptr) store_f16(q_f16, stats[h].sq);
    load8(kc);
    if (k_f16 != nullptr) store_f16(k_f16, stats[h].sk);
    split8();
    *reinterpret_cast<bf16x8 *>(ks_hi + tile_base + dst) = hi;
    *reinterpret_cast<bf16x8 *>(ks_lo + tile_base + dst) = lo;
    load8(vc);
#pragma unroll
    for (int i = 0; i < 8; ++i) vsf[r][c * 8 + i] = f[i];
    __syncthreads();
    // transposed tile: chunk ci = (u * 2 + dt) * 64 + lane, 256 chunks, one per thread
    {
        const int l = tid & 63, dt = (tid >> 6) & 1, u = tid >> 7;
        const int d = 32 * dt + (l & 31);
#pragma unroll
        for (int i = 0; i < 8; ++i) f[i] = vsf[tr_tile_key(u, l, i)][d];
        split8();
        *reinterpret_cast<bf16x8 *>(vt_hi + tile_base + tid * 8) = hi;
        if (vt_lo != nullptr) *reinterpret_cast<bf16x8 *>(vt_lo + tile_base + tid * 8) = lo;
    }
}

__global__ void clear_words_kernel(unsigned *__restrict__ w, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) w[i] = 0u;
}

// grid: (tiles_padded, heads); 256 threads; the rows of one 32-row tile.  Largest |component| of Qc and
// of Kc and largest squared L2 norm of a Kc row, as atomic maxima into slots [head][3][kStatSlots]
// (non-negative floats order like their bit patterns; a maximum does not depend on the order of the
// atomics; many slots per head because atomics on one address queue up).
__global__ __launch_bounds__(256) void pooled_stats_kernel(const float *__restrict__ qc, const float *__restrict__ kc,
                                                           int64_t n_blk, unsigned *__restrict__ slots)
{
    __shared__ float part[4][3];
    const int tile = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
    const int r = tid >> 3, c = tid & 7;
    const int64_t row = static_cast<int64_t>(tile) * 32 + r;
    const bool valid = row < n_blk;
    const int64_t src = (static_cast<int64_t>(h) * n_blk + row) * 64 + c * 8;
    float qm = 0.f, km = 0.f, kn2 = 0.f;
    if (valid) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            qm = fmaxf(qm, fabsf(qc[src + i]));
            const float kv = kc[src + i];
            km = fmaxf(km, fabsf(kv));
            kn2 = fmaf(kv, kv, kn2);
        }
    }
    kn2 += __shfl_xor(kn2, 1, 64);  // the 8 threads of a row
    kn2 += __shfl_xor(kn2, 2, 64);
    kn2 += __shfl_xor(kn2, 4, 64);
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        qm = fmaxf(qm, __shfl_xor(qm, d, 64));
        km = fmaxf(km, __shfl_xor(km, d, 64));
        kn2 = fmaxf(kn2, __shfl_xor(kn2, d, 64));
    }
    if ((tid & 63) == 0) { part[tid >> 6][0] = qm; part[tid >> 6][1] = km; part[tid >> 6][2] = kn2; }
    __syncthreads();
    if (tid < 3) {
        const float m = fmaxf(fmaxf(part[0][tid], part[1][tid]), fmaxf(part[2][tid], part[3][tid]));
        atomicMax(slots + (h * 3 + tid) * kStatSlots + (tile % kStatSlots), __float_as_uint(m));
    }
}

// grid: heads; 64 threads.  Slots -> the head's scale factors and scaled key norm.
__global__ __launch_bounds__(64) void head_stats_kernel(const unsigned *__restrict__ slots, HeadStats *__restrict__ stats)
{
    static_assert(kStatSlots == 64, "one slot per lane");
    const int h = blockIdx.x, lane = threadIdx.x;
    float m[3];
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        m[a] = __uint_as_float(slots[(h * 3 + a) * kStatSlots + lane]);
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) m[a] = fmaxf(m[a], __shfl_xor(m[a], d, 64));
    }
    if (lane != 0) return;
    // 2^-e with max * 2^-e in [0.5, 1); exponents kept within +-60 (beyond that the scaling only helps less)
    auto exponent = [](float mx) -> int {
        if (!(mx > 0.f) || !(mx < INFINITY)) return 0;
        int e;
        frexpf(mx, &e);
        return e < -60 ? -60 : e > 60 ? 60 : e;
    };
    const int eq = exponent(m[0]), ek = exponent(m[1]);
    HeadStats st;
    st.sq = ldexpf(1.f, -eq);
    st.sk = ldexpf(1.f, -ek);
    st.sqsk = ldexpf(1.f, -eq - ek);
    st.inv_sqsk = ldexpf(1.f, eq + ek);
    st.kn = sqrtf(m[2]) * st.sk * 1.0001f;  // largest scaled key norm, rounded up
    stats[h] = st;
}

hipError_t launch_pooled_stats(const float *qc, const float *kc, int64_t n_blk, int heads, void *slots,
                               HeadStats *stats, hipStream_t stream)
{
    const int64_t tiles = pooled_tiles_padded(n_blk);
    if (tiles > 0x7fffffffLL || heads > 65535) return hipErrorInvalidValue;
    const int n_words = heads * 3 * kStatSlots;
    // a kernel rather than a memset: callers may capture this stream into a graph
    hipLaunchKernelGGL(clear_words_kernel, dim3((n_words + 255) / 256), dim3(256), 0, stream,
                       static_cast<unsigned *>(slots), n_words);
    hipLaunchKernelGGL(pooled_stats_kernel, dim3(static_cast<unsigned>(tiles), heads), dim3(256), 0, stream, qc, kc,
                       n_blk, static_cast<unsigned *>(slots));
    hipLaunchKernelGGL(head_stats_kernel, dim3(heads), dim3(64), 0, stream, static_cast<const unsigned *>(slots), stats);
    return hipGetLastError();
}

hipError_t launch_split(const float *qc, const float *kc, const float *vc, void *qs_hi, void *qs_lo,
                        void *ks_hi, void *ks_lo, void *vt_hi, void *vt_lo, void *q_f16, void *k_f16,
                        const HeadStats *stats, int64_t n_blk, int heads, hipStream_t stream)
{
    const int64_t tiles = pooled_tiles_padded(n_blk);
    if (tiles > 0x7fffffffLL || heads > 65535) return hipErrorInvalidValue;
    if ((q_f16 != nullptr || k_f16 != nullptr) && stats == nullptr) return hipErrorInvalidValue;
    hipLaunchKernelGGL(split_kernel, dim3(static_cast<unsigned>(tiles), heads), dim3(256), 0, stream,
                       qc, kc, vc, static_cast<bf16_t *>(qs_hi), static_cast<bf16_t *>(qs_lo),
                       static_cast<bf16_t *>(ks_hi), static_cast<bf16_t *>(ks_lo),
                       static_cast<bf16_t *>(vt_hi), static_cast<bf16_t *>(vt_lo),
                       static_cast<_Float16 *>(q_f16), static_cast<_Float16 *>(k_f16), n_blk, tiles, stats);
    return hipGetLastError();
}

}  // namespace s3r
