// Pooled fp32 tensors -> bf16 operand tiles for the compression-branch kernel.
// Each fp32 value x is written as hi = bf16(x) and lo = bf16(x - hi), so that products of
// hi/lo pairs recover fp32-level accuracy for S_guide (eq. 4), whose ordering decides TopK.
// Tiny: touches 3 * heads * n_blk * 64 floats once.  Optionally also leaves, per head, the largest
// squared L2 norm of a pooled key (as the maximum of kKeyNormSlots partial maxima): the filter sweep
// of TopK, which computes scores from the hi parts alone, turns it into an error bound (compress.hip).
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
                                                    int64_t n_blk, int64_t tiles_padded,
                                                    unsigned *__restrict__ kmax2)
{
    __shared__ float vsf[32][65];
    __shared__ float wave_max[4];
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
    load8(qc);
    split8();
    *reinterpret_cast<bf16x8 *>(qs_hi + tile_base + dst) = hi;
    *reinterpret_cast<bf16x8 *>(qs_lo + tile_base + dst) = lo;
    load8(kc);
    split8();
    *reinterpret_cast<bf16x8 *>(ks_hi + tile_base + dst) = hi;
    *reinterpret_cast<bf16x8 *>(ks_lo + tile_base + dst) = lo;
    if (kmax2 != nullptr) {
        // squared norm of each key row (8 threads per row), largest of the tile, one atomic per workgroup;
        // non-negative floats order like their bit patterns, and a maximum does not depend on the order
        // of the atomics
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) ss = fmaf(f[i], f[i], ss);
        ss += __shfl_xor(ss, 1, 64);
        ss += __shfl_xor(ss, 2, 64);
        ss += __shfl_xor(ss, 4, 64);
        ss = fmaxf(ss, __shfl_xor(ss, 8, 64));
        ss = fmaxf(ss, __shfl_xor(ss, 16, 64));
        ss = fmaxf(ss, __shfl_xor(ss, 32, 64));
        if ((tid & 63) == 0) wave_max[tid >> 6] = ss;
    }
    load8(vc);
#pragma unroll
    for (int i = 0; i < 8; ++i) vsf[r][c * 8 + i] = f[i];
    __syncthreads();
    if (kmax2 != nullptr && tid == 0)  // 64 words per head: atomics on one address would queue up
        atomicMax(kmax2 + h * kKeyNormSlots + (tile % kKeyNormSlots),
                  __float_as_uint(fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]))));
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

hipError_t launch_split(const float *qc, const float *kc, const float *vc, void *qs_hi, void *qs_lo,
                        void *ks_hi, void *ks_lo, void *vt_hi, void *vt_lo, int64_t n_blk,
                        int heads, float *kmax2, hipStream_t stream)
{
    const int64_t tiles = pooled_tiles_padded(n_blk);
    if (tiles > 0x7fffffffLL || heads > 65535) return hipErrorInvalidValue;
    if (kmax2 != nullptr)  // a kernel rather than a memset: callers may capture this stream into a graph
        hipLaunchKernelGGL(clear_words_kernel, dim3((heads * kKeyNormSlots + 255) / 256), dim3(256), 0, stream,
                           reinterpret_cast<unsigned *>(kmax2), heads * kKeyNormSlots);
    hipLaunchKernelGGL(split_kernel, dim3(static_cast<unsigned>(tiles), heads), dim3(256), 0, stream,
                       qc, kc, vc, static_cast<bf16_t *>(qs_hi), static_cast<bf16_t *>(qs_lo),
                       static_cast<bf16_t *>(ks_hi), static_cast<bf16_t *>(ks_lo),
                       static_cast<bf16_t *>(vt_hi), static_cast<bf16_t *>(vt_lo), n_blk, tiles,
                       reinterpret_cast<unsigned *>(kmax2));
    return hipGetLastError();
}

}  // namespace s3r
