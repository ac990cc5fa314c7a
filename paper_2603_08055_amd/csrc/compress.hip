// Compression branch (Sec. 3.2, eqs. 3-4; supplementary Alg. 1 without its TopK part):
//   S_guide = Qc Kc^T (unscaled, written out for TopK) and Oc' = softmax(scale * S_guide) Vc,
// one pass over the pooled keys with an online softmax.
//
// gfx950 design: each wave owns 32 pooled queries and computes the TRANSPOSED score tile
// S^T[key][query] with v_mfma_f32_32x32x16_bf16 (A = pooled keys from LDS, B = pooled queries
// held in registers).  In that orientation a lane holds 16 keys of ONE query per 32-key tile, so
// row max / row sum are in-lane reductions plus one exchange with the lane 32 positions away, and
// the probabilities already sit in the register order the next MFMA (O^T = Vc^T P^T) wants.
// Scores use bf16 hi/lo operand pairs (hi*hi + hi*lo + lo*hi): about 2^-16 relative to |q||k|,
// which keeps the TopK ordering at fp32 quality at bf16 MFMA rates.
#include "s3r_device.h"
#include "s3r_kernels.h"

namespace s3r {

template <bool SPLIT_PV>
__global__ __launch_bounds__(256, 2) void compress_kernel(
    const bf16_t *__restrict__ qs_hi, const bf16_t *__restrict__ qs_lo,
    const bf16_t *__restrict__ ks_hi, const bf16_t *__restrict__ ks_lo,
    const bf16_t *__restrict__ vt_hi, const bf16_t *__restrict__ vt_lo, float *__restrict__ s_guide,
    int64_t ld_s, float *__restrict__ o_comp, int64_t n_blk, int64_t tiles_padded, float scale_log2)
{
    constexpr int NARR = SPLIT_PV ? 4 : 3;         // ks_hi, ks_lo, vt_hi [, vt_lo]
    constexpr int STAGE_ELEMS = 2 * kRowTileElems;  // 64 keys x 64 channels per array
    __shared__ __attribute__((aligned(16))) bf16_t lds[2][NARR][STAGE_ELEMS];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5;
    const int h = blockIdx.y;
    const int64_t qtile = static_cast<int64_t>(blockIdx.x) * 4 + wave;
    const int64_t qrow = qtile * 32 + (lane & 31);
    const bool wave_active = qtile * 32 < n_blk;
    const int64_t n_kt = (n_blk + 63) / 64;
    const int64_t head_tiles = static_cast<int64_t>(h) * tiles_padded;

    const bf16_t *src[NARR];
    src[0] = ks_hi + head_tiles * kRowTileElems;
    src[1] = ks_lo + head_tiles * kRowTileElems;
    src[2] = vt_hi + head_tiles * kRowTileElems;
    if constexpr (SPLIT_PV) src[3] = vt_lo + head_tiles * kRowTileElems;

    bf16x8 qhi[4], qlo[4];
    {
        const int64_t qb = (head_tiles + qtile) * kRowTileElems;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            qhi[s] = *reinterpret_cast<const bf16x8 *>(qs_hi + qb + (s * 64 + lane) * 8);
            qlo[s] = *reinterpret_cast<const bf16x8 *>(qs_lo + qb + (s * 64 + lane) * 8);
        }
    }

    bf16x8 pf[NARR][2];
    auto fetch = [&](int64_t kt) {
#pragma unroll
        for (int a = 0; a < NARR; ++a)
#pragma unroll
            for (int c = 0; c < 2; ++c)
                pf[a][c] = *reinterpret_cast<const bf16x8 *>(src[a] + kt * STAGE_ELEMS + (tid + c * 256) * 8);
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int a = 0; a < NARR; ++a)
#pragma unroll
            for (int c = 0; c < 2; ++c)
                *reinterpret_cast<bf16x8 *>(&lds[buf][a][(tid + c * 256) * 8]) = pf[a][c];
    };

    floatx16 oacc[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
    float m_run = -1e30f, l_run = 0.f;

    fetch(0);
    stash(0);
    __syncthreads();

    for (int64_t kt = 0; kt < n_kt; ++kt) {
        const int cur = static_cast<int>(kt & 1);
        if (kt + 1 < n_kt) fetch(kt + 1);

        if (wave_active) {
            floatx16 sacc[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[mt][r] = 0.f;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const int off = mt * kRowTileElems + (s * 64 + lane) * 8;
                    const bf16x8 a_hi = *reinterpret_cast<const bf16x8 *>(&lds[cur][0][off]);
                    const bf16x8 a_lo = *reinterpret_cast<const bf16x8 *>(&lds[cur][1][off]);
                    sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo, qhi[s], sacc[mt], 0, 0, 0);
                    sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, qlo[s], sacc[mt], 0, 0, 0);
                    sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, qhi[s], sacc[mt], 0, 0, 0);
                }
            }
            // eq. 4: raw scores out, 4 consecutive keys of one query row per store
            if (qrow < n_blk) {
                float *srow = s_guide + (static_cast<int64_t>(h) * n_blk + qrow) * ld_s;
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const int64_t key0 = kt * 64 + mt * 32 + 8 * r4 + 4 * g;
                        if (key0 < ld_s) {
                            floatx4 o;
#pragma unroll
                            for (int i = 0; i < 4; ++i) o[i] = sacc[mt][4 * r4 + i];
                            *reinterpret_cast<floatx4 *>(srow + key0) = o;
                        }
                    }
            }
            if (kt * 64 + 64 > n_blk) {  // pooled keys past the end of the sequence do not exist
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (kt * 64 + mt * 32 + acc_row(lane, r) >= n_blk) sacc[mt][r] = -INFINITY;
            }
            // online softmax (eq. 3), base-2 exponent with the scale folded in
            float mx = sacc[0][0];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[mt][r]);
            mx = fmaxf(mx, other_half(mx));
            const float m_new = fmaxf(m_run, mx * scale_log2);
            const float alpha = fast_exp2(m_run - m_new);
            m_run = m_new;
            float lsum = 0.f;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    sacc[mt][r] = fast_exp2(sacc[mt][r] * scale_log2 - m_new);
                    lsum += sacc[mt][r];
                }
            l_run = l_run * alpha + lsum;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
            // O^T += Vc^T P^T, contraction over the 64 keys in four 16-key steps
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int mt = u >> 1, w = u & 1;
                bf16x8 p_hi, p_lo;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float p = sacc[mt][8 * w + i];
                    p_hi[i] = static_cast<bf16_t>(p);
                    if constexpr (SPLIT_PV) p_lo[i] = static_cast<bf16_t>(p - static_cast<float>(p_hi[i]));
                }
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) {
                    const int off = mt * kRowTileElems + ((w * 2 + dt) * 64 + lane) * 8;
                    const bf16x8 v_hi = *reinterpret_cast<const bf16x8 *>(&lds[cur][2][off]);
                    oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_hi, p_hi, oacc[dt], 0, 0, 0);
                    if constexpr (SPLIT_PV) {
                        const bf16x8 v_lo = *reinterpret_cast<const bf16x8 *>(&lds[cur][NARR - 1][off]);
                        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_lo, p_hi, oacc[dt], 0, 0, 0);
                        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_hi, p_lo, oacc[dt], 0, 0, 0);
                    }
                }
            }
        }
        if (kt + 1 < n_kt) stash(cur ^ 1);
        __syncthreads();
    }

    if (wave_active && qrow < n_blk) {
        const float inv = 1.f / (l_run + other_half(l_run));
        float *orow = o_comp + (static_cast<int64_t>(h) * n_blk + qrow) * 64;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                floatx4 o;
#pragma unroll
                for (int i = 0; i < 4; ++i) o[i] = oacc[dt][4 * r4 + i] * inv;
                *reinterpret_cast<floatx4 *>(orow + 32 * dt + 8 * r4 + 4 * g) = o;
            }
    }
}

hipError_t launch_compress(const void *qs_hi, const void *qs_lo, const void *ks_hi,
                           const void *ks_lo, const void *vt_hi, const void *vt_lo, float *s_guide,
                           int64_t ld_s, float *o_comp, int64_t n_blk, int heads, float scale,
                           hipStream_t stream)
{
    const int64_t tiles = pooled_tiles_padded(n_blk);
    const dim3 grid(static_cast<unsigned>(tiles / 4), heads);
    const float scale_log2 = scale * kLog2e;
    if (vt_lo != nullptr) {
        hipLaunchKernelGGL(compress_kernel<true>, grid, dim3(256), 0, stream,
                           static_cast<const bf16_t *>(qs_hi), static_cast<const bf16_t *>(qs_lo),
                           static_cast<const bf16_t *>(ks_hi), static_cast<const bf16_t *>(ks_lo),
                           static_cast<const bf16_t *>(vt_hi), static_cast<const bf16_t *>(vt_lo),
                           s_guide, ld_s, o_comp, n_blk, tiles, scale_log2);
    } else {
        hipLaunchKernelGGL(compress_kernel<false>, grid, dim3(256), 0, stream,
                           static_cast<const bf16_t *>(qs_hi), static_cast<const bf16_t *>(qs_lo),
                           static_cast<const bf16_t *>(ks_hi), static_cast<const bf16_t *>(ks_lo),
                           static_cast<const bf16_t *>(vt_hi), static_cast<const bf16_t *>(vt_lo),
                           s_guide, ld_s, o_comp, n_blk, tiles, scale_log2);
    }
    return hipGetLastError();
}

}  // namespace s3r
