// Selection attention + merge (Sec. 3.2 eq. 6, supplementary Alg. 2; eqs. 5, 7, 8) and dense
// attention (eq. 2 form) on bf16 MFMA for gfx950.
//
// Layout of the work: a wave owns 32 query rows and keeps their Q operands in registers for the
// whole kernel.  Per selected key block it computes the TRANSPOSED score tile S^T[key][query] =
// K_j Q^T with v_mfma_f32_32x32x16_bf16 (A = K tile from LDS, B = Q^T registers), so a lane holds
// keys of ONE query: the online-softmax row max / row sum are in-lane reductions plus one
// exchange with the lane 32 positions away, and the probabilities already sit in the register
// order of the B operand of the next MFMA, O^T = V^T P^T (A = V^T tile from LDS).
// K and V tiles come from the operand-order copies written by the pooling kernel: each tile is one
// contiguous run in HBM, copied to LDS as is (double buffered), read back with one conflict-free
// ds_read_b128 per MFMA operand.
#include "s3r_device.h"
#include "s3r_kernels.h"
#include <cstdlib>

namespace s3r {

// B      : tokens per key block (64 or 128) = rows of one staged K / V tile
// NWAVES : waves per workgroup; the workgroup covers 32 * NWAVES consecutive query rows starting
//          at row (blockIdx / heads) * 32 * NWAVES.  For selection NWAVES = B / 32 (one query block).
// DENSE  : iterate over every key block instead of an index list
template <int B, int NWAVES, bool DENSE>
__global__ __launch_bounds__(NWAVES * 64) void select_mfma_kernel(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ kb, const bf16_t *__restrict__ vb,
    const int32_t *__restrict__ idx, const float *__restrict__ o_comp, const bf16_t *__restrict__ gate,
    bf16_t *__restrict__ out, bf16_t *__restrict__ o_sel, float *__restrict__ lse, int64_t n_tok,
    int64_t n_blk, int heads, int kk, float scale_log2, int64_t group_offset, int64_t n_groups, int map_mode)
{
    constexpr int NT = B / 32;             // 32-key MFMA tiles per key block
    constexpr int TILE = B * 64;           // elements of one K (or V) tile
    constexpr int NTHR = NWAVES * 64;
    constexpr int CHUNKS = TILE / 8 / NTHR;  // 16-byte chunks per thread per array
    static_assert(TILE / 8 % NTHR == 0, "tile must split evenly over the workgroup");
    __shared__ __attribute__((aligned(16))) bf16_t lds[2][2][TILE];  // [stage][K, V]

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5;
    const int64_t bid = blockIdx.x;
    int h;
    int64_t qgroup;
    if (map_mode == 0) {
        h = static_cast<int>(bid % heads);
        qgroup = bid / heads + group_offset;        // query block (selection) / row group
    } else if (map_mode == 1) {
        const int64_t total = n_groups * heads, per = (total + 7) / 8;
        const int64_t id = (bid % 8) * per + bid / 8;
        if (id >= total) return;
        h = static_cast<int>(id / n_groups);
        qgroup = id % n_groups + group_offset;
    } else {
        const int64_t per = (n_groups + 7) / 8;
        h = static_cast<int>(bid / (8 * per));
        const int64_t r = bid % (8 * per);
        const int64_t g_in = (r % 8) * per + r / 8;
        if (g_in >= n_groups) return;
        qgroup = g_in + group_offset;
    }
    const int64_t t = qgroup * (32 * NWAVES) + wave * 32 + (lane & 31);
    const bool row_valid = t < n_tok;

    bf16x8 qb[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        if (row_valid) {
            qb[s] = *reinterpret_cast<const bf16x8 *>(q + (t * heads + h) * 64 + 16 * s + 8 * g);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) qb[s][i] = static_cast<bf16_t>(0.f);
        }
    }

    const int64_t n_sel = DENSE ? n_blk : kk;
    const int32_t *sel = DENSE ? nullptr : idx + (static_cast<int64_t>(h) * n_blk + qgroup) * kk;
    const bf16_t *kb_h = kb + static_cast<int64_t>(h) * n_blk * TILE;
    const bf16_t *vb_h = vb + static_cast<int64_t>(h) * n_blk * TILE;
    const int tail_len = static_cast<int>(n_tok - (n_blk - 1) * B);  // valid keys of the last block

    bf16x8 pf[2][CHUNKS];
    auto fetch = [&](int64_t j) {
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            pf[0][c] = *reinterpret_cast<const bf16x8 *>(kb_h + j * TILE + (tid + c * NTHR) * 8);
            pf[1][c] = *reinterpret_cast<const bf16x8 *>(vb_h + j * TILE + (tid + c * NTHR) * 8);
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            *reinterpret_cast<bf16x8 *>(&lds[buf][0][(tid + c * NTHR) * 8]) = pf[0][c];
            *reinterpret_cast<bf16x8 *>(&lds[buf][1][(tid + c * NTHR) * 8]) = pf[1][c];
        }
    };

    floatx16 oacc[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
    float m_run = -1e30f, l_run = 0.f;

    int64_t j_cur = DENSE ? 0 : sel[0];
    fetch(j_cur);
    stash(0);
    __syncthreads();

    for (int64_t a = 0; a < n_sel; ++a) {
        const int cur = static_cast<int>(a & 1);
        int64_t j_next = 0;
        if (a + 1 < n_sel) {
            j_next = DENSE ? a + 1 : sel[a + 1];
            fetch(j_next);
        }

        floatx16 sacc[NT];
#pragma unroll
        for (int mt = 0; mt < NT; ++mt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[mt][r] = 0.f;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const bf16x8 ka = *reinterpret_cast<const bf16x8 *>(&lds[cur][0][((mt * 4 + s) * 64 + lane) * 8]);
                sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qb[s], sacc[mt], 0, 0, 0);
            }
        }
        if (j_cur == n_blk - 1 && tail_len < B) {  // keys past the end of the sequence do not exist
#pragma unroll
            for (int mt = 0; mt < NT; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (mt * 32 + acc_row(lane, r) >= tail_len) sacc[mt][r] = -INFINITY;
        }
        float mx = sacc[0][0];
#pragma unroll
        for (int mt = 0; mt < NT; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[mt][r]);
        mx = fmaxf(mx, other_half(mx));
        const float m_new = fmaxf(m_run, mx * scale_log2);
        const float alpha = fast_exp2(m_run - m_new);
        m_run = m_new;
        float lsum = 0.f;
#pragma unroll
        for (int mt = 0; mt < NT; ++mt)
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
#pragma unroll
        for (int u = 0; u < 2 * NT; ++u) {
            const int mt = u >> 1, w = u & 1;
            bf16x8 pb;
#pragma unroll
            for (int i = 0; i < 8; ++i) pb[i] = static_cast<bf16_t>(sacc[mt][8 * w + i]);
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                const bf16x8 va = *reinterpret_cast<const bf16x8 *>(&lds[cur][1][((u * 2 + dt) * 64 + lane) * 8]);
                oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb, oacc[dt], 0, 0, 0);
            }
        }

        if (a + 1 < n_sel) stash(cur ^ 1);
        j_cur = j_next;
        __syncthreads();
    }

    if (!row_valid) return;
    const float l_tot = l_run + other_half(l_run);
    const float inv = 1.f / l_tot;
    if (lse != nullptr && g == 0) lse[static_cast<int64_t>(h) * n_tok + t] = (m_run + __builtin_log2f(l_tot)) * kLn2;
    const int64_t o = (t * heads + h) * 64;
    const float *oc = (o_comp != nullptr) ? o_comp + (static_cast<int64_t>(h) * n_blk + t / B) * 64 : nullptr;
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const int d0 = 32 * dt + 8 * r4 + 4 * g;
            float os[4], res[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) res[i] = os[i] = oacc[dt][4 * r4 + i] * inv;
            if (oc != nullptr) {
                const floatx4 c4 = *reinterpret_cast<const floatx4 *>(oc + d0);
                float gt[4] = {0.5f, 0.5f, 0.5f, 0.5f};
                if (gate != nullptr) {
                    const bf16x4 gl = *reinterpret_cast<const bf16x4 *>(gate + o + d0);
#pragma unroll
                    for (int i = 0; i < 4; ++i) gt[i] = 1.f / (1.f + __expf(-static_cast<float>(gl[i])));
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) res[i] = gt[i] * c4[i] + (1.f - gt[i]) * os[i];
            }
            bf16x4 ro;
#pragma unroll
            for (int i = 0; i < 4; ++i) ro[i] = static_cast<bf16_t>(res[i]);
            *reinterpret_cast<bf16x4 *>(out + o + d0) = ro;
            if (o_sel != nullptr) {
#pragma unroll
                for (int i = 0; i < 4; ++i) ro[i] = static_cast<bf16_t>(os[i]);
                *reinterpret_cast<bf16x4 *>(o_sel + o + d0) = ro;
            }
        }
}

template <int B, int NWAVES, bool DENSE>
static hipError_t run_select(const SelectArgs &a, hipStream_t stream)
{
    const int64_t rows_per_wg = 32 * NWAVES;
    const int64_t groups = DENSE ? (a.n_tok + rows_per_wg - 1) / rows_per_wg : a.n_blk;
    // Dense attention is quadratic: keep each launch to roughly 2e14 FLOP (a fraction of a second)
    // so that no single kernel occupies the GPU for seconds.
    int64_t per_launch = groups;
    if (DENSE) {
        const double flops_per_group = 4.0 * 64.0 * rows_per_wg * static_cast<double>(a.n_tok) * a.heads;
        per_launch = static_cast<int64_t>(2e14 / flops_per_group);
        if (per_launch < 1) per_launch = 1;
    }
    if ((per_launch + 8) * a.heads > 0x7fffffffLL) return hipErrorInvalidValue;
    const char *mm = getenv("S3R_SELECT_MAP");
    const int map_mode = mm ? atoi(mm) : 0;
    for (int64_t g0 = 0; g0 < groups; g0 += per_launch) {
        const int64_t ng = (groups - g0 < per_launch) ? groups - g0 : per_launch;
        int64_t grid = ng * a.heads;
        if (map_mode == 1) grid = (grid + 7) / 8 * 8;
        if (map_mode == 2) grid = (ng + 7) / 8 * 8 * a.heads;
        hipLaunchKernelGGL((select_mfma_kernel<B, NWAVES, DENSE>), dim3(static_cast<unsigned>(grid)),
                           dim3(NWAVES * 64), 0, stream, static_cast<const bf16_t *>(a.q),
                           static_cast<const bf16_t *>(a.kb), static_cast<const bf16_t *>(a.vb), a.idx,
                           a.o_comp, static_cast<const bf16_t *>(a.gate), static_cast<bf16_t *>(a.out),
                           static_cast<bf16_t *>(a.o_sel), a.lse, a.n_tok, a.n_blk, a.heads, a.kk,
                           a.scale * kLog2e, g0, ng, map_mode);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_select_mfma(const SelectArgs &a, hipStream_t stream)
{
    if (!a.is_bf16 || a.kb == nullptr || a.vb == nullptr) return hipErrorInvalidValue;
    if (a.idx == nullptr) {
        if (a.block != 64) return hipErrorInvalidValue;
        return run_select<64, 8, true>(a, stream);
    }
    if (a.block == 64) return run_select<64, 2, false>(a, stream);
    if (a.block == 128) return run_select<128, 4, false>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace s3r
