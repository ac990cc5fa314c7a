// Selection attention + merge (Sec. 3.2 eq. 6, supplementary Alg. 2; eqs. 5, 7, 8) and dense
// attention (eq. 2 form) on bf16 MFMA for gfx950.
//
// Layout of the work: a wave owns 32 query rows and keeps their Q operands in registers for the
// whole item.  Per selected key block it computes the TRANSPOSED score tile S^T[key][query] =
// K_j Q^T with v_mfma_f32_32x32x16_bf16 (A = K tile from LDS, B = Q^T registers), so a lane holds
// keys of ONE query: the online-softmax row max / row sum are in-lane reductions plus one
// exchange with the lane 32 positions away, and the probabilities already sit in the register
// order of the B operand of the next MFMA, O^T = V^T P^T (A = V^T tile from LDS).
// K and V tiles come from the operand-order copies written by the pooling kernel: each tile is one
// contiguous run in HBM, copied to LDS as is, read back with one conflict-free ds_read_b128 per
// MFMA operand.
//
// The gather of 16 KiB tiles is latency-bound unless several tiles per workgroup are in flight, so
// tiles travel HBM -> registers -> LDS through a ring of NPF register sets: while tile a is being
// multiplied out of LDS, tiles a+1 .. a+NPF are in flight (the register file, 512 KiB per CU, is
// the deep buffer; LDS holds two tiles).
// The running row maximum is only raised when a tile exceeds it by more than kRescaleSlack (in
// log2 units), so the rescale of the output accumulators is skipped for almost every tile;
// probabilities then range up to 2^kRescaleSlack, which fp32 sums and bf16 operands carry exactly
// as well as values below 1, and the final normalisation uses the same maximum, so the result is
// the plain softmax.
#include "s3r_device.h"
#include "s3r_kernels.h"

#include <cstdlib>

namespace s3r {

constexpr float kRescaleSlack = 8.0f;

__device__ __forceinline__ float max_with_other_half(float x)
{
    // v_permlane32_swap exchanges the two half-waves: one VALU instruction, no LDS traffic
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

__device__ __forceinline__ float sum_with_other_half(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// B      : tokens per key block (64 or 128) = rows of one staged K / V tile
// NWAVES : waves per workgroup; an item covers 32 * NWAVES consecutive query rows.  For selection
//          NWAVES = B / 32 (one query block per item).
// DENSE  : iterate over every key block instead of an index list
// NPF    : register sets of the tile ring (tiles in flight per workgroup)
template <int B, int NWAVES, bool DENSE, int NPF>
__global__ __launch_bounds__(NWAVES * 64, 2) void select_mfma_kernel(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ kb, const bf16_t *__restrict__ vb,
    const int32_t *__restrict__ idx, const float *__restrict__ o_comp, const bf16_t *__restrict__ gate,
    bf16_t *__restrict__ out, bf16_t *__restrict__ o_sel, float *__restrict__ lse, int64_t n_tok,
    int64_t n_blk, int heads, int kk, float scale_log2, int64_t group_offset, int64_t n_groups, int map_mode)
{
    constexpr int NT = B / 32;               // 32-key MFMA tiles per key block
    constexpr int TILE = B * 64;             // elements of one K (or V) tile
    constexpr int NTHR = NWAVES * 64;
    constexpr int CHUNKS = TILE / 8 / NTHR;  // 16-byte chunks per thread per array
    static_assert(TILE / 8 % NTHR == 0, "tile must split evenly over the workgroup");
    __shared__ __attribute__((aligned(16))) bf16_t lds[2][2][TILE];  // [stage][K, V]

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5;
    const int64_t total_items = n_groups * heads;
    int64_t item_stride = total_items;  // one item per workgroup unless persistent
    int64_t item0;
    {
        const int64_t bid = blockIdx.x;
        if (map_mode == 0) {  // head fastest
            item0 = (bid % heads) * n_groups + bid / heads;
        } else if (map_mode == 2) {  // head-major, each XCD (workgroup id mod 8) a contiguous range
            const int64_t per = (n_groups + 7) / 8;
            const int64_t hh = bid / (8 * per), r = bid % (8 * per);
            const int64_t g_in = (r % 8) * per + r / 8;
            if (g_in >= n_groups) return;
            item0 = hh * n_groups + g_in;
        } else {  // persistent, head-major
            item0 = bid;
            item_stride = gridDim.x;
        }
    }
    const int tail_len = static_cast<int>(n_tok - (n_blk - 1) * B);  // valid keys of the last block

    for (int64_t item = item0; item < total_items; item += item_stride) {
        const int h = static_cast<int>(item / n_groups);
        const int64_t qgroup = item % n_groups + group_offset;  // query block (selection) / row group
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
        auto tile_of = [&](int64_t a) -> int64_t { return DENSE ? a : static_cast<int64_t>(sel[a]); };

        bf16x8 pf[NPF][2][CHUNKS];
        floatx16 oacc[2];
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
        float m_run = -1e30f, l_run = 0.f;

        // prologue: tiles 0 .. NPF-1 into the register ring, tile 0 on to LDS, tile NPF requested
#pragma unroll
        for (int u = 0; u < NPF; ++u) {
            if (u < n_sel) {
                const int64_t j = tile_of(u);
#pragma unroll
                for (int c = 0; c < CHUNKS; ++c) {
                    pf[u][0][c] = *reinterpret_cast<const bf16x8 *>(kb_h + j * TILE + (tid + c * NTHR) * 8);
                    pf[u][1][c] = *reinterpret_cast<const bf16x8 *>(vb_h + j * TILE + (tid + c * NTHR) * 8);
                }
            }
        }
#pragma unroll
        for (int c = 0; c < CHUNKS; ++c) {
            *reinterpret_cast<bf16x8 *>(&lds[0][0][(tid + c * NTHR) * 8]) = pf[0][0][c];
            *reinterpret_cast<bf16x8 *>(&lds[0][1][(tid + c * NTHR) * 8]) = pf[0][1][c];
        }
        __syncthreads();
        if (NPF < n_sel) {
            const int64_t j = tile_of(NPF);
#pragma unroll
            for (int c = 0; c < CHUNKS; ++c) {
                pf[0][0][c] = *reinterpret_cast<const bf16x8 *>(kb_h + j * TILE + (tid + c * NTHR) * 8);
                pf[0][1][c] = *reinterpret_cast<const bf16x8 *>(vb_h + j * TILE + (tid + c * NTHR) * 8);
            }
        }

        for (int64_t a0 = 0; a0 < n_sel; a0 += NPF) {
#pragma unroll
            for (int u = 0; u < NPF; ++u) {
                // tile a sits in LDS stage a & 1; tile a + 1 is (arriving) in register set (u + 1) % NPF
                const int64_t a = a0 + u;
                if (a >= n_sel) break;
                const int cur = static_cast<int>(a & 1);

                floatx16 sacc[NT];
#pragma unroll
                for (int mt = 0; mt < NT; ++mt) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) sacc[mt][r] = 0.f;
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        const bf16x8 ka =
                            *reinterpret_cast<const bf16x8 *>(&lds[cur][0][((mt * 4 + s) * 64 + lane) * 8]);
                        sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qb[s], sacc[mt], 0, 0, 0);
                    }
                }
                if (tail_len < B && tile_of(a) == n_blk - 1) {  // keys past the end of the sequence do not exist
                    asm volatile("" ::: "memory");                // keep this rare path a real branch
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
                const float m_tile = max_with_other_half(mx) * scale_log2;
                const bool grow = m_tile > m_run + kRescaleSlack;
                if (__any(grow)) {  // rare after the first tile: raise the maximum, rescale the accumulators
                    const float m_new = grow ? m_tile : m_run;
                    const float alpha = fast_exp2(m_run - m_new);
                    m_run = m_new;
                    l_run *= alpha;
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
                }
                float lsum = 0.f;
#pragma unroll
                for (int mt = 0; mt < NT; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        sacc[mt][r] = fast_exp2(sacc[mt][r] * scale_log2 - m_run);
                        lsum += sacc[mt][r];
                    }
                l_run += lsum;
#pragma unroll
                for (int v = 0; v < 2 * NT; ++v) {
                    const int mt = v >> 1, w = v & 1;
                    bf16x8 pb;
#pragma unroll
                    for (int i = 0; i < 8; ++i) pb[i] = static_cast<bf16_t>(sacc[mt][8 * w + i]);
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt) {
                        const bf16x8 va =
                            *reinterpret_cast<const bf16x8 *>(&lds[cur][1][((v * 2 + dt) * 64 + lane) * 8]);
                        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb, oacc[dt], 0, 0, 0);
                    }
                }

                const int nset = (u + 1) % NPF;
                if (a + 1 < n_sel) {
#pragma unroll
                    for (int c = 0; c < CHUNKS; ++c) {
                        *reinterpret_cast<bf16x8 *>(&lds[cur ^ 1][0][(tid + c * NTHR) * 8]) = pf[nset][0][c];
                        *reinterpret_cast<bf16x8 *>(&lds[cur ^ 1][1][(tid + c * NTHR) * 8]) = pf[nset][1][c];
                    }
                }
                __syncthreads();
                if (a + 1 + NPF < n_sel) {
                    const int64_t j = tile_of(a + 1 + NPF);
#pragma unroll
                    for (int c = 0; c < CHUNKS; ++c) {
                        pf[nset][0][c] = *reinterpret_cast<const bf16x8 *>(kb_h + j * TILE + (tid + c * NTHR) * 8);
                        pf[nset][1][c] = *reinterpret_cast<const bf16x8 *>(vb_h + j * TILE + (tid + c * NTHR) * 8);
                    }
                }
            }
        }

        if (row_valid) {
            const float l_tot = sum_with_other_half(l_run);
            const float inv = 1.f / l_tot;
            if (lse != nullptr && g == 0)
                lse[static_cast<int64_t>(h) * n_tok + t] = (m_run + __builtin_log2f(l_tot)) * kLn2;
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
    }
}

template <int B, int NWAVES, bool DENSE, int NPF>
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
    const int map_mode = mm ? atoi(mm) : (DENSE ? 0 : 2);
    for (int64_t g0 = 0; g0 < groups; g0 += per_launch) {
        const int64_t ng = (groups - g0 < per_launch) ? groups - g0 : per_launch;
        int64_t grid = ng * a.heads;
        if (map_mode == 2) grid = (ng + 7) / 8 * 8 * a.heads;
        if (map_mode >= 3) {
            const char *pg = getenv("S3R_SELECT_GRID");
            const int64_t want = pg ? atoll(pg) : 1024;
            if (grid > want) grid = want;
        }
        hipLaunchKernelGGL((select_mfma_kernel<B, NWAVES, DENSE, NPF>), dim3(static_cast<unsigned>(grid)),
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
    const char *pn = getenv("S3R_SELECT_NPF");
    const int npf = pn ? atoi(pn) : 2;
    if (a.idx == nullptr) {
        if (a.block != 64) return hipErrorInvalidValue;
        return run_select<64, 4, true, 1>(a, stream);
    }
    if (a.block == 64) {
        if (npf == 1) return run_select<64, 2, false, 1>(a, stream);
        if (npf == 2) return run_select<64, 2, false, 2>(a, stream);
        if (npf == 4) return run_select<64, 2, false, 4>(a, stream);
        return run_select<64, 2, false, 3>(a, stream);
    }
    if (a.block == 128) {
        if (npf == 1) return run_select<128, 4, false, 1>(a, stream);
        if (npf == 3) return run_select<128, 4, false, 3>(a, stream);
        return run_select<128, 4, false, 2>(a, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace s3r
