// Selection attention + merge (Sec. 3.2 eq. 6, Alg. 2; eqs. 5, 7, 8) and dense attention (eq. 2
// form), generic version: one thread per query row, fp32 FMA arithmetic, key/value chunks of 32
// tokens staged through LDS.  Serves fp32 problems and block sizes the MFMA kernels do not cover.
// Not tuned for throughput; the bf16 MFMA kernels are the fast path.
#include "s3r_device.h"
#include "s3r_kernels.h"

namespace s3r {

constexpr int kChunk = 32;  // keys staged per step

// grid: one workgroup per (query block i, head h), head fastest; blockDim = max(64, block).
// idx == nullptr: attend to every block (dense attention).
template <typename T>
__global__ void select_generic_kernel(const T *__restrict__ q, const T *__restrict__ k,
                                      const T *__restrict__ v, const int32_t *__restrict__ idx,
                                      const float *__restrict__ o_comp, const T *__restrict__ gate,
                                      T *__restrict__ out, T *__restrict__ o_sel, float *__restrict__ lse,
                                      int64_t n_tok, int64_t n_qblk, int64_t n_keys, int heads, int block,
                                      int kk, float scale_log2, TokenMap qmap, TokenMap kmap,
                                      int64_t lse_stride, const int32_t *__restrict__ blk_len, SelectExtras x)
{
    __shared__ __attribute__((aligned(16))) float ks[kChunk][64];
    __shared__ __attribute__((aligned(16))) float vs[kChunk][64];

    const int64_t bid = blockIdx.x;
    const int h = static_cast<int>(bid % heads);
    const int64_t i = bid / heads;
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int64_t t = i * block + tid;
    // blk_len (spatial windows) describes the key blocks; it applies to the query blocks too when
    // the queries are the same sequence (selection: idx given)
    const bool active = tid < block && t < n_tok && (blk_len == nullptr || idx == nullptr || tid < blk_len[i]) &&
                        (idx != nullptr || x.q_blk_len == nullptr || t % x.q_block < x.q_blk_len[t / x.q_block]);
    const int64_t trow = qmap.row(active ? t : 0);  // the caller's row of this query
    const int64_t n_kblk = (n_keys + block - 1) / block;
    // layout of k and v: that of q unless strides of their own are given (dense attention over pooled tensors)
    const int64_t k_rs = x.k_row_stride != 0 ? x.k_row_stride : x.in.tok != 0 ? x.in.tok : static_cast<int64_t>(heads) * 64;
    const int64_t k_hs = x.k_row_stride != 0 ? x.k_head_stride : x.in.tok != 0 ? x.in.head : 64;

    float qr[64], acc[64];
#pragma unroll
    for (int c = 0; c < 64; ++c) {
        qr[c] = active ? to_float(q[x.in.at(trow, h, heads) + c]) : 0.f;
        acc[c] = 0.f;
    }
    float m_run = -1e30f, l_run = 0.f;

    const int64_t n_sel = (idx != nullptr) ? kk : n_kblk;
    const int32_t *sel = (idx != nullptr) ? idx + (static_cast<int64_t>(h) * n_qblk + i) * kk : nullptr;

    for (int64_t a = 0; a < n_sel; ++a) {
        int64_t j = (sel != nullptr) ? sel[a] : a;
        j = j < 0 ? 0 : (j >= n_kblk ? n_kblk - 1 : j);   // a caller's list is not trusted with the address arithmetic
        const int64_t u0 = j * block;
        const int len = (blk_len != nullptr) ? blk_len[j] : static_cast<int>((n_keys - u0 < block) ? (n_keys - u0) : block);
        for (int c0 = 0; c0 < len; c0 += kChunk) {
            const int nk = (len - c0 < kChunk) ? (len - c0) : kChunk;
            __syncthreads();
            for (int e = tid; e < nk * 64; e += nthr) {
                const int r = e >> 6, c = e & 63;
                const int64_t src = kmap.row(u0 + c0 + r) * k_rs + h * k_hs + c;
                ks[r][c] = to_float(k[src]);
                vs[r][c] = to_float(v[src]);
            }
            __syncthreads();
            float s[kChunk];
            float mx = -INFINITY;
#pragma unroll
            for (int r = 0; r < kChunk; ++r) {
                float d = 0.f;
                if (r < nk) {
#pragma unroll
                    for (int c = 0; c < 64; c += 4) {
                        const floatx4 kv = *reinterpret_cast<const floatx4 *>(&ks[r][c]);
                        d += qr[c] * kv[0] + qr[c + 1] * kv[1] + qr[c + 2] * kv[2] + qr[c + 3] * kv[3];
                    }
                    d *= scale_log2;
                    mx = fmaxf(mx, d);
                } else {
                    d = -INFINITY;
                }
                s[r] = d;
            }
            const float m_new = fmaxf(m_run, mx);
            const float alpha = fast_exp2(m_run - m_new);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int c = 0; c < 64; ++c) acc[c] *= alpha;
#pragma unroll
            for (int r = 0; r < kChunk; ++r) {
                if (r < nk) {
                    const float p = fast_exp2(s[r] - m_new);
                    l_run += p;
#pragma unroll
                    for (int c = 0; c < 64; c += 4) {
                        const floatx4 vv = *reinterpret_cast<const floatx4 *>(&vs[r][c]);
                        acc[c] += p * vv[0];
                        acc[c + 1] += p * vv[1];
                        acc[c + 2] += p * vv[2];
                        acc[c + 3] += p * vv[3];
                    }
                }
            }
        }
    }

    if (!active) return;
    const float inv = 1.f / l_run;
    const int64_t o = (trow * heads + h) * 64;
    if (lse != nullptr) lse[static_cast<int64_t>(h) * lse_stride + trow] = (m_run + __builtin_log2f(l_run)) * kLn2;
    const float *oc = (o_comp != nullptr) ? o_comp + (static_cast<int64_t>(h) * n_qblk + i) * 64 : nullptr;
    if (x.o_comp_tok != nullptr) oc = x.o_comp_tok + (t * heads + h) * 64;  // this query's own compressed output
    if (x.out_f32 != nullptr) {  // fp32, by query slot
#pragma unroll
        for (int c = 0; c < 64; ++c) x.out_f32[(t * heads + h) * 64 + c] = acc[c] * inv;
        return;
    }
#pragma unroll
    for (int c = 0; c < 64; ++c) {
        const float os = acc[c] * inv;
        if (o_sel != nullptr) o_sel[o + c] = from_float<T>(os);
        float r = os;
        if (oc != nullptr) {
            float gt = 0.5f;
            if (gate != nullptr) gt = 1.f / (1.f + __expf(-to_float(gate[o + c])));
            r = gt * oc[c] + (1.f - gt) * os;
        }
        out[o + c] = from_float<T>(r);
    }
}

hipError_t launch_select_generic(const SelectArgs &a, hipStream_t stream)
{
    const int64_t n_qblk = (a.n_tok + a.block - 1) / a.block;
    const int64_t grid = n_qblk * a.heads;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    if ((a.qmap.period != 0 && a.n_tok > 0x7fffffffLL) || (a.kmap.period != 0 && a.n_keys > 0x7fffffffLL))
        return hipErrorInvalidValue;
    if (a.idx != nullptr && a.n_keys != a.n_tok) return hipErrorInvalidValue;
    const int threads = a.block < 64 ? 64 : a.block;
    const float scale_log2 = a.scale * kLog2e;
    if (a.is_bf16) {
        hipLaunchKernelGGL(select_generic_kernel<bf16_t>, dim3(static_cast<unsigned>(grid)), dim3(threads),
                           0, stream, static_cast<const bf16_t *>(a.q), static_cast<const bf16_t *>(a.k),
                           static_cast<const bf16_t *>(a.v), a.idx, a.o_comp,
                           static_cast<const bf16_t *>(a.gate), static_cast<bf16_t *>(a.out),
                           static_cast<bf16_t *>(a.o_sel), a.lse, a.n_tok, n_qblk, a.n_keys, a.heads,
                           a.block, a.kk, scale_log2, a.qmap, a.kmap, a.lse_stride, a.blk_len, a.x);
    } else {
        hipLaunchKernelGGL(select_generic_kernel<float>, dim3(static_cast<unsigned>(grid)), dim3(threads),
                           0, stream, static_cast<const float *>(a.q), static_cast<const float *>(a.k),
                           static_cast<const float *>(a.v), a.idx, a.o_comp,
                           static_cast<const float *>(a.gate), static_cast<float *>(a.out),
                           static_cast<float *>(a.o_sel), a.lse, a.n_tok, n_qblk, a.n_keys, a.heads, a.block,
                           a.kk, scale_log2, a.qmap, a.kmap, a.lse_stride, a.blk_len, a.x);
    }
    return hipGetLastError();
}

}  // namespace s3r
