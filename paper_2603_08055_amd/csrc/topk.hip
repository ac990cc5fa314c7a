// TopKSelect (Sec. 3.2 "Selection Branch"): for every (head, query block) row of S_guide, the
// indices of its k largest entries, equal scores resolved towards the smaller index, written in
// ascending index order.  Integer output, deterministic (no result depends on atomic ordering).
//
// One 256-thread workgroup per row.  Fast path (k <= 256): the k-th largest of the 256 per-thread
// maxima is a lower bound of the row's k-th largest value, so a second sweep (served by L2 / MALL)
// keeps only the few entries at or above it; exact ranks are then resolved among those candidates
// in LDS.  Rows that defeat the bound (long runs of equal values, adversarial layouts) or k > 256
// take an exact bitwise threshold search plus an ordered compaction.  HBM-bound: one read of S.
#include "s3r_device.h"
#include "s3r_kernels.h"

namespace s3r {

constexpr int kTopkThreads = 256;
constexpr int kTopkCap = 1024;  // candidate slots of the fast path

// Monotone map float -> uint32 (larger float <=> larger key); -0.0 is folded onto +0.0 first so
// that equal scores compare equal.
__device__ __forceinline__ uint32_t order_key(float x)
{
    x += 0.f;
    const uint32_t b = __float_as_uint(x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

__device__ __forceinline__ int block_sum(int v, int *scratch /*[4]*/)
{
    // sum over the 256 threads; every thread gets the result
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    return scratch[0] + scratch[1] + scratch[2] + scratch[3];
}

__global__ __launch_bounds__(kTopkThreads) void topk_kernel(const float *__restrict__ s_guide,
                                                             int64_t ld_s, int32_t *__restrict__ idx,
                                                             int n_blk, int k)
{
    __shared__ uint32_t tmax[kTopkThreads];
    __shared__ uint32_t cand_key[kTopkCap];
    __shared__ int32_t cand_idx[kTopkCap];
    __shared__ uint8_t cand_sel[kTopkCap];
    __shared__ int n_cand;
    __shared__ uint32_t thr_sh;
    __shared__ int scratch[4];
    __shared__ int wave_cnt[2][4];

    const int tid = threadIdx.x;
    const float *row = s_guide + static_cast<int64_t>(blockIdx.x) * ld_s;
    int32_t *out = idx + static_cast<int64_t>(blockIdx.x) * k;

    bool slow = k > kTopkThreads;
    if (!slow) {
        uint32_t mx = 0u;
        for (int j = tid; j < n_blk; j += kTopkThreads) {
            const uint32_t key = order_key(row[j]);
            mx = key > mx ? key : mx;
        }
        tmax[tid] = mx;
        if (tid == 0) n_cand = 0;
        __syncthreads();
        int gt = 0, ge = 0;
        for (int t = 0; t < kTopkThreads; ++t) {
            const uint32_t o = tmax[t];
            gt += o > mx;
            ge += o >= mx;
        }
        if (gt < k && ge >= k) thr_sh = mx;  // the k-th largest per-thread maximum (all writers agree)
        __syncthreads();
        const uint32_t thr = thr_sh;
        for (int j = tid; j < n_blk; j += kTopkThreads) {
            const uint32_t key = order_key(row[j]);
            if (key >= thr) {
                const int pos = atomicAdd(&n_cand, 1);
                if (pos < kTopkCap) { cand_key[pos] = key; cand_idx[pos] = j; }
            }
        }
        __syncthreads();
        const int nc = n_cand;
        if (nc > kTopkCap) {
            slow = true;  // uniform: every thread reads the same n_cand
        } else {
            // exact rank among the candidates: larger score first, then smaller index
            for (int c = tid; c < nc; c += kTopkThreads) {
                const uint32_t key = cand_key[c];
                const int32_t j = cand_idx[c];
                int rank = 0;
                for (int o = 0; o < nc; ++o) {
                    const uint32_t ok = cand_key[o];
                    rank += (ok > key) || (ok == key && cand_idx[o] < j);
                }
                cand_sel[c] = rank < k;
            }
            __syncthreads();
            // ascending index order: position = number of selected candidates with a smaller index
            for (int c = tid; c < nc; c += kTopkThreads) {
                if (!cand_sel[c]) continue;
                const int32_t j = cand_idx[c];
                int pos = 0;
                for (int o = 0; o < nc; ++o) pos += cand_sel[o] && cand_idx[o] < j;
                out[pos] = j;
            }
            return;
        }
    }

    // Exact path: T = k-th largest key by a bitwise search, then ordered compaction.
    uint32_t T = 0u;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t trial = T | (1u << bit);
        int cnt = 0;
        for (int j = tid; j < n_blk; j += kTopkThreads) cnt += order_key(row[j]) >= trial;
        if (block_sum(cnt, scratch) >= k) T = trial;
    }
    int cnt_gt = 0;
    for (int j = tid; j < n_blk; j += kTopkThreads) cnt_gt += order_key(row[j]) > T;
    const int need_eq = k - block_sum(cnt_gt, scratch);  // ties at T to keep, smallest indices first

    const int lane = tid & 63, wave = tid >> 6;
    int base_sel = 0, base_eq = 0;
    for (int j0 = 0; j0 < n_blk; j0 += kTopkThreads) {
        const int j = j0 + tid;
        uint32_t key = 0u;
        const bool in = j < n_blk;
        if (in) key = order_key(row[j]);
        const bool eq = in && key == T, gtr = in && key > T;
        const unsigned long long eq_mask = __ballot(eq);
        const unsigned long long below = (1ull << lane) - 1ull;
        if (lane == 0) wave_cnt[0][wave] = __popcll(eq_mask);
        __syncthreads();
        int eq_before = base_eq + __popcll(eq_mask & below);
        int eq_total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w < wave) eq_before += wave_cnt[0][w];
            eq_total += wave_cnt[0][w];
        }
        const bool sel = gtr || (eq && eq_before < need_eq);
        const unsigned long long sel_mask = __ballot(sel);
        if (lane == 0) wave_cnt[1][wave] = __popcll(sel_mask);
        __syncthreads();
        int pos = base_sel + __popcll(sel_mask & below);
        int sel_total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w < wave) pos += wave_cnt[1][w];
            sel_total += wave_cnt[1][w];
        }
        if (sel) out[pos] = j;
        base_sel += sel_total;
        base_eq += eq_total;
        __syncthreads();
    }
}

hipError_t launch_topk(const float *s_guide, int64_t ld_s, int32_t *idx, int64_t n_blk,
                       int64_t n_rows, int k, hipStream_t stream)
{
    if (n_rows > 0x7fffffffLL || n_blk > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(topk_kernel, dim3(static_cast<unsigned>(n_rows)), dim3(kTopkThreads), 0, stream,
                       s_guide, ld_s, idx, static_cast<int>(n_blk), k);
    return hipGetLastError();
}

}  // namespace s3r
