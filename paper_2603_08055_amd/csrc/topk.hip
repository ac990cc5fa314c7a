// TopKSelect (Sec. 3.2 "Selection Branch"): for every (head, query block) row of S_guide, the
// indices of its k largest entries, equal scores resolved towards the smaller index, written in
// ascending index order.  Integer output, deterministic (no result depends on atomic ordering).
//
// One 256-thread workgroup per row, HBM-bound by design: S is read once.
//  * topk_reg_kernel<NV> (rows of up to 32768 entries, k <= 256): the row is loaded once into
//    registers, each wave owning a contiguous quarter.  The k-th largest of the 256 per-lane maxima
//    is a lower bound of the row's k-th largest value; entries at or above it (typically ~1.2 k of
//    them) are appended to LDS in index order with wave ballots; one wave then finds the exact k-th
//    largest candidate by a bitwise search with ballots and writes the winners, already in order.
//  * topk_stream_kernel (any row length, any k): same idea with two sweeps over global memory and
//    rank counting, plus the exact path below.
//  * exact path (rows that defeat the bound, e.g. long runs of equal values; k > 256): bitwise
//    search of the k-th largest order-preserving key over the whole row, then an ordered
//    ballot/popcount compaction.
#include "s3r_device.h"
#include "s3r_kernels.h"

namespace s3r {

constexpr int kTopkThreads = 256;
constexpr int kTopkCap = 1024;  // candidate slots of the streaming fast path

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

// Exact selection over the whole row, all 256 threads: T = k-th largest key by a bitwise search,
// then ordered compaction (entries above T, then the first ties at T in index order).
__device__ void topk_exact_path(const float *__restrict__ row, int32_t *__restrict__ out, int n_blk, int k,
                                int *scratch /*[4]*/, int (*wave_cnt)[4] /*[2][4]*/)
{
    const int tid = threadIdx.x;
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
        if (lane == 0) wave_cnt[0][wave] = __popcll(eq_mask);
        __syncthreads();
        int eq_before = base_eq + lanes_below(eq_mask);
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
        int pos = base_sel + lanes_below(sel_mask);
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

// NV = maximum row entries per lane; the four waves own equal contiguous shares of the row.
// Requires n_blk <= NV * 256 and k <= 256.
template <int NV>
__device__ __forceinline__ void topk_reg_row(const float *__restrict__ s_guide, int64_t ld_s,
                                             int32_t *__restrict__ idx, int n_blk, int k, unsigned row_id)
{
    constexpr int CAPW = 256;  // candidate slots per wave
    __shared__ uint32_t lane_max[kTopkThreads];
    __shared__ uint32_t cand_key[4][CAPW];
    __shared__ int32_t cand_idx[4][CAPW];
    __shared__ int n_w[4];
    __shared__ uint32_t thr_sh;
    __shared__ int scratch[4];
    __shared__ int wave_cnt[2][4];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const float *row = s_guide + static_cast<int64_t>(row_id) * ld_s;
    int32_t *out = idx + static_cast<int64_t>(row_id) * k;
    // equal shares: each wave owns wave_len consecutive entries (a multiple of 64, <= NV * 64)
    const int wave_len = ((n_blk + 3) / 4 + 63) / 64 * 64;
    const int wave_base = __builtin_amdgcn_readfirstlane(wave) * wave_len;
    const int wave_end = (wave_base + wave_len < n_blk) ? wave_base + wave_len : n_blk;
    const int base = wave_base + lane;
    const int leader = row_id & 3;  // the wave that does the serial parts rotates with the row

    // Entries past the end of the row are NaN: v_max ignores them and every ordered compare fails.
    float x[NV];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        if (wave_base + i * 64 + 64 <= wave_end) {  // wave-uniform: the 64 entries of this step all exist
            x[i] = row[base + i * 64];
        } else if (wave_base + i * 64 >= wave_end) {  // wave-uniform: none exists
            x[i] = __builtin_nanf("");
        } else {
            const int j = base + i * 64;
            const float v = row[j < wave_end ? j : wave_end - 1];  // clamped address, then masked
            x[i] = (j < wave_end) ? v : __builtin_nanf("");
        }
        mx = fmaxf(mx, x[i]);
    }
    lane_max[tid] = order_key(mx);
    __syncthreads();
    if (wave == leader) {
        // k-th largest of the 256 lane maxima: at least k row entries are >= it
        const uint32_t m0 = lane_max[lane], m1 = lane_max[lane + 64], m2 = lane_max[lane + 128],
                       m3 = lane_max[lane + 192];
        uint32_t T = 0u;
        for (int bit = 31; bit >= 0; --bit) {
            const uint32_t trial = T | (1u << bit);
            const int c = __popcll(__ballot(m0 >= trial)) + __popcll(__ballot(m1 >= trial)) +
                          __popcll(__ballot(m2 >= trial)) + __popcll(__ballot(m3 >= trial));
            if (c >= k) T = trial;
        }
        if (lane == 0) thr_sh = T;
    }
    __syncthreads();
    // The threshold as a float: x >= thr_f  <=>  order_key(x) >= thr (signed zeros compare equal
    // either way; the key of -inf, reached only when fewer than k lanes hold data, maps back to -inf).
    const uint32_t thr = thr_sh;
    const float thr_f = key_to_float(thr);
    int cnt = 0;
    constexpr int GRP = (NV % 4 == 0) ? 4 : 1;
#pragma unroll
    for (int i0 = 0; i0 < NV; i0 += GRP) {
        bool any = false;
#pragma unroll
        for (int i = i0; i < i0 + GRP; ++i) any = any || (x[i] >= thr_f);
        if (__ballot(any) == 0ull) continue;  // wave-uniform: most groups hold no candidate
#pragma unroll
        for (int i = i0; i < i0 + GRP; ++i) {
            const bool flag = x[i] >= thr_f;
            const unsigned long long mask = __ballot(flag);
            const int pos = cnt + lanes_below(mask);
            if (flag && pos < CAPW) {
                cand_key[wave][pos] = order_key(x[i]);
                cand_idx[wave][pos] = base + i * 64;
            }
            cnt += __popcll(mask);
        }
    }
    if (lane == 0) n_w[wave] = cnt;
    __syncthreads();
    const int n0 = n_w[0], n1 = n_w[1], n2 = n_w[2], n3 = n_w[3];
    if (n0 > CAPW || n1 > CAPW || n2 > CAPW || n3 > CAPW) {  // uniform over the workgroup
        topk_exact_path(row, out, n_blk, k, scratch, wave_cnt);
        return;
    }
    if (wave != leader) return;

    // Leader wave: exact k-th largest among the candidates (all entries >= thr, at least k of them).
    const int nws[4] = {n0, n1, n2, n3};
    uint32_t ck[4][CAPW / 64];
#pragma unroll
    for (int w = 0; w < 4; ++w)
#pragma unroll
        for (int s = 0; s < CAPW / 64; ++s) ck[w][s] = (s * 64 + lane < nws[w]) ? cand_key[w][s * 64 + lane] : 0u;
    uint32_t T = 0u;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t trial = T | (1u << bit);
        int c = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w)
#pragma unroll
            for (int s = 0; s < CAPW / 64; ++s)
                if (s * 64 < nws[w]) c += __popcll(__ballot(ck[w][s] >= trial));
        if (c >= k) T = trial;
    }
    int cnt_gt = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w)
#pragma unroll
        for (int s = 0; s < CAPW / 64; ++s)
            if (s * 64 < nws[w]) cnt_gt += __popcll(__ballot(ck[w][s] > T));
    const int need_eq = k - cnt_gt;
    int base_sel = 0, base_eq = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w)
#pragma unroll
        for (int s = 0; s < CAPW / 64; ++s) {
            if (s * 64 >= nws[w]) continue;
            const bool valid = s * 64 + lane < nws[w];
            const bool eq = valid && ck[w][s] == T, gtr = valid && ck[w][s] > T;
            const unsigned long long eq_mask = __ballot(eq);
            const bool sel = gtr || (eq && base_eq + lanes_below(eq_mask) < need_eq);
            const unsigned long long sel_mask = __ballot(sel);
            if (sel) out[base_sel + lanes_below(sel_mask)] = cand_idx[w][s * 64 + lane];
            base_sel += __popcll(sel_mask);
            base_eq += __popcll(eq_mask);
        }
}

__device__ __forceinline__ void topk_stream_row(const float *__restrict__ s_guide, int64_t ld_s,
                                                int32_t *__restrict__ idx, int n_blk, int k, unsigned row_id)
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
    const float *row = s_guide + static_cast<int64_t>(row_id) * ld_s;
    int32_t *out = idx + static_cast<int64_t>(row_id) * k;

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

    topk_exact_path(row, out, n_blk, k, scratch, wave_cnt);
}

// One workgroup per row; or, with a run flag (device word), a small grid that does nothing when the
// word is 0 and walks over all rows otherwise (the rarely needed second route of a caller that
// cannot read the word on the host: launching one workgroup per row just to return costs
// hundreds of microseconds at 10^5 rows).
template <int NV>
__global__ __launch_bounds__(kTopkThreads) void topk_reg_kernel(const float *__restrict__ s_guide, int64_t ld_s,
                                                                 int32_t *__restrict__ idx, int n_blk, int k,
                                                                 unsigned n_rows, const int *__restrict__ run_flag)
{
    if (run_flag == nullptr) {
        topk_reg_row<NV>(s_guide, ld_s, idx, n_blk, k, blockIdx.x);
        return;
    }
    if (*run_flag == 0) return;  // uniform over the grid
    for (unsigned r = blockIdx.x; r < n_rows; r += gridDim.x) {
        topk_reg_row<NV>(s_guide, ld_s, idx, n_blk, k, r);
        __syncthreads();
    }
}

__global__ __launch_bounds__(kTopkThreads) void topk_stream_kernel(const float *__restrict__ s_guide, int64_t ld_s,
                                                                    int32_t *__restrict__ idx, int n_blk, int k,
                                                                    unsigned n_rows, const int *__restrict__ run_flag)
{
    if (run_flag == nullptr) {
        topk_stream_row(s_guide, ld_s, idx, n_blk, k, blockIdx.x);
        return;
    }
    if (*run_flag == 0) return;  // uniform over the grid
    for (unsigned r = blockIdx.x; r < n_rows; r += gridDim.x) {
        topk_stream_row(s_guide, ld_s, idx, n_blk, k, r);
        __syncthreads();
    }
}

// Exact TopK among the candidates the filter sweep of the compression kernel left for a row (two
// lists per row, see compress.hip).  One wave per row.  The scores are recomputed here as plain fp32
// dot products of the pooled query and key (fused multiply-adds in a fixed order), so the result
// does not depend on how the filter computed its own copy beyond which keys became candidates.
// Ties go to the smaller index; output ascending.  Requires k <= 64 and at most 2 * cap <= 2048
// candidates (lists that were cut are read up to cap: the caller redoes such launches).
constexpr int kCandSlots = 8;  // candidates per lane (at most 2 * cap = 512 per row)
__global__ __launch_bounds__(64) void topk_candidates_kernel(const float *__restrict__ qc, const float *__restrict__ kc,
                                                            const int32_t *__restrict__ cand,
                                                            const int *__restrict__ cand_count, int cap,
                                                            int32_t *__restrict__ idx, int n_blk, int k)
{
    __shared__ int32_t ids[kCandSlots * 64];
    __shared__ float sc[kCandSlots * 64];
    __shared__ int32_t ties[kCandSlots * 64];
    __shared__ int32_t win[64];
    const int lane = threadIdx.x;
    const int64_t row = blockIdx.x;           // head * n_blk + query block
    const int64_t head = row / n_blk;
    const int c0 = cand_count[row * 2], c1 = cand_count[row * 2 + 1];
    const int n0 = c0 < cap ? c0 : cap, n1 = c1 < cap ? c1 : cap;
    const int n = n0 + n1;
    const int32_t *l0 = cand + row * 2 * cap, *l1 = l0 + cap;
    const float *kh = kc + head * n_blk * 64;
    const int kk = k < n ? k : n;

    // the two lists, one after the other
#pragma unroll
    for (int s = 0; s < kCandSlots; ++s)
        if (s * 64 < n) {  // wave-uniform
            const int c = s * 64 + lane;
            if (c < n) ids[c] = c < n0 ? l0[c] : l1[c - n0];
        }
    // Scores.  16 lanes per candidate, 4 consecutive channels each, so that a pooled-key row is read as
    // one contiguous 256 bytes (one lane per candidate would touch 64 cache lines per load
    // instruction).  Fixed order of operations: 4 fused multiply-adds per lane,
    // then a butterfly over the 16 lanes.
    const int sub = lane & 15, quad = lane >> 4;
    const floatx4 qv = *reinterpret_cast<const floatx4 *>(qc + row * 64 + 4 * sub);
    __syncthreads();
    constexpr int U = 8;  // loads in flight per lane: 4 U candidates per pass
    for (int p0 = 0; p0 < n; p0 += 4 * U) {
        int32_t j[U];
        floatx4 kv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = p0 + 4 * u + quad;
            j[u] = c < n ? ids[c] : 0;
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            kv[u] = *reinterpret_cast<const floatx4 *>(kh + static_cast<int64_t>(j[u]) * 64 + 4 * sub);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = p0 + 4 * u + quad;
            float acc = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) acc = __builtin_fmaf(qv[i], kv[u][i], acc);
            acc += __shfl_xor(acc, 1, 64);
            acc += __shfl_xor(acc, 2, 64);
            acc += __shfl_xor(acc, 4, 64);
            acc += __shfl_xor(acc, 8, 64);
            if (sub == 0 && c < n) sc[c] = acc;
        }
    }
    __syncthreads();

    uint32_t key[kCandSlots];
    int32_t id[kCandSlots];
#pragma unroll
    for (int s = 0; s < kCandSlots; ++s) {
        key[s] = 0u;  // below the key of every real number
        id[s] = 0;
        if (s * 64 < n) {  // wave-uniform
            const int c = s * 64 + lane;
            if (c < n) {
                key[s] = order_key(sc[c]);
                id[s] = ids[c];
            }
        }
    }
    // k-th largest key by a bitwise search with wave ballots
    uint32_t T = 0u;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t trial = T | (1u << bit);
        int c = 0;
#pragma unroll
        for (int s = 0; s < kCandSlots; ++s)
            if (s * 64 < n) c += __popcll(__ballot(key[s] >= trial));
        if (c >= kk) T = trial;
    }
    // winners above T, in any order; ties at T collected for the index rule
    int n_win = 0, n_tie = 0;
#pragma unroll
    for (int s = 0; s < kCandSlots; ++s)
        if (s * 64 < n) {
            const bool gt = key[s] > T, eq = key[s] == T;
            const unsigned long long gm = __ballot(gt), em = __ballot(eq);
            if (gt) win[n_win + lanes_below(gm)] = id[s];
            if (eq) ties[n_tie + lanes_below(em)] = id[s];
            n_win += __popcll(gm);
            n_tie += __popcll(em);
        }
    __syncthreads();
    const int need = kk - n_win;  // ties to keep: the `need` smallest indices among them
#pragma unroll
    for (int s = 0; s < kCandSlots; ++s)
        if (s * 64 < n && __ballot(key[s] == T) != 0ull) {
            int rank = 0;
            for (int o = 0; o < n_tie; ++o) rank += ties[o] < id[s] ? 1 : 0;
            if (key[s] == T && rank < need) win[n_win + rank] = id[s];
        }
    __syncthreads();
    // ascending order: place = number of winners with a smaller index
    if (lane < kk) {
        const int32_t v = win[lane];
        int place = 0;
        for (int o = 0; o < kk; ++o) place += win[o] < v ? 1 : 0;
        idx[row * k + place] = v;
    } else if (lane < k) {
        idx[row * k + lane] = 0;  // fewer candidates than k (only after a cut list): keep the row in range
    }
}

hipError_t launch_topk_candidates(const float *qc, const float *kc, const int32_t *cand, const int *cand_count,
                                  int cap, int32_t *idx, int64_t n_blk, int heads, int k, hipStream_t stream)
{
    const int64_t rows = n_blk * heads;
    if (rows > 0x7fffffffLL || n_blk > 0x7fffffffLL) return hipErrorInvalidValue;
    if (k < 1 || k > 64 || cap < 1 || 2 * cap > kCandSlots * 64) return hipErrorInvalidValue;
    hipLaunchKernelGGL(topk_candidates_kernel, dim3(static_cast<unsigned>(rows)), dim3(64), 0, stream, qc, kc, cand,
                       cand_count, cap, idx, static_cast<int>(n_blk), k);
    return hipGetLastError();
}

// Forced blocks (Sec. 3.3): one workgroup turns the caller's list into the per-64-key bit words and into
// forced_clean, the list every later kernel works with: n_forced entries in [0, n_blk), ascending.  For a list
// that keeps its contract (in range, strictly ascending) that is the list itself.  Whatever else the caller
// passes is made safe rather than trusted, because an index row with a hole or an out-of-range entry would send
// the attention kernels to memory that is not theirs: entries are clamped into range, put in ascending order
// (read back from the bit words), and what duplicates leave over is filled with the last block, which is then
// simply attended more than once.  What was wrong is left in *status (when given): bit 0 = an entry outside
// [0, n_blk), bit 1 = entries not strictly ascending; 0 = fine.  The library never synchronises the host, so
// this word is how a broken list is reported.
__global__ __launch_bounds__(256) void forced_prepare_kernel(const int32_t *__restrict__ forced, int n_forced,
                                                             int n_blk, int32_t *__restrict__ forced_clean,
                                                             unsigned long long *__restrict__ words, int n_words,
                                                             int32_t *__restrict__ status)
{
    __shared__ int flags;
    __shared__ int part[256];   // set bits in each thread's run of words, then their exclusive prefix sums
    const int tid = threadIdx.x;
    if (tid == 0) flags = 0;
    for (int w = tid; w < n_words; w += 256) words[w] = 0ull;
    __syncthreads();
    int mine = 0;
    for (int a = tid; a < n_forced; a += 256) {
        int j = forced[a];
        if (j < 0 || j >= n_blk) mine |= 1;
        if (a > 0 && forced[a - 1] >= j) mine |= 2;
        j = j < 0 ? 0 : (j >= n_blk ? n_blk - 1 : j);
        atomicOr(&words[j >> 6], 1ull << (j & 63));
    }
    if (mine != 0) atomicOr(&flags, mine);
    __syncthreads();
    if (tid == 0 && status != nullptr) *status = flags;
    // the ascending list of distinct blocks, read back from the bit words: thread t owns words [t * run, (t + 1) * run)
    const int run = (n_words + 255) / 256;
    const int w0 = tid * run, w1 = (w0 + run < n_words) ? w0 + run : n_words;
    int cnt = 0;
    for (int w = w0; w < w1; ++w) cnt += __popcll(words[w]);
    part[tid] = cnt;
    __syncthreads();
    if (tid == 0) {
        int acc = 0;
        for (int t = 0; t < 256; ++t) { const int c = part[t]; part[t] = acc; acc += c; }
        flags = acc;   // number of distinct blocks (the status word has been written)
    }
    __syncthreads();
    int pos = part[tid];
    for (int w = w0; w < w1; ++w) {
        unsigned long long bits = words[w];
        while (bits != 0ull) {
            const int b = __ffsll(static_cast<long long>(bits)) - 1;
            bits &= bits - 1ull;
            if (pos < n_forced) forced_clean[pos] = w * 64 + b;
            ++pos;
        }
    }
    __syncthreads();
    const int n_distinct = flags;
    if (n_distinct > 0 && n_distinct < n_forced) {
        const int last = forced_clean[n_distinct - 1];
        for (int a = n_distinct + tid; a < n_forced; a += 256) forced_clean[a] = last;
    }
}

// One thread per output entry: an element's place in the merged list is its own position plus the
// number of elements of the other list that sort before it (forced entries first on equal values,
// which only arises if the caller's list breaks its contract).
__global__ __launch_bounds__(256) void merge_forced_kernel(const int32_t *__restrict__ dyn, int k_dyn,
                                                           const int32_t *__restrict__ forced, int n_forced,
                                                           int32_t *__restrict__ out, int64_t n_rows)
{
    const int w = k_dyn + n_forced;
    const int64_t gid = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (gid >= n_rows * w) return;
    const int64_t r = gid / w;
    const int e = static_cast<int>(gid % w);
    const int32_t *drow = dyn + r * k_dyn;
    int32_t v;
    int pos;
    if (e < n_forced) {  // a forced entry: count dynamic entries strictly smaller
        v = forced[e];
        int lo = 0, hi = k_dyn;
        while (lo < hi) { const int mid = (lo + hi) >> 1; if (drow[mid] < v) lo = mid + 1; else hi = mid; }
        pos = e + lo;
    } else {  // a dynamic entry: count forced entries smaller or equal
        const int d = e - n_forced;
        v = drow[d];
        int lo = 0, hi = n_forced;
        while (lo < hi) { const int mid = (lo + hi) >> 1; if (forced[mid] <= v) lo = mid + 1; else hi = mid; }
        pos = d + lo;
    }
    out[r * w + pos] = v;
}

hipError_t launch_forced_prepare(const int32_t *forced, int n_forced, int64_t n_blk, int32_t *forced_clean,
                                 unsigned long long *forced_words, int32_t *status, hipStream_t stream)
{
    const int n_words = n_forced > 0 ? static_cast<int>((n_blk + 63) / 64) : 0;
    hipLaunchKernelGGL(forced_prepare_kernel, dim3(1), dim3(256), 0, stream, forced, n_forced,
                       static_cast<int>(n_blk), forced_clean, forced_words, n_words, status);
    return hipGetLastError();
}

hipError_t launch_merge_forced(const int32_t *dyn, int k_dyn, const int32_t *forced_clean, int n_forced,
                               int32_t *out, int64_t n_rows, hipStream_t stream)
{
    const int64_t total = n_rows * (k_dyn + n_forced);
    const int64_t grid = (total + 255) / 256;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(merge_forced_kernel, dim3(static_cast<unsigned>(grid)), dim3(256), 0, stream, dyn, k_dyn,
                       forced_clean, n_forced, out, n_rows);
    return hipGetLastError();
}

hipError_t launch_topk(const float *s_guide, int64_t ld_s, int32_t *idx, int64_t n_blk,
                       int64_t n_rows, int k, const int *run_flag, hipStream_t stream)
{
    if (n_rows > 0x7fffffffLL || n_blk > 0x7fffffffLL) return hipErrorInvalidValue;
    const unsigned rows = static_cast<unsigned>(n_rows);
    const dim3 grid(run_flag != nullptr && rows > kFlaggedGrid ? kFlaggedGrid : rows), block(kTopkThreads);
    const int nb = static_cast<int>(n_blk);
#define S3R_TOPK_REG(NV)                                                                            \
    if (k <= kTopkThreads && nb <= (NV) * 256) {                                                    \
        hipLaunchKernelGGL(topk_reg_kernel<NV>, grid, block, 0, stream, s_guide, ld_s, idx, nb, k, rows, run_flag); \
        return hipGetLastError();                                                                   \
    }
    S3R_TOPK_REG(1)
    S3R_TOPK_REG(2)
    S3R_TOPK_REG(4)
    S3R_TOPK_REG(8)
    S3R_TOPK_REG(16)
    S3R_TOPK_REG(32)
    S3R_TOPK_REG(48)
    S3R_TOPK_REG(64)
    S3R_TOPK_REG(96)
    S3R_TOPK_REG(128)
#undef S3R_TOPK_REG
    hipLaunchKernelGGL(topk_stream_kernel, grid, block, 0, stream, s_guide, ld_s, idx, nb, k, rows, run_flag);
    return hipGetLastError();
}

}  // namespace s3r
