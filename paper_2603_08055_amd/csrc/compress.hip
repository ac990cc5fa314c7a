// Compression branch (Sec. 3.2, eqs. 3-4; supplementary Alg. 1 without its TopK part):
//   S_guide = Qc Kc^T (unscaled, written out for TopK) and Oc' = softmax(scale * S_guide) Vc,
// one pass over the pooled keys with an online softmax.
//
// gfx950 design.  Each compute wave owns 32 pooled queries and computes the TRANSPOSED score tile
// S^T[key][query] with v_mfma_f32_32x32x16_bf16 (A = pooled keys from LDS, B = pooled queries held
// in registers).  In that orientation a lane holds 16 keys of ONE query per 32-key tile, so row
// max / row sum are in-lane reductions plus one exchange with the lane 32 positions away, and the
// probabilities already sit in the register order the next MFMA (O^T = Vc^T P^T) wants.
// Scores that are written out, and all scores of fp32 problems, use bf16 hi/lo operand pairs
// (hi*hi + hi*lo + lo*hi): about 2^-16 relative to |q||k|, which keeps the TopK ordering at fp32
// quality at bf16 MFMA rates.
//
// Waves are specialised.  The kernel streams 4 N_b^2 H bytes of scores out while it streams the
// pooled keys in.  On this ISA vector loads and stores share one in-flight counter (vmcnt) and
// return out of order with respect to each other, so a wave that both stores scores and waits for
// its next key tile has to wait for its stores as well: every step would then cost a full
// store-acknowledge latency.  Hence the compute waves never load inside the loop (their score
// stores are fire-and-forget) and one more wave does nothing but move key/value operand tiles
// HBM -> LDS with LDS-direct loads, a ring of NS stages ahead, pacing itself with exact vmcnt
// counts (its counter only ever holds loads, which return in order).  One barrier per step.
//
// TopK without S_guide in memory (supplementary Sec. 1: selection fused with the compression
// sweep; here as a threshold filter that suits 64-wide waves better than a per-tile sort).
//   THRESHOLD mode: same sweep, no score stores.  Each lane keeps the running maximum of each of its
//     32 score registers, even and odd steps apart: 128 buckets per query (two lanes), every pooled
//     key falling in exactly one.  The maxima are kept as packed fp16 rounded down (32 registers):
//     a value below a bucket's true maximum is still a valid bound.  The k-th largest of the 128
//     bucket maxima is a lower bound of the query's k-th largest score (k <= 64: that many distinct
//     keys reach it); it is written out per query.
//   FILTER mode: the scores are recomputed and the index of every score at or above the query's
//     bound is appended to that lane's private candidate list (about a hundred per query instead of
//     N_b).  No softmax, no Vc, no atomics, deterministic.
// The exact TopK among the candidates is a small kernel of its own (topk.hip), which recomputes their
// scores as fp32 dot products.  Because of that the sweeps need no fp32-grade scores for TopK, only
// a rigorous error bound, and work on single fp16 copies of the pooled tensors (one MFMA per tile
// and channel step instead of three, a third of the LDS reads), scaled per head by powers of two so
// that fp16's range is never an issue (split.hip).  An fp16 score s~ and the fp32-grade score s of
// the same pair differ by at most eps = 2^-10 (1 + small) |q||k| (two operand roundings of 2^-11
// plus fp32 accumulation).  With T the k-th largest bucket maximum of the s~: k keys have
// s >= T - eps, so every key of the exact TopK has s >= T - eps and s~ >= T - 2 eps.  The threshold
// sweep therefore writes T - 2 eps, with eps from the query's own norm and the largest key norm of
// the head (topk_margin), and the filter keeps every s~ at or above that.
// For bf16 problems the threshold sweep's fp16 scores also feed the softmax of the compressed
// attention: their 2^-10 |q||k| is an eighth of what rounding the pooled tensors to bf16 would cost
// (that was measured: 2.7 % error in Oc' on N(0,1) pooled inputs, over the 2 % bar; fp16 stays far
// inside it).  fp32 problems keep the three-MFMA scores and split P and Vc as well.
#include "s3r_device.h"
#include "s3r_kernels.h"

#include <type_traits>

namespace s3r {

constexpr float kCompressRescaleSlack = 8.0f;  // see select_mfma.hip: lazy raise of the running maximum

__device__ __forceinline__ void compress_lds_dma_16(const void *src, unsigned lds_byte)
{
    // 64 lanes x 16 bytes from per-lane `src` to LDS byte address lds_byte + 16 * lane
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(lds_byte)
                 : "memory", "m0");
}

template <int N> __device__ __forceinline__ void compress_wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ float compress_max_halves(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

__device__ __forceinline__ float compress_sum_halves(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));

// Two floats to packed fp16, rounded toward zero (out-of-range values clamp to the largest finite).
__device__ __forceinline__ half2_t pack_rtz(float a, float b)
{
    return __builtin_bit_cast(half2_t, __builtin_amdgcn_cvt_pkrtz(a, b));
}

// max of packed fp16 pairs without the canonicalising copy the generic builtin adds (no NaNs here)
__device__ __forceinline__ half2_t pk_max(half2_t a, half2_t b)
{
    half2_t r;
    asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// L2 norm of the query whose operands this lane and the lane 32 positions away hold.
__device__ __forceinline__ float query_norm_f16(const bf16x8 (&q)[4])  // registers hold fp16 bits
{
    float ss = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const half8_t hv = __builtin_bit_cast(half8_t, q[s]);
#pragma unroll
        for (int i = 0; i < 8; ++i) ss = fmaf(static_cast<float>(hv[i]), static_cast<float>(hv[i]), ss);
    }
    return __builtin_sqrtf(compress_sum_halves(ss));
}
__device__ __forceinline__ float query_norm_bf16(const bf16x8 (&q)[4])
{
    float ss = 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int i = 0; i < 8; ++i) ss = fmaf(static_cast<float>(q[s][i]), static_cast<float>(q[s][i]), ss);
    return __builtin_sqrtf(compress_sum_halves(ss));
}

// How far the bound of a query must be lowered, in the scaled units of the fp16 tiles: qn = norm of the
// scaled query, kn = largest norm of a scaled key of the head.  An fp16 score and the fp32-grade score
// of the same pair differ by at most eps = 2^-10 |q||k| (two operand roundings of 2^-11 each), plus
// 2^-22 (|q| + |k|) for components that fp16 flushes or holds as subnormals (scaled components are
// below 1), plus fp32 accumulation; the bound comes from such scores and the filter compares such
// scores: 2 eps.  The factor 1.03 covers the accumulations, the roundings of the norms and of this
// expression, and (fp32 problems, whose bound comes from three-MFMA bf16 scores) the 2^-16 of those.
__device__ __forceinline__ float topk_margin(float qn, float kn)
{
    return 1.03f * (1.f / 512.f) * qn * kn + (1.f / 1048576.f) * (qn + kn);
}

enum CompressMode { kStoreScores = 0, kThreshold = 1, kFilter = 2, kThresholdPipe = 3 };

// What the TopK-in-the-sweep modes read and write besides the operands.
struct FusedTopkArgs {
    const HeadStats *stats;  // [heads]: scale factors of the fp16 tiles, largest scaled key norm (threshold modes)
    float *thr;            // [heads][n_blk]: what a key's fp16 score (scaled units) must reach to be a candidate
    int32_t *cand;         // [heads][n_blk][2][cap] candidate key indices, one list per lane of a query
    int *cand_count;       // [heads][n_blk][2] entries asked for (may exceed cap: the list is then cut)
    int *overflow;         // set to 1 when any list was cut (the caller then redoes TopK the plain way)
    const int *run_flag;   // kStoreScores only: when given and 0, the launch does nothing
    int cap;
    int k;                 // 1..64
};

// One workgroup's share: query tiles bx * CW .. + CW - 1 of head by.
template <bool SPLIT_PV, int NS, int CW, int MODE>
__device__ __forceinline__ void compress_block(
    const bf16_t *__restrict__ qs_hi, const bf16_t *__restrict__ qs_lo,
    const bf16_t *__restrict__ ks_hi, const bf16_t *__restrict__ ks_lo,
    const bf16_t *__restrict__ vt_hi, const bf16_t *__restrict__ vt_lo, float *__restrict__ s_guide,
    int64_t ld_s, float *__restrict__ o_comp, int64_t n_blk, int64_t tiles_padded, float scale_log2,
    const unsigned long long *__restrict__ forced_words, const FusedTopkArgs &ft, unsigned bx, unsigned by)
{
    // operand arrays staged per step: ks_hi, ks_lo [, vt_hi [, vt_lo]]; the sweeps on fp16 tiles: the keys'
    // fp16 tile [, vt_hi] (their q and k pointers arrive in the qs_hi / ks_hi arguments: same element size and
    // tile layout, reinterpreted where the MFMA is issued)
    constexpr int NARR = (MODE == kFilter) ? 1 : (MODE == kThresholdPipe) ? 2 : (SPLIT_PV ? 4 : 3);
    constexpr int STAGE_ELEMS = 2 * kRowTileElems;   // 64 keys x 64 channels per array: 8 KiB
    constexpr int CPS = NARR * 8;                    // 1 KiB chunks per step, all issued by the loader wave
    constexpr int D = NS - 1;                        // steps in flight
    static_assert(CPS * (D - 1) < 64, "vmcnt budget");
    __shared__ __attribute__((aligned(1024))) bf16_t ring[NS][NARR][STAGE_ELEMS];

    const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = by;
    const int n_kt = static_cast<int>((n_blk + 63) / 64);  // 64-key steps (n_blk < 2^31)
    if constexpr (MODE == kThreshold || MODE == kThresholdPipe) {
        if (bx == 0 && by == 0 && tid == 0) *ft.overflow = 0;  // the filter launch comes later in the stream
    }
    const int64_t head_tiles = static_cast<int64_t>(h) * tiles_padded;

    if constexpr (MODE == kStoreScores || MODE == kThreshold) {  // (the pipelined sweeps have no loader wave)
        if (wave == CW) {
            // ---- loader wave ---------------------------------------------------------------------
            const bf16_t *src[NARR];
            src[0] = ks_hi + head_tiles * kRowTileElems;
            src[1] = ks_lo + head_tiles * kRowTileElems;
            if constexpr (NARR >= 3) src[2] = vt_hi + head_tiles * kRowTileElems;
            if constexpr (NARR == 4) src[3] = vt_lo + head_tiles * kRowTileElems;
            const unsigned ring_base = static_cast<unsigned>(reinterpret_cast<size_t>(&ring[0][0][0]));
            auto issue = [&](int kt, int stage) {
                const unsigned stage_byte = ring_base + static_cast<unsigned>(stage) * (NARR * STAGE_ELEMS * 2);
#pragma unroll
                for (int a = 0; a < NARR; ++a)
#pragma unroll
                    for (int c = 0; c < 8; ++c)
                        compress_lds_dma_16(src[a] + static_cast<int64_t>(kt) * STAGE_ELEMS + c * 512 + lane * 8,
                                            __builtin_amdgcn_readfirstlane(stage_byte + (a * 8 + c) * 1024));
            };
            for (int kt = 0; kt < D && kt < n_kt; ++kt) issue(kt, kt);  // D < NS: stage = kt
            int stage_ahead = D - 1;  // stage of step kt + D, stepped at the loop head
            for (int kt = 0; kt < n_kt; ++kt) {
                stage_ahead = (stage_ahead + 1 == NS) ? 0 : stage_ahead + 1;
                // step kt landed (loads return in order), tell everybody; the barrier also says the
                // compute waves are done with step kt - 1, whose stage the next request overwrites
                if (kt + D <= n_kt) compress_wait_vmcnt<CPS *(D - 1)>(); else compress_wait_vmcnt<0>();
                lds_barrier();
                if (kt + D < n_kt) issue(kt + D, stage_ahead);
            }
            return;
        }
    }

    // ---- compute waves ---------------------------------------------------------------------------
    if constexpr (MODE == kThresholdPipe) {
        // The threshold sweep, software-pipelined in half steps of 32 keys inside each wave: while the
        // matrix pipe computes the scores of the next half step and the P.V product of the previous
        // one, the vector ALU runs the softmax of the current one.  (Without this every wave runs
        // MFMA and VALU phases one after the other, and the waves of a CU fall into step.)
        // Queries and keys come as fp16 tiles scaled by the head's sq and sk (qs_hi, ks_hi point at them;
        // qhi, k_hi below hold fp16 bits): scores come out multiplied by sq sk, which the logits undo.
        const float scale_log2_h = scale_log2 * ft.stats[h].inv_sqsk;
        const int64_t qtile = static_cast<int64_t>(bx) * CW + wave;
        const int64_t qrow = qtile * 32 + (lane & 31);
        const bool wave_active = qtile * 32 < n_blk;
        const int64_t row_id = static_cast<int64_t>(h) * n_blk + (qrow < n_blk ? qrow : 0);
        // Loads.  The keys of step t are read one barrier before its values, so request group t =
        // {keys of step t -> stage t % 3, values of step t - 1 -> stage (t - 1) % 3}, t = 0 .. n_kt,
        // out-of-range steps clamped (loaded, never used) so that every group has the same 16 chunks of
        // 1 KiB; each wave issues CPW of them.  Group t + 2 is requested right after the barrier that
        // publishes group t; before a barrier a wave waits until only its newest request is in flight.
        static_assert(NS == 3 && NARR == 2 && 16 % CW == 0, "pipelined sweep: three stages, one key and one value array");
        constexpr int CPW = 16 / CW;
        const bf16_t *src_k_hi = ks_hi + head_tiles * kRowTileElems;
        const bf16_t *src_v = vt_hi + head_tiles * kRowTileElems;
        const unsigned ring_base = static_cast<unsigned>(reinterpret_cast<size_t>(&ring[0][0][0]));
        auto issue_group = [&](int t, int kstage, int vstage) __attribute__((always_inline)) {
            const int tk = t < n_kt ? t : n_kt - 1, tv = t >= 1 ? t - 1 : 0;
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                static_assert(CW == 4, "chunk i * CW + wave: the array (i / 2) is then known at compile time");
                const int a = i >> 1, c = (i & 1) * 4 + wave;  // chunk i * 4 + wave of 0..7 k_hi, 8..15 v
                const bf16_t *src = (a == 0 ? src_k_hi : src_v) +
                                    static_cast<int64_t>(a == 0 ? tk : tv) * STAGE_ELEMS + c * 512 + lane * 8;
                const unsigned dst = ring_base + static_cast<unsigned>(a == 0 ? kstage : vstage) * (NARR * STAGE_ELEMS * 2) +
                                     (a * 8 + c) * 1024;
                compress_lds_dma_16(src, __builtin_amdgcn_readfirstlane(dst));
            }
        };
        issue_group(0, 0, 2);
        if (n_kt >= 1) issue_group(1, 1, 0);
        int g_kstage = 1, g_vstage = 0;  // stages of the group requested last
        auto publish = [&](int j) __attribute__((always_inline)) {  // barrier j: group j has landed everywhere; then request group j + 2
            if (j + 1 <= n_kt) compress_wait_vmcnt<CPW>(); else compress_wait_vmcnt<0>();
            lds_barrier();
            if (j + 2 <= n_kt) {
                g_kstage = (g_kstage + 1 == 3) ? 0 : g_kstage + 1;
                g_vstage = (g_vstage + 1 == 3) ? 0 : g_vstage + 1;
                issue_group(j + 2, g_kstage, g_vstage);
            }
        };
        bf16x8 qhi[4];
        {
            // query tiles past the end of the head's range (inactive waves) still take part in the loads
            // and barriers; they compute on the last tile and write nothing
            const int64_t qt = wave_active ? qtile : (n_blk - 1) / 32;
            const int64_t qb = (head_tiles + qt) * kRowTileElems;
#pragma unroll
            for (int s = 0; s < 4; ++s) qhi[s] = *reinterpret_cast<const bf16x8 *>(qs_hi + qb + (s * 64 + lane) * 8);
        }
        floatx16 oacc[2];
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
        float m_run = -1e30f, l_run = 0.f;
        half2_t bmax[2][16];  // [step parity][mt * 8 + register pair]
#pragma unroll
        for (int par = 0; par < 2; ++par)
#pragma unroll
            for (int i = 0; i < 16; ++i) bmax[par][i] = half2_t{-INFINITY, -INFINITY};

        // scores of half step mt of the keys in `stage` (only used before the loop)
        auto scores = [&](int stage, int mt, floatx16 &acc) __attribute__((always_inline)) {
            const bf16_t *k_hi = &ring[stage][0][0];
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const bf16x8 a_hi = *reinterpret_cast<const bf16x8 *>(k_hi + mt * kRowTileElems + (s * 64 + lane) * 8);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, a_hi), __builtin_bit_cast(half8_t, qhi[s]), acc, 0, 0, 0);
            }
        };
        // O^T += Vc^T P^T for half step mt of the values in `stage` (only used after the loop)
        auto pv = [&](int stage, int mt, const bf16x8 (&p)[2]) __attribute__((always_inline)) {
            const bf16_t *v_hi = &ring[stage][1][0];
#pragma unroll
            for (int w = 0; w < 2; ++w)
#pragma unroll
                for (int dt = 0; dt < 2; ++dt) {
                    const bf16x8 b = *reinterpret_cast<const bf16x8 *>(v_hi + mt * kRowTileElems + ((w * 2 + dt) * 64 + lane) * 8);
                    oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, p[w], oacc[dt], 0, 0, 0);
                }
        };
        // before the overlapped region: keys that do not exist, the running maximum (rarely raised).
        // p_pending: the probabilities of the half step before, whose P.V product has not been issued yet (it
        // runs inside the half step that follows): they were formed against the old maximum, so a raise
        // rescales them together with the accumulators (Alg. 1's rescaling applies to everything summed so far).
        auto soft_pre = [&](int kt, int mt, floatx16 &acc, bf16x8 (&p_pending)[2]) __attribute__((always_inline)) {
            if (kt * 64 + mt * 32 + 32 > n_blk) {
                asm volatile("" ::: "memory");  // keep this rare path a real branch
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (kt * 64 + mt * 32 + acc_row(lane, r) >= n_blk) acc[r] = -INFINITY;
            }
            float mx = acc[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, acc[r]);
            const float m_tile = compress_max_halves(mx) * scale_log2_h;
            const bool grow = m_tile > m_run + kCompressRescaleSlack;
            if (__any(grow)) {
                const float m_new = grow ? m_tile : m_run;
                const float alpha = fast_exp2(m_run - m_new);
                m_run = m_new;
                l_run *= alpha;
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
#pragma unroll
                for (int w = 0; w < 2; ++w)
#pragma unroll
                    for (int e = 0; e < 8; ++e) p_pending[w][e] = static_cast<bf16_t>(static_cast<float>(p_pending[w][e]) * alpha);
            }
        };
        // One half step, written out as 16 slots of vector work on one score register each, every other
        // one led by an MFMA and by the LDS operand read for the MFMA three places later, with a
        // scheduling fence after every slot so that the order stays as written.  The MFMAs: P.V of the
        // half step before (values in stage pv_stage, half pv_mt, operands p_in), then the scores of the
        // half step after (keys in stage k_stage, half k_mt, into acc_next).  The vector work: the softmax
        // of this half step (scores acc, half mt): bucket maxima, probabilities, their sum, bf16 operands
        // p_out.
        auto half_step = [&](auto forced_tag, unsigned long long fw, int mt, floatx16 &acc, half2_t (&bm)[16],
                             bf16x8 (&p_out)[2], int pv_stage, int pv_mt, const bf16x8 (&p_in)[2], int k_stage,
                             int k_mt, floatx16 &acc_next) __attribute__((always_inline)) {
            constexpr bool FORCED = decltype(forced_tag)::value;
            const bf16_t *v_src = &ring[pv_stage][1][0] + pv_mt * kRowTileElems + lane * 8;
            const bf16_t *khi_src = &ring[k_stage][0][0] + k_mt * kRowTileElems + lane * 8;
            bf16x8 rd[8];  // reads in order of need: V chunks 0..3, then the keys of channel steps 0..3
            auto read = [&](int i) __attribute__((always_inline)) {
                rd[i] = *reinterpret_cast<const bf16x8 *>(i < 4 ? v_src + i * 512 : khi_src + (i - 4) * 512);
            };
            read(0); read(1); read(2);
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_next[r] = 0.f;
            float lsum[4] = {0.f, 0.f, 0.f, 0.f};
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                // ---- matrix pipe
                if ((j & 1) == 0) {
                    const int m = j >> 1;
                    if (m < 4) oacc[m & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rd[m], p_in[m >> 1], oacc[m & 1], 0, 0, 0);
                    else acc_next = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, rd[m]), __builtin_bit_cast(half8_t, qhi[m - 4]), acc_next, 0, 0, 0);
                    if (m + 3 < 8) read(m + 3);
                }
                // ---- vector ALU, score register j
                if ((j & 1) == 0) {
                    float a0 = acc[j], a1 = acc[j + 1];
                    if constexpr (FORCED) {  // forced blocks do not compete (Sec. 3.3)
                        const unsigned two = static_cast<unsigned>(fw >> (mt * 32 + acc_row(lane, j))) & 3u;
                        a0 = (two & 1u) ? -INFINITY : a0;
                        a1 = (two & 2u) ? -INFINITY : a1;
                    }
                    bm[mt * 8 + (j >> 1)] = pk_max(bm[mt * 8 + (j >> 1)], pack_rtz(a0, a1));
                }
                acc[j] = fast_exp2(acc[j] * scale_log2_h - m_run);
                if (j & 1) {
                    // the pair as bf16 operands of P.V; the row sum adds the same rounded values (one
                    // dot-product instruction per pair)
                    const bf16x2 pr = {static_cast<bf16_t>(acc[j - 1]), static_cast<bf16_t>(acc[j])};
                    p_out[j >> 3][(j & 7) - 1] = pr[0];
                    p_out[j >> 3][j & 7] = pr[1];
                    lsum[(j >> 1) & 3] = __builtin_amdgcn_fdot2_f32_bf16(pr, bf16x2{static_cast<bf16_t>(1.f), static_cast<bf16_t>(1.f)},
                                                                         lsum[(j >> 1) & 3], false);
                }
                // nothing needs these values before the next barrier: tie them to this slot, or the
                // compiler moves the vector work away from the MFMAs it is meant to overlap with
                if (j & 1) asm volatile("" : "+v"(lsum[(j >> 1) & 3]));
                else asm volatile("" : "+v"(acc[j]));
                if ((j & 1) == 0) asm volatile("" : "+v"(bm[mt * 8 + (j >> 1)]));
                if ((j & 7) == 7) asm volatile("" : "+v"(p_out[j >> 3]));
                __builtin_amdgcn_sched_barrier(0);
            }
            l_run += (lsum[0] + lsum[1]) + (lsum[2] + lsum[3]);
        };

        floatx16 sacc0, sacc1;
        bf16x8 p0[2], p1[2];
#pragma unroll
        for (int w = 0; w < 2; ++w)
#pragma unroll
            for (int i = 0; i < 8; ++i) p1[w][i] = static_cast<bf16_t>(0.f);  // first P.V of the loop adds nothing
        publish(0);  // group 0: keys of step 0 (and a copy of the values of step 0 in stage 2)
        scores(0, 0, sacc0);
        int kst = 0, vprev = 2;  // stage of the keys of step kt; stage of the values of step kt - 1
        // one 64-key step; PAR = step parity (which bucket set), as a compile-time choice
        auto step = [&](auto forced_tag, auto par_tag, int kt) __attribute__((always_inline)) {
            constexpr int PAR = decltype(par_tag)::value;
            const unsigned long long fw = decltype(forced_tag)::value ? forced_words[kt] : 0ull;  // wave-uniform
            const int knext = (kst + 1 == 3) ? 0 : kst + 1;
            // half step 0: softmax here; P.V of the previous half step and scores of half step 1 on the matrix pipe
            soft_pre(kt, 0, sacc0, p1);
            half_step(forced_tag, fw, 0, sacc0, bmax[PAR], p0, vprev, 1, p1, kst, 1, sacc1);
            publish(kt + 1);  // group kt + 1: keys of step kt + 1, values of step kt
            // half step 1: softmax here; P.V of half step 0 and the first scores of the next step on the matrix pipe
            // (after the last step: a copy of its keys, result unused)
            soft_pre(kt, 1, sacc1, p0);
            half_step(forced_tag, fw, 1, sacc1, bmax[PAR], p1, kst, 0, p0, knext, 0, sacc0);
            vprev = kst;
            kst = knext;
        };
        auto sweep = [&](auto forced_tag) __attribute__((always_inline)) {
            int kt = 0;
            for (; kt + 1 < n_kt; kt += 2) {
                step(forced_tag, std::integral_constant<int, 0>{}, kt);
                step(forced_tag, std::integral_constant<int, 1>{}, kt + 1);
            }
            if (kt < n_kt) step(forced_tag, std::integral_constant<int, 0>{}, kt);
        };
        if (forced_words != nullptr) sweep(std::true_type{}); else sweep(std::false_type{});
        pv(vprev, 1, p1);

        {
            float bm[64];
#pragma unroll
            for (int par = 0; par < 2; ++par)
#pragma unroll
                for (int i = 0; i < 16; ++i)
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        unsigned short bits = __builtin_bit_cast(unsigned short, static_cast<_Float16>(bmax[par][i][e]));
                        if ((bits & 0x8000u) && bits != 0xfc00u) bits += 1;  // rounded toward zero: step negatives down
                        bm[par * 32 + i * 2 + e] = static_cast<float>(__builtin_bit_cast(_Float16, bits));
                    }
            uint32_t T = 0u;
            for (int bit = 31; bit >= 0; --bit) {
                const uint32_t trial = T | (1u << bit);
                const float trial_f = key_to_float(trial);
                int c = 0;
                if (trial_f == trial_f) {
#pragma unroll
                    for (int i = 0; i < 64; ++i) c += bm[i] >= trial_f ? 1 : 0;
                }
                const auto sw = __builtin_amdgcn_permlane32_swap(static_cast<unsigned>(c), static_cast<unsigned>(c), false, false);
                if (static_cast<int>(sw[0] + sw[1]) >= ft.k) T = trial;
            }
            const float margin = topk_margin(query_norm_f16(qhi), ft.stats[h].kn);
            if (qrow < n_blk && g == 0) ft.thr[row_id] = T < 0x007fffffu ? -INFINITY : key_to_float(T) - margin;
        }
        if (qrow < n_blk) {
            const float inv = 1.f / compress_sum_halves(l_run);
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
        return;
    }
    if constexpr (MODE == kFilter) {
        // Scores only (hi parts), software-pipelined in half steps of 32 keys like the threshold sweep:
        // while the matrix pipe computes the scores of the next half step, the vector ALU compares the
        // current ones with the query's bound; the (few) keys that pass are then appended to the lane's
        // list.  (Two query tiles per wave, which halves the LDS reads per MFMA, measured no faster.)
        const int64_t qtile = static_cast<int64_t>(bx) * CW + wave;
        const int64_t qrow = qtile * 32 + (lane & 31);
        const bool wave_active = qtile * 32 < n_blk;
        const bool row_ok = qrow < n_blk;
        const int64_t row_id = static_cast<int64_t>(h) * n_blk + (row_ok ? qrow : 0);
        // Loads: no loader wave; each wave issues CPW of the 8 one-KiB chunks of a step, D steps ahead,
        // right after the barrier that publishes a step, and before a barrier waits until only its
        // requests for later steps are in flight.  (The candidate stores share the counter; they only
        // make the wait stricter.  Collecting the candidates in LDS and writing them out in batches
        // was measured: slower.)
        static_assert(NARR == 1 && 8 % CW == 0, "filter sweep: hi parts of the keys only");
        constexpr int CPW = 8 / CW;
        static_assert(CPW * (D - 1) < 64, "vmcnt budget");
        const bf16_t *src_k_hi = ks_hi + head_tiles * kRowTileElems;
        const unsigned ring_base = static_cast<unsigned>(reinterpret_cast<size_t>(&ring[0][0][0]));
        auto issue_step = [&](int t, int stage) __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < CPW; ++i) {
                const int chunk = i * CW + wave;
                compress_lds_dma_16(src_k_hi + static_cast<int64_t>(t) * STAGE_ELEMS + chunk * 512 + lane * 8,
                                    __builtin_amdgcn_readfirstlane(
                                        ring_base + static_cast<unsigned>(stage) * (NARR * STAGE_ELEMS * 2) + chunk * 1024));
            }
        };
        for (int t = 0; t < D && t < n_kt; ++t) issue_step(t, t);  // D < NS: stage = t
        int stage_ahead = D - 1;
        auto publish = [&](int j) __attribute__((always_inline)) {  // barrier j: step j has landed everywhere (j = n_kt: nothing new); then request step j + D
            if (j + D <= n_kt) compress_wait_vmcnt<CPW *(D - 1)>(); else compress_wait_vmcnt<0>();
            lds_barrier();
            stage_ahead = (stage_ahead + 1 == NS) ? 0 : stage_ahead + 1;
            if (j + D < n_kt) issue_step(j + D, stage_ahead);
        };
        // A score passes when score - bound is not negative.  Scores are finite; the bound is kept finite
        // or +inf so that the difference is never NaN: -inf (fewer than k keys compete: every real key
        // passes) becomes the lowest finite float, rows that do not exist get +inf (nothing passes).
        float thr_f = INFINITY;
        if (wave_active && row_ok) thr_f = fmaxf(ft.thr[row_id], -3.4028234664e38f);
        floatx16 neg_thr;  // where the MFMA chains start
#pragma unroll
        for (int r = 0; r < 16; ++r) neg_thr[r] = -thr_f;
        int32_t *cand_row = ft.cand + (row_id * 2 + g) * ft.cap;
        int n_cand = 0;
        bf16x8 qhi[4];
        {
            // waves past the end of the head's range still take part in loads and barriers
            const int64_t qt = wave_active ? qtile : (n_blk - 1) / 32;
            const int64_t qb = (head_tiles + qt) * kRowTileElems;
#pragma unroll
            for (int s = 0; s < 4; ++s) qhi[s] = *reinterpret_cast<const bf16x8 *>(qs_hi + qb + (s * 64 + lane) * 8);
        }
        // One half step as 4 slots of {one MFMA of the next half step's scores, its LDS operand read two
        // slots ahead, the vector work on four of the current scores}, order fixed by scheduling fences;
        // then the emission of the keys that passed.  The MFMA chain starts from minus the bound instead
        // of zero, so a register holds score - bound, and the vector work per score is a single funnel
        // shift that appends its sign bit to the lane's mask (compare, select and shift-or would be three
        // instructions, and this sweep is bound by the vector ALU).  Adding the bound inside the chain
        // moves the result by a few fp32 roundings of |bound| + |score|, far inside the margin the bound
        // already carries.
        auto half_step = [&](int kt, int mt, floatx16 &acc, int k_stage, int k_mt, floatx16 &acc_next,
                             unsigned long long fw) __attribute__((always_inline)) {
            // keys that do not exist or are forced never become candidates: -inf is below every bound
            if (kt * 64 + mt * 32 + 32 > n_blk || fw != 0ull) {
                asm volatile("" ::: "memory");  // keep this rare path a real branch
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int b = mt * 32 + acc_row(lane, r);
                    if (kt * 64 + b >= n_blk || ((fw >> b) & 1ull)) acc[r] = -INFINITY;
                }
            }
            const bf16_t *khi_src = &ring[k_stage][0][0] + k_mt * kRowTileElems + lane * 8;
            bf16x8 rd[4];  // keys of channel steps 0..3
            auto read = [&](int i) __attribute__((always_inline)) {
                rd[i] = *reinterpret_cast<const bf16x8 *>(khi_src + i * 512);
            };
            read(0); read(1);
            unsigned fail = 0u;  // register r -> bit 15 - r, set when the score is below the bound
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                acc_next = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, rd[j]), __builtin_bit_cast(half8_t, qhi[j]),
                                                                  j == 0 ? neg_thr : acc_next, 0, 0, 0);
                if (j + 2 < 4) read(j + 2);
#pragma unroll
                for (int r = 4 * j; r < 4 * j + 4; ++r)
                    fail = __builtin_amdgcn_alignbit(fail, __float_as_uint(acc[r]), 31);  // (fail << 1) | sign
                asm volatile("" : "+v"(fail));
                __builtin_amdgcn_sched_barrier(0);
            }
            unsigned pass = ~fail & 0xffffu;
            while (pass != 0u) {
                const int r = __clz(pass) - 16;
                pass &= ~(0x8000u >> r);
                const int key = kt * 64 + 32 * mt + acc_row(lane, r);
                if (n_cand < ft.cap) cand_row[n_cand] = key;
                ++n_cand;
            }
        };
        floatx16 sacc0, sacc1;
        publish(0);  // keys of step 0
        {
            const bf16_t *k_hi = &ring[0][0][0];
            sacc0 = neg_thr;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const bf16x8 a_hi = *reinterpret_cast<const bf16x8 *>(k_hi + (s * 64 + lane) * 8);
                sacc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, a_hi), __builtin_bit_cast(half8_t, qhi[s]), sacc0, 0, 0, 0);
            }
        }
        int kst = 0;
        for (int kt = 0; kt < n_kt; ++kt) {
            const unsigned long long fw = (forced_words != nullptr) ? forced_words[kt] : 0ull;  // wave-uniform
            const int knext = (kst + 1 == NS) ? 0 : kst + 1;
            half_step(kt, 0, sacc0, kst, 1, sacc1, fw);
            publish(kt + 1);  // keys of step kt + 1 (after the last step: nothing new; the scores computed
                              // from that stage are never looked at)
            half_step(kt, 1, sacc1, knext, 0, sacc0, fw);
            kst = knext;
        }
        if (wave_active && row_ok) {
            ft.cand_count[row_id * 2 + g] = n_cand;
            if (n_cand > ft.cap) atomicOr(ft.overflow, 1);
        }
        return;
    }
    if constexpr (MODE == kStoreScores || MODE == kThreshold) {
        const int64_t qtile = static_cast<int64_t>(bx) * CW + wave;
        const int64_t qrow = qtile * 32 + (lane & 31);
        const bool wave_active = qtile * 32 < n_blk;

        bf16x8 qhi[4], qlo[4];
        if (wave_active) {
            const int64_t qb = (head_tiles + qtile) * kRowTileElems;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                qhi[s] = *reinterpret_cast<const bf16x8 *>(qs_hi + qb + (s * 64 + lane) * 8);
                qlo[s] = *reinterpret_cast<const bf16x8 *>(qs_lo + qb + (s * 64 + lane) * 8);
            }
        }
        floatx16 oacc[2];
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
        float m_run = -1e30f, l_run = 0.f;
        float *srow = s_guide + (static_cast<int64_t>(h) * n_blk + (qrow < n_blk ? qrow : 0)) * ld_s;
        const int64_t row_id = static_cast<int64_t>(h) * n_blk + (qrow < n_blk ? qrow : 0);

        half2_t bmax[2][16];         // kThreshold: running maxima of the score registers (pairs, fp16 rounded
                                     // toward zero), even and odd steps apart
        if constexpr (MODE == kThreshold) {
#pragma unroll
            for (int par = 0; par < 2; ++par)
#pragma unroll
                for (int i = 0; i < 16; ++i) bmax[par][i] = half2_t{-INFINITY, -INFINITY};
        }

        int stage = NS - 1;
        for (int kt = 0; kt < n_kt; ++kt) {
            stage = (stage + 1 == NS) ? 0 : stage + 1;
            lds_barrier();
            if (!wave_active) continue;
            const bf16_t *k_hi = &ring[stage][0][0];
            const bf16_t *k_lo = &ring[stage][1][0];

            floatx16 sacc[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[mt][r] = 0.f;
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const int off = mt * kRowTileElems + (s * 64 + lane) * 8;
                    const bf16x8 a_hi = *reinterpret_cast<const bf16x8 *>(k_hi + off);
                    const bf16x8 a_lo = *reinterpret_cast<const bf16x8 *>(k_lo + off);
                    sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo, qhi[s], sacc[mt], 0, 0, 0);
                    sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, qlo[s], sacc[mt], 0, 0, 0);
                    sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, qhi[s], sacc[mt], 0, 0, 0);
                }
            }
            const unsigned long long fw = (forced_words != nullptr) ? forced_words[kt] : 0ull;  // wave-uniform
            if constexpr (MODE == kStoreScores) {
                // eq. 4: raw scores out, 4 consecutive keys of one query row per store; never waited for
                if (qrow < n_blk) {
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                        for (int r4 = 0; r4 < 4; ++r4) {
                            const int64_t key0 = kt * 64 + mt * 32 + 8 * r4 + 4 * g;
                            if (key0 < ld_s) {
                                floatx4 o;
#pragma unroll
                                for (int i = 0; i < 4; ++i) o[i] = sacc[mt][4 * r4 + i];
                                if (fw != 0ull) {  // forced blocks leave the TopK competition (Sec. 3.3)
                                    const unsigned nib = static_cast<unsigned>(fw >> (mt * 32 + 8 * r4 + 4 * g)) & 0xFu;
#pragma unroll
                                    for (int i = 0; i < 4; ++i)
                                        if (nib & (1u << i)) o[i] = -INFINITY;
                                }
                                *reinterpret_cast<floatx4 *>(srow + key0) = o;
                            }
                        }
                }
            }
            if (kt * 64 + 64 > n_blk) {           // pooled keys past the end of the sequence do not exist
                asm volatile("" ::: "memory");    // keep this rare path a real branch
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (kt * 64 + mt * 32 + acc_row(lane, r) >= n_blk) sacc[mt][r] = -INFINITY;
            }
            if constexpr (MODE == kThreshold) {
                auto raise = [&](half2_t (&bm)[16]) {
                    if (fw == 0ull) {
#pragma unroll
                        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                            for (int r2 = 0; r2 < 8; ++r2)
                                bm[mt * 8 + r2] = __builtin_elementwise_max(
                                    bm[mt * 8 + r2], pack_rtz(sacc[mt][2 * r2], sacc[mt][2 * r2 + 1]));
                    } else {  // forced blocks do not compete (Sec. 3.3)
#pragma unroll
                        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                            for (int r2 = 0; r2 < 8; ++r2) {
                                const unsigned two = static_cast<unsigned>(fw >> (mt * 32 + acc_row(lane, 2 * r2))) & 3u;
                                bm[mt * 8 + r2] = __builtin_elementwise_max(
                                    bm[mt * 8 + r2], pack_rtz((two & 1u) ? -INFINITY : sacc[mt][2 * r2],
                                                              (two & 2u) ? -INFINITY : sacc[mt][2 * r2 + 1]));
                            }
                    }
                };
                if (kt & 1) raise(bmax[1]); else raise(bmax[0]);  // wave-uniform
            }
            const bf16_t *v_hi = &ring[stage][NARR >= 3 ? 2 : 0][0];
            const bf16_t *v_lo = &ring[stage][NARR - 1][0];
            // online softmax (eq. 3), base-2 exponent with the scale folded in
            float mx = sacc[0][0];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[mt][r]);
            const float m_tile = compress_max_halves(mx) * scale_log2;
            const bool grow = m_tile > m_run + kCompressRescaleSlack;
            if (__any(grow)) {
                const float m_new = grow ? m_tile : m_run;
                const float alpha = fast_exp2(m_run - m_new);
                m_run = m_new;
                l_run *= alpha;
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
            }
            float lsum[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    sacc[mt][r] = fast_exp2(sacc[mt][r] * scale_log2 - m_run);
                    lsum[r & 3] += sacc[mt][r];
                }
            l_run += (lsum[0] + lsum[1]) + (lsum[2] + lsum[3]);
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
                    const bf16x8 b_hi = *reinterpret_cast<const bf16x8 *>(v_hi + off);
                    oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b_hi, p_hi, oacc[dt], 0, 0, 0);
                    if constexpr (SPLIT_PV) {
                        const bf16x8 b_lo = *reinterpret_cast<const bf16x8 *>(v_lo + off);
                        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b_lo, p_hi, oacc[dt], 0, 0, 0);
                        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b_hi, p_lo, oacc[dt], 0, 0, 0);
                    }
                }
            }
        }

        if constexpr (MODE == kThreshold) {
            if (wave_active) {
                // k-th largest of the query's 128 bucket maxima (64 here, 64 in the lane 32 positions away),
                // by a bitwise search over order-preserving keys.  Buckets that saw no key hold -inf; with
                // fewer than k real maxima the bound is -inf and every key becomes a candidate.
                // The stored maxima were rounded toward zero: step the negative ones one fp16 down so that
                // every bucket value is at most the bucket's true maximum.
                float bm[64];
#pragma unroll
                for (int par = 0; par < 2; ++par)
#pragma unroll
                    for (int i = 0; i < 16; ++i)
#pragma unroll
                        for (int e = 0; e < 2; ++e) {
                            unsigned short bits = __builtin_bit_cast(unsigned short, static_cast<_Float16>(bmax[par][i][e]));
                            if ((bits & 0x8000u) && bits != 0xfc00u) bits += 1;  // -65504 steps to -inf
                            bm[par * 32 + i * 2 + e] = static_cast<float>(__builtin_bit_cast(_Float16, bits));
                        }
                uint32_t T = 0u;
                for (int bit = 31; bit >= 0; --bit) {
                    const uint32_t trial = T | (1u << bit);
                    const float trial_f = key_to_float(trial);  // x >= trial_f  <=>  order_key(x) >= trial
                    int c = 0;
                    if (trial_f == trial_f) {  // keys above +inf's are NaN patterns: nothing reaches them
#pragma unroll
                        for (int i = 0; i < 64; ++i) c += bm[i] >= trial_f ? 1 : 0;
                    }
                    const auto sw = __builtin_amdgcn_permlane32_swap(static_cast<unsigned>(c), static_cast<unsigned>(c), false, false);
                    if (static_cast<int>(sw[0] + sw[1]) >= ft.k) T = trial;
                }
                // trial keys below the key of -inf are NaN patterns and never taken: T stays under it exactly
                // when fewer than k buckets hold a real maximum
                // these scores are in the inputs' own units; the filter works in the scaled units of the fp16 tiles
                const HeadStats st = ft.stats[h];
                const float margin = topk_margin(query_norm_bf16(qhi) * st.sq * 1.004f, st.kn);
                if (qrow < n_blk && g == 0) ft.thr[row_id] = T < 0x007fffffu ? -INFINITY : key_to_float(T) * st.sqsk - margin;
            }
        }
        if (wave_active && qrow < n_blk) {
            const float inv = 1.f / compress_sum_halves(l_run);
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
}

// grid: (ceil(tiles / CW), heads); CW compute waves (32 pooled queries each) + 1 loader wave.  With a
// run flag (kStoreScores only): a small 1-D grid that does nothing when the device word is 0 and
// walks over the (gx, gy) shares otherwise.
// The pipelined sweeps have no loader wave: all CW waves compute and each issues its share of the loads.
template <int CW, int MODE> constexpr int compress_threads() { return (MODE == kThresholdPipe || MODE == kFilter) ? CW * 64 : (CW + 1) * 64; }

template <bool SPLIT_PV, int NS, int CW, int MODE>
__global__ __launch_bounds__((compress_threads<CW, MODE>()), (MODE == kFilter ? 4 : 2)) void compress_kernel(
    const bf16_t *__restrict__ qs_hi, const bf16_t *__restrict__ qs_lo,
    const bf16_t *__restrict__ ks_hi, const bf16_t *__restrict__ ks_lo,
    const bf16_t *__restrict__ vt_hi, const bf16_t *__restrict__ vt_lo, float *__restrict__ s_guide,
    int64_t ld_s, float *__restrict__ o_comp, int64_t n_blk, int64_t tiles_padded, float scale_log2,
    const unsigned long long *__restrict__ forced_words, FusedTopkArgs ft, unsigned gx, unsigned gy)
{
    if (MODE != kStoreScores || ft.run_flag == nullptr) {
        compress_block<SPLIT_PV, NS, CW, MODE>(qs_hi, qs_lo, ks_hi, ks_lo, vt_hi, vt_lo, s_guide, ld_s, o_comp, n_blk,
                                               tiles_padded, scale_log2, forced_words, ft, blockIdx.x, blockIdx.y);
        return;
    }
    if (*ft.run_flag == 0) return;  // uniform over the grid
    for (unsigned v = blockIdx.x; v < gx * gy; v += gridDim.x) {
        compress_block<SPLIT_PV, NS, CW, MODE>(qs_hi, qs_lo, ks_hi, ks_lo, vt_hi, vt_lo, s_guide, ld_s, o_comp, n_blk,
                                               tiles_padded, scale_log2, forced_words, ft, v % gx, v / gx);
        __syncthreads();
    }
}

template <bool SPLIT_PV, int NS, int CW, int MODE>
static hipError_t run_compress(const void *qs_hi, const void *qs_lo, const void *ks_hi, const void *ks_lo,
                               const void *vt_hi, const void *vt_lo, float *s_guide, int64_t ld_s,
                               float *o_comp, int64_t n_blk, int heads, float scale_log2,
                               const unsigned long long *forced_words, const FusedTopkArgs &ft,
                               hipStream_t stream)
{
    const int64_t tiles = pooled_tiles_padded(n_blk);
    const int64_t q_tiles = (n_blk + 31) / 32;
    const unsigned gx = static_cast<unsigned>((q_tiles + CW - 1) / CW), gy = static_cast<unsigned>(heads);
    dim3 grid(gx, gy);
    if (MODE == kStoreScores && ft.run_flag != nullptr) {
        const unsigned long long total = static_cast<unsigned long long>(gx) * gy;
        if (total > 0xffffffffull) return hipErrorInvalidValue;
        grid = dim3(total > kFlaggedGrid ? kFlaggedGrid : static_cast<unsigned>(total), 1);
    }
    hipLaunchKernelGGL((compress_kernel<SPLIT_PV, NS, CW, MODE>), grid, dim3(compress_threads<CW, MODE>()), 0, stream,
                       static_cast<const bf16_t *>(qs_hi), static_cast<const bf16_t *>(qs_lo),
                       static_cast<const bf16_t *>(ks_hi), static_cast<const bf16_t *>(ks_lo),
                       static_cast<const bf16_t *>(vt_hi), static_cast<const bf16_t *>(vt_lo), s_guide, ld_s,
                       o_comp, n_blk, tiles, scale_log2, forced_words, ft, gx, gy);
    return hipGetLastError();
}

hipError_t launch_compress(const void *qs_hi, const void *qs_lo, const void *ks_hi,
                           const void *ks_lo, const void *vt_hi, const void *vt_lo, float *s_guide,
                           int64_t ld_s, float *o_comp, int64_t n_blk, int heads, float scale,
                           const unsigned long long *forced_words, const int *run_flag, hipStream_t stream)
{
    const float sl = scale * kLog2e;
    FusedTopkArgs ft{};
    ft.run_flag = run_flag;
    if (vt_lo != nullptr)
        return run_compress<true, 2, 3, kStoreScores>(qs_hi, qs_lo, ks_hi, ks_lo, vt_hi, vt_lo, s_guide, ld_s, o_comp, n_blk, heads, sl, forced_words, ft, stream);
    // 3 compute waves + 1 loader wave, 3 LDS stages (72 KiB): two workgroups per CU.  Measured
    // best on MI355X against 4 + 1 waves and 2 or 4 stages.
    return run_compress<false, 3, 3, kStoreScores>(qs_hi, qs_lo, ks_hi, ks_lo, vt_hi, vt_lo, s_guide, ld_s, o_comp, n_blk, heads, sl, forced_words, ft, stream);
}

hipError_t launch_compress_threshold(const void *qs_hi, const void *qs_lo, const void *ks_hi, const void *ks_lo,
                                     const void *vt_hi, const void *vt_lo, const void *q_f16, const void *k_f16,
                                     float *o_comp, int64_t n_blk, int heads, float scale,
                                     const unsigned long long *forced_words, int k, const HeadStats *stats,
                                     float *thr, int *overflow, hipStream_t stream)
{
    if (k < 1 || k > kFusedTopkMaxK || stats == nullptr) return hipErrorInvalidValue;
    const float sl = scale * kLog2e;
    FusedTopkArgs ft{};
    ft.stats = stats; ft.thr = thr; ft.overflow = overflow; ft.k = k;
    if (vt_lo != nullptr)
        return run_compress<true, 2, 3, kThreshold>(qs_hi, qs_lo, ks_hi, ks_lo, vt_hi, vt_lo, nullptr, 0, o_comp, n_blk, heads, sl, forced_words, ft, stream);
    // (the fp16 tiles travel through the kernel's bf16-typed operand pointers: same size, same tile layout)
    return run_compress<false, 3, 4, kThresholdPipe>(q_f16, nullptr, k_f16, nullptr, vt_hi, nullptr, nullptr, 0, o_comp, n_blk, heads, sl, forced_words, ft, stream);
}

hipError_t launch_compress_filter(const void *q_f16, const void *k_f16,
                                  int64_t n_blk, int heads, const unsigned long long *forced_words,
                                  const float *thr, int32_t *cand, int *cand_count, int cap, int *overflow,
                                  hipStream_t stream)
{
    FusedTopkArgs ft{};
    ft.thr = const_cast<float *>(thr); ft.cand = cand; ft.cand_count = cand_count; ft.cap = cap; ft.overflow = overflow;
    // (the fp16 tiles travel through the kernel's bf16-typed operand pointers: same size, same tile layout)
    return run_compress<false, 4, 4, kFilter>(q_f16, nullptr, k_f16, nullptr, nullptr, nullptr, nullptr, 0, nullptr, n_blk, heads, 0.f, forced_words, ft, stream);
}

}  // namespace s3r
