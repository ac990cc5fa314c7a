// Selection attention + merge (Sec. 3.2 eq. 6, supplementary Alg. 2; eqs. 5, 7, 8) on bf16 MFMA for gfx950:
// the kernel for plain index rows of blocks of 64 tokens, built around what binds this stage on MI355X.
//
// What binds it.  Every (query block, selected key block, head) moves 16 KiB of K/V for 1 MFLOP, so the
// stage runs at the rate at which K/V units arrive, and that rate is set by how many of the requests hit in
// the L2 of the XCD that issues them: L2 misses are delivered at about 7.8 TB/s whatever the kernel does,
// while neighbouring query blocks, which the work mapping runs on the same XCD at the same time, select
// overlapping key blocks.  A unit fetched for one query block is still in the 4 MiB L2 when a neighbour asks
// for it only if few other units have come in between, i.e. if FEW query blocks are in progress per XCD.
// The same index lists measured with the arithmetic taken out (speed3r_probe_select_loads): five
// workgroups per CU 39 ms with 20 % L2 hits, three 34 ms, one 32 ms with 33 % hits.
//
// Hence few workgroups per CU, and a wave that keeps both of its pipes busy by itself instead of relying on
// many waves per SIMD to fill the gaps.  As in select_mfma.hip a workgroup is one query block, a wave owns
// 32 query rows and computes the transposed score tile S^T = K Q^T of a 64-key unit (a lane holds keys of
// one query, so row maxima and sums are lane-local).  New: a wave's unit j goes through three phases in three
// consecutive iterations,
//   iteration i:  S(i + 1) = K(i + 1) Q^T  |  softmax of S(i) -> P(i)  |  O += V(i - 1)^T P(i - 1)
// so that in every iteration the matrix pipe (16 MFMAs) and the vector ALU (softmax of 32 scores per lane)
// of one wave have independent work; the loop body is written out as slots that alternate between the two.
// K/V units come from the operand-order copies written by the pooling kernel by LDS-direct loads into a K
// ring and a V ring (K(j) is read in iteration j - 1, V(j) in iteration j + 1), paced by explicit vmcnt
// counts; one barrier per iteration.
#include "s3r_attn_device.h"
#include "s3r_kernels.h"
#include <type_traits>

namespace s3r {

// P       : key units in work at a time, each by its own pair of waves (one wave per 32 query rows); with P > 1
//           a pair sees every P-th unit of the list, runs an online softmax of its own over them, and the P
//           partial results of each row group (m, l, O) are combined through LDS at the end:
//           m* = max_j m_j,  l* = sum_j l_j 2^(m_j - m*),  O = sum_j O_j 2^(m_j - m*) / l*
// NSK, NSV: stages of the K ring and of the V ring (a stage holds the K or V parts of an iteration's P units)
// AHEAD   : LDS operand reads run this many MFMAs ahead
template <int P, int NSK, int NSV, int AHEAD>
__global__ __launch_bounds__(128 * P, 2) void select_pipe_kernel(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ kb, const bf16_t *__restrict__ vb,
    const int32_t *__restrict__ idx, const float *__restrict__ o_comp, const bf16_t *__restrict__ gate,
    bf16_t *__restrict__ out, bf16_t *__restrict__ o_sel, float *__restrict__ lse, int64_t n_tok, int64_t n_blk,
    int heads, int kk, float scale_log2, int64_t n_sets, TokenMap qmap, int64_t n_keys, int64_t lse_stride,
    const int32_t *__restrict__ blk_len)
{
    constexpr int BLOCK = 64;
    constexpr int L = 8;                                  // 1 KiB chunks a wave requests per iteration
    constexpr int kHalfBytes = kUnitElems * 2;            // the K (or V) part of a unit: 8 KiB
    constexpr int kStageBytes = P * kHalfBytes;           // a ring stage
    constexpr int kAhead = AHEAD;
    constexpr int NW = 2 * P;                             // waves
    constexpr int kRingBytes = (NSK + NSV) * kStageBytes;  // K ring, then V ring
    constexpr int kCombineBytes = P > 1 ? NW * 32 * 64 * 4 + 2 * NW * 32 * 4 : 0;
    static_assert(P == 1 || P == 2 || P == 4, "the partners of a row group share its 32 accumulator registers evenly");
    static_assert(NSK >= 2 && NSV >= 2, "a stage being read and one being requested");
    static_assert(L * (NSK - 1) < 64 && L * (NSV - 1) < 64, "vmcnt budget");
    __shared__ __attribute__((aligned(1024))) unsigned char smem[kRingBytes > kCombineBytes ? kRingBytes : kCombineBytes];

    const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int h;
    int64_t set;
    {   // head-major, each XCD (workgroup id mod 8) takes a contiguous range of query blocks
        const int64_t bid = blockIdx.x;
        const int64_t per = (n_sets + 7) / 8;
        h = static_cast<int>(bid / (8 * per));
        const int64_t rr = bid % (8 * per);
        set = (rr % 8) * per + rr / 8;
        if (set >= n_sets) return;
    }
    const int r = wave & 1, p = wave >> 1;   // row group; which of an iteration's units
    const int64_t t = set * BLOCK + r * 32 + (lane & 31);
    bool row_valid = t < n_tok;
    if (blk_len != nullptr) row_valid = r * 32 + (lane & 31) < blk_len[set];  // spatial windows
    const int64_t trow = qmap.row(row_valid ? t : 0);

    const int32_t *sel = idx + (static_cast<int64_t>(h) * n_blk + set) * kk;
    const int n_units = kk;
    const int n_iter = (n_units + P - 1) / P;
    const int n_tiles = p < n_units ? (n_units - p + P - 1) / P : 0;  // units this pair of waves works on: p, p + P, ...
    const bf16_t *kb_h = kb + static_cast<int64_t>(h) * n_blk * BLOCK * 64;
    const bf16_t *vb_h = vb + static_cast<int64_t>(h) * n_blk * BLOCK * 64;
    const unsigned ring_base = static_cast<unsigned>(reinterpret_cast<size_t>(&smem[0]));

    // The index row (at most 128 entries) sits in two registers per lane, entry e in lane e % 64: looking one
    // up is a v_readlane, where a scalar load from memory would put its latency into every iteration.
    // (Loaded by inline asm that carries its own wait: a load the compiler knows of would get a vmcnt(0) of the
    // compiler's making in front of its uses inside the loop, where the LDS-direct loads are in flight.)
    int sel_lo, sel_hi;
    {
        const int32_t *a_lo = sel + (lane < kk ? lane : kk - 1);
        const int32_t *a_hi = sel + (lane + 64 < kk ? lane + 64 : kk - 1);
        asm volatile("global_load_dword %0, %2, off\n\t"
                     "global_load_dword %1, %3, off\n\t"
                     "s_waitcnt vmcnt(0)"
                     : "=&v"(sel_lo), "=&v"(sel_hi)
                     : "v"(a_lo), "v"(a_hi)
                     : "memory");
    }
    // (held into [0, n_blk): a caller's list is not trusted with the address arithmetic)
    sel_lo = sel_lo < 0 ? 0 : (sel_lo >= static_cast<int>(n_blk) ? static_cast<int>(n_blk) - 1 : sel_lo);
    sel_hi = sel_hi < 0 ? 0 : (sel_hi >= static_cast<int>(n_blk) ? static_cast<int>(n_blk) - 1 : sel_hi);
    auto unit_of = [&](int u) -> int { return __builtin_amdgcn_readlane(u < 64 ? sel_lo : sel_hi, u & 63); };

    // ---- loads: of its pair's units the first wave moves the K part, the second the V part (eight 1 KiB chunks)
    const bool is_k = r == 0;
    const bf16_t *my_src = is_k ? kb_h : vb_h;
    const unsigned my_ring = ring_base + (is_k ? 0u : static_cast<unsigned>(NSK * kStageBytes)) + p * kHalfBytes;
    const unsigned voff_lo = lane * 16, voff_hi = lane * 16 + 4096;
    // this pair's unit of iteration j into stage `stage` of this wave's ring
    auto issue_unit = [&](int j, int stage) {
        if (j < 0 || j >= n_tiles) return;
        const bf16_t *src = my_src + static_cast<int64_t>(unit_of(j * P + p)) * kUnitElems;   // wave-uniform
        const unsigned dst = my_ring + static_cast<unsigned>(stage) * kStageBytes;
        lds_dma_16_x4(src, voff_lo, dst);
        lds_dma_16_x4(src, voff_hi, dst + 4096);
    };
    // which of unit w's 64 keys exist (wave-uniform): with blocks that are runs of the sequence only its last
    // unit can be short; spatial windows have a length per block
    const int w_last = static_cast<int>((n_keys - 1) / kUnitKeys);
    const int left_last = static_cast<int>(n_keys - static_cast<int64_t>(w_last) * kUnitKeys);  // 1..64
    const unsigned long long tail_mask = left_last >= kUnitKeys ? ~0ull : (1ull << left_last) - 1ull;
    auto unit_mask = [&](int w) -> unsigned long long {
        if (blk_len == nullptr) return w == w_last ? tail_mask : ~0ull;
        const int left = blk_len[w];
        return left >= kUnitKeys ? ~0ull : left <= 0 ? 0ull : (1ull << left) - 1ull;
    };

    // K(j) is requested in iteration j - NSK (or before the loop), V(j) in iteration j + 2 - NSV: NSK - 1 and
    // NSV - 1 iterations before the barrier that needs them.
    for (int j = 0; j <= (is_k ? NSK - 2 : NSV - 4); ++j) issue_unit(j, j);
    // Q by inline asm with its own wait (which also covers the requests above), see sel_lo
    bf16x8 qb[4];
    {
        typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
        u32x4 q0, q1, q2, q3;
        const bf16_t *qrow = q + (trow * heads + h) * 64 + 8 * g;
        asm volatile("global_load_dwordx4 %0, %4, off\n\t"
                     "global_load_dwordx4 %1, %4, off offset:32\n\t"
                     "global_load_dwordx4 %2, %4, off offset:64\n\t"
                     "global_load_dwordx4 %3, %4, off offset:96\n\t"
                     "s_waitcnt vmcnt(0)"
                     : "=&v"(q0), "=&v"(q1), "=&v"(q2), "=&v"(q3)
                     : "v"(qrow)
                     : "memory");
        const u32x4 zero = {0u, 0u, 0u, 0u};
        qb[0] = __builtin_bit_cast(bf16x8, row_valid ? q0 : zero);
        qb[1] = __builtin_bit_cast(bf16x8, row_valid ? q1 : zero);
        qb[2] = __builtin_bit_cast(bf16x8, row_valid ? q2 : zero);
        qb[3] = __builtin_bit_cast(bf16x8, row_valid ? q3 : zero);
    }

    floatx16 oacc[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int x = 0; x < 16; ++x) oacc[dt][x] = 0.f;
    float m_run = -1e30f, l_run = 0.f;
    const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    floatx16 accs[2][2];  // scores, then probabilities, of unit j in accs[j & 1][32-key tile]
    bf16x8 ps[2][4];      // P(j) as MFMA operands in ps[j & 1][16-key step]
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        accs[a][0] = zero16;
        accs[a][1] = zero16;
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int e = 0; e < 8; ++e) ps[a][v][e] = static_cast<bf16_t>(0.f);
    }
    const bf16x2 ones = {static_cast<bf16_t>(1.f), static_cast<bf16_t>(1.f)};

    // keys that do not exist, then the running maximum: raised only when a unit exceeds it by more than the
    // slack (rare after the first unit).  A raise rescales what has been summed so far: the accumulators, the
    // row sum, and P(i - 1), whose product with V is still to come.
    auto soft_pre = [&](floatx16 (&acc)[2], bf16x8 (&p_pending)[4], unsigned long long vmask) __attribute__((always_inline)) {
        if (vmask != ~0ull) {
            asm volatile("" ::: "memory");  // keep this rare path a real branch
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int x = 0; x < 16; ++x)
                    if (!((vmask >> (mt * 32 + acc_row(lane, x))) & 1ull)) acc[mt][x] = -INFINITY;
        }
        float mx4[4];  // four independent chains instead of one of 32 dependent instructions
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            mx4[c] = acc[c >> 1][8 * (c & 1)];
#pragma unroll
            for (int x = 1; x < 8; ++x) mx4[c] = fmaxf(mx4[c], acc[c >> 1][8 * (c & 1) + x]);
        }
        const float mx = fmaxf(fmaxf(mx4[0], mx4[1]), fmaxf(mx4[2], mx4[3]));
        const float m_tile = max_with_other_half(mx) * scale_log2;
        const bool grow = m_tile > m_run + kRescaleSlack;
        if (__any(grow)) {
            const float m_new = grow ? m_tile : m_run;
            const float alpha = fast_exp2(m_run - m_new);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int x = 0; x < 16; ++x) oacc[dt][x] *= alpha;
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int e = 0; e < 8; ++e) p_pending[v][e] = static_cast<bf16_t>(static_cast<float>(p_pending[v][e]) * alpha);
        }
    };
    // Operand m of an iteration's 16 MFMAs, in order of need: m < 8 the K chunks of unit i + 1, the two
    // 32-key tiles taking turns so that no MFMA waits for the one issued just before it (chunk (m & 1) * 4 +
    // m / 2); then the 8 V chunks of unit i - 1.
    auto operand = [&](int m, const bf16_t *k_src, const bf16_t *v_src) __attribute__((always_inline)) -> bf16x8 {
        return *reinterpret_cast<const bf16x8 *>(m < 8 ? k_src + ((m & 1) * 4 + (m >> 1)) * 512 : v_src + (m - 8) * 512);
    };
    // The overlapped part of an iteration, written out as 8 groups of two MFMAs (the scores of the unit after,
    // then P.V of the unit before; each with the LDS read of the operand a few MFMAs ahead) and the vector
    // work on four score registers (four exponents, issued next to each other so that none waits for the
    // one before it, then their packs and sums), with scheduling fences so that the order stays as written.  rd[0..2] are read by the caller, before the softmax prologue, so that
    // their LDS latency runs under it.
    auto overlapped = [&](floatx16 (&acc)[2], floatx16 (&acc_next)[2], bf16x8 (&p_out)[4], const bf16x8 (&p_in)[4],
                          bf16x8 (&rd)[16], const bf16_t *k_src, const bf16_t *v_src) __attribute__((always_inline)) {
        float lsum[4] = {0.f, 0.f, 0.f, 0.f};
        auto mfma = [&](int m) __attribute__((always_inline)) {
            if (m < 8) acc_next[m & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rd[m], qb[m >> 1], m < 2 ? zero16 : acc_next[m & 1], 0, 0, 0);
            else oacc[m & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rd[m], p_in[(m - 8) >> 1], oacc[m & 1], 0, 0, 0);
            if (m + kAhead < 16) rd[m + kAhead] = operand(m + kAhead, k_src, v_src);
        };
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q4 = 0; q4 < 8; ++q4) {  // four score registers and two MFMAs per group
            const int mt = q4 >> 2, x0 = 4 * (q4 & 3);
            mfma(2 * q4);
            // independent instructions next to each other: four exponents, then their two packs and sums
            float e[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) e[c] = acc[mt][x0 + c] * scale_log2 - m_run;
#pragma unroll
            for (int c = 0; c < 4; ++c) e[c] = fast_exp2(e[c]);
            __builtin_amdgcn_sched_barrier(0);
            mfma(2 * q4 + 1);
#pragma unroll
            for (int c = 0; c < 4; c += 2) {
                const bf16x2 pr = {static_cast<bf16_t>(e[c]), static_cast<bf16_t>(e[c + 1])};
                const int x = x0 + c;
                p_out[2 * mt + (x >> 3)][x & 7] = pr[0];
                p_out[2 * mt + (x >> 3)][(x & 7) + 1] = pr[1];
                lsum[(q4 * 2 + (c >> 1)) & 3] = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, lsum[(q4 * 2 + (c >> 1)) & 3], false);
            }
            // nothing needs these values before the next barrier: tie them to this group, or the compiler
            // moves the vector work away from the MFMAs it is meant to overlap with
            asm volatile("" : "+v"(lsum[(q4 * 2) & 3]), "+v"(lsum[(q4 * 2 + 1) & 3]));
            if (q4 & 1) asm volatile("" : "+v"(p_out[2 * mt + (x0 >> 3)]));
            __builtin_amdgcn_sched_barrier(0);
        }
        l_run += (lsum[0] + lsum[1]) + (lsum[2] + lsum[3]);
    };
    // the same three phases one after the other, each only if its unit exists (first and last iterations)
    auto plain = [&](bool soft, bool pv, bool ss, floatx16 (&acc)[2], floatx16 (&acc_next)[2], bf16x8 (&p_out)[4],
                     bf16x8 (&p_in)[4], const bf16_t *k_src, const bf16_t *v_src, unsigned long long vmask) __attribute__((always_inline)) {
        if (soft) soft_pre(acc, p_in, vmask);
        if (pv) {
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                const bf16x8 va = *reinterpret_cast<const bf16x8 *>(v_src + m * 512);
                oacc[m & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, p_in[m >> 1], oacc[m & 1], 0, 0, 0);
            }
        }
        if (soft) {
            float lsum[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    const int mt = v >> 1, x = 8 * (v & 1) + e;
                    const bf16x2 pr = {static_cast<bf16_t>(fast_exp2(acc[mt][x] * scale_log2 - m_run)),
                                       static_cast<bf16_t>(fast_exp2(acc[mt][x + 1] * scale_log2 - m_run))};
                    p_out[v][e] = pr[0];
                    p_out[v][e + 1] = pr[1];
                    lsum[(e >> 1) & 3] = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, lsum[(e >> 1) & 3], false);
                }
            l_run += (lsum[0] + lsum[1]) + (lsum[2] + lsum[3]);
        }
        if (ss) {
#pragma unroll
            for (int m = 0; m < 8; ++m) {
                const bf16x8 ka = operand(m, k_src, v_src);
                acc_next[m & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qb[m >> 1], m < 2 ? zero16 : acc_next[m & 1], 0, 0, 0);
            }
        }
    };

    // Every iteration starts the same way: this wave's part of the unit that the coming reads need has landed
    // (the later ones may still be on their way; the count only holds while every unit up to the last one
    // assumed in flight exists), then the other wave's: the barrier also says both waves are done with
    // iteration i - 1, whose K stage and the V stage before it the next requests overwrite.
    // before iteration -1: K(-1 + NSK) goes to stage NSK - 1, V(NSV - 3) to stage (NSV - 3) mod NSV; K(0) is in
    // stage 0; V(-2) would be in stage (NSV - 2) mod NSV.  Each is stepped when an iteration opens.
    int st_issue = is_k ? NSK - 1 : (2 * NSV - 3) % NSV;
    int st_k = NSK - 1, st_v = (2 * NSV - 3) % NSV;   // one step before K(0)'s stage 0 and V(-2)'s stage
    auto open_iteration = [&](int i) __attribute__((always_inline)) {
        if (is_k) {
            if (i + NSK - 1 <= n_tiles - 1) wait_vmcnt<L *(NSK - 2)>(); else wait_vmcnt<0>();
        } else {
            if (i + NSV - 3 <= n_tiles - 1) wait_vmcnt<L *(NSV - 2)>(); else wait_vmcnt<0>();
        }
        lds_barrier();
        // K(i + NSK) goes where K(i) was, V(i + NSV - 2) where V(i - 2) was
        issue_unit(is_k ? i + NSK : i + NSV - 2, st_issue);
        st_issue = st_issue + 1 == (is_k ? NSK : NSV) ? 0 : st_issue + 1;
        st_k = st_k + 1 == NSK ? 0 : st_k + 1;
        st_v = st_v + 1 == NSV ? 0 : st_v + 1;
    };
    // (st_k, st_v: stages of K(i + 1) and V(i - 1) once iteration i is open)
    auto k_of = [&](int) -> const bf16_t * {
        return reinterpret_cast<const bf16_t *>(smem + st_k * kStageBytes + p * kHalfBytes) + lane * 8;
    };
    auto v_of = [&](int) -> const bf16_t * {
        return reinterpret_cast<const bf16_t *>(smem + (NSK + st_v) * kStageBytes + p * kHalfBytes) + lane * 8;
    };
    // an iteration in which all three phases have a unit: PAR = i & 1
    auto fast = [&](auto par_tag, int i) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par_tag)::value;
        open_iteration(i);
        const bf16_t *k_src = k_of(i), *v_src = v_of(i);
        bf16x8 rd[16];
#pragma unroll
        for (int m = 0; m < kAhead; ++m) rd[m] = operand(m, k_src, v_src);
        soft_pre(accs[PAR], ps[1 - PAR], unit_mask(unit_of(i * P + p)));
        overlapped(accs[PAR], accs[1 - PAR], ps[PAR], ps[1 - PAR], rd, k_src, v_src);
    };
    // the first and last iterations
    auto edge = [&](auto par_tag, int i) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par_tag)::value;
        open_iteration(i);
        const bool soft = i >= 0 && i < n_tiles, pv = i >= 1 && i <= n_tiles, ss = i + 1 < n_tiles;
        plain(soft, pv, ss, accs[PAR], accs[1 - PAR], ps[PAR], ps[1 - PAR], k_of(i), v_of(i),
              soft ? unit_mask(unit_of(i * P + p)) : ~0ull);
    };
    const std::integral_constant<int, 0> even{};
    const std::integral_constant<int, 1> odd{};
    edge(odd, -1);
    edge(even, 0);
    int i = 1;
    for (; i + 1 <= n_tiles - 2; i += 2) {  // iterations i and i + 1 have all three phases (1 <= i, i + 2 < n_tiles)
        fast(odd, i);
        fast(even, i + 1);
    }
    for (; i <= n_iter; i += 2) {  // (every wave runs all the iterations, and so all the barriers, of the workgroup)
        edge(odd, i);
        if (i + 1 <= n_iter) edge(even, i + 1);
    }

    // ---- the softmax over all selected keys from the P partial ones of each row group
    constexpr int kShare = 32 / P;           // accumulator registers each partner adds up and writes
    float osum[kShare];
    float m_all = m_run, l_all = sum_with_other_half(l_run);
    if constexpr (P == 1) {
#pragma unroll
        for (int x = 0; x < 32; ++x) osum[x] = oacc[x >> 4][x & 15];
    } else {
        float *mbuf = reinterpret_cast<float *>(smem);   // [NW][32]
        float *lbuf = mbuf + NW * 32;                    // [NW][32]
        float *obuf = lbuf + NW * 32;                    // [NW][32 registers][64 lanes]
        lds_barrier();                                   // every wave is done with the rings
        if (lane < 32) {
            mbuf[wave * 32 + lane] = m_run;
            lbuf[wave * 32 + lane] = l_all;
        }
        lds_barrier();
        m_all = -1e30f;
#pragma unroll
        for (int j = 0; j < P; ++j) m_all = fmaxf(m_all, mbuf[(2 * j + r) * 32 + (lane & 31)]);
        l_all = 0.f;
#pragma unroll
        for (int j = 0; j < P; ++j) l_all += lbuf[(2 * j + r) * 32 + (lane & 31)] * fast_exp2(mbuf[(2 * j + r) * 32 + (lane & 31)] - m_all);
        const float f_own = fast_exp2(m_run - m_all);
#pragma unroll
        for (int x = 0; x < 32; ++x) obuf[(wave * 32 + x) * 64 + lane] = oacc[x >> 4][x & 15] * f_own;
        lds_barrier();
#pragma unroll
        for (int x = 0; x < kShare; ++x) osum[x] = 0.f;
#pragma unroll
        for (int j = 0; j < P; ++j)
#pragma unroll
            for (int x = 0; x < kShare; ++x) osum[x] += obuf[((2 * j + r) * 32 + p * kShare + x) * 64 + lane];
    }
    if (!row_valid) return;
    const float inv = l_all > 0.f ? 1.f / l_all : 0.f;
    if (lse != nullptr && g == 0 && p == 0) lse[static_cast<int64_t>(h) * lse_stride + trow] = (m_all + __builtin_log2f(l_all)) * kLn2;
    const int64_t o = (trow * heads + h) * 64;
    const float *oc = (o_comp != nullptr) ? o_comp + (static_cast<int64_t>(h) * n_blk + set) * 64 : nullptr;
#pragma unroll
    for (int x4 = 0; x4 < kShare / 4; ++x4) {
        {
            const int reg = p * kShare + 4 * x4;         // accumulator register dt * 16 + 4 r4 (+ e)
            const int dt = reg >> 4, r4 = (reg & 15) >> 2;
            const int d0 = 32 * dt + 8 * r4 + 4 * g;
            float os[4], res[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) res[e] = os[e] = osum[4 * x4 + e] * inv;
            if (oc != nullptr) {
                const floatx4 c4 = *reinterpret_cast<const floatx4 *>(oc + d0);
                float gt[4] = {0.5f, 0.5f, 0.5f, 0.5f};
                if (gate != nullptr) {
                    const bf16x4 gl = *reinterpret_cast<const bf16x4 *>(gate + o + d0);
#pragma unroll
                    for (int e = 0; e < 4; ++e) gt[e] = 1.f / (1.f + __expf(-static_cast<float>(gl[e])));
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) res[e] = gt[e] * c4[e] + (1.f - gt[e]) * os[e];
            }
            bf16x4 ro;
#pragma unroll
            for (int e = 0; e < 4; ++e) ro[e] = static_cast<bf16_t>(res[e]);
            *reinterpret_cast<bf16x4 *>(out + o + d0) = ro;
            if (o_sel != nullptr) {
#pragma unroll
                for (int e = 0; e < 4; ++e) ro[e] = static_cast<bf16_t>(os[e]);
                *reinterpret_cast<bf16x4 *>(o_sel + o + d0) = ro;
            }
        }
    }
}

template <int P, int NSK, int NSV, int AHEAD>
static hipError_t run_pipe(const SelectArgs &a, hipStream_t stream)
{
    const int64_t sets = a.n_blk;
    const int64_t grid = (sets + 7) / 8 * 8 * a.heads;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((select_pipe_kernel<P, NSK, NSV, AHEAD>), dim3(static_cast<unsigned>(grid)), dim3(128 * P), 0, stream,
                       static_cast<const bf16_t *>(a.q), static_cast<const bf16_t *>(a.kb),
                       static_cast<const bf16_t *>(a.vb), a.idx, a.o_comp, static_cast<const bf16_t *>(a.gate),
                       static_cast<bf16_t *>(a.out), static_cast<bf16_t *>(a.o_sel), a.lse, a.n_tok, a.n_blk, a.heads,
                       a.kk, a.scale * kLog2e, sets, a.qmap, a.n_keys, a.lse_stride, a.blk_len);
    return hipGetLastError();
}

// Plain selection (index rows of at most 128 blocks, packed q, per-block compressed outputs) for bf16 blocks
// of 64 tokens.
hipError_t launch_select_pipe(const SelectArgs &a, hipStream_t stream)
{
    if (!a.is_bf16 || a.kb == nullptr || a.vb == nullptr || a.idx == nullptr) return hipErrorInvalidValue;
    if (a.n_keys != a.n_tok || a.n_keys2 != 0 || a.kk < 1 || a.kk > 128 || a.block != 64) return hipErrorInvalidValue;
    if (a.x.o_comp_tok != nullptr || a.x.in.tok != 0) return hipErrorInvalidValue;
    if (a.qmap.period != 0 && a.n_tok > 0x7fffffffLL) return hipErrorInvalidValue;
    // Measured on MI355X (1000 views x 1374 tokens, 16 heads, clustered keys; ms of this kernel for 8 / 16 / 32 /
    // 48 / 64 / 96 blocks per row): one pair of waves per query block, four workgroups per CU 5.2 / 9.1 / 18.5 /
    // 29.1 / 39.7 / 61.4; two pairs, two workgroups per CU 6.3 / 10.3 / 18.4 / 26.7 / 35.2 / 54.5 (the kernel
    // of select_mfma.hip, five workgroups per CU: 5.6 / 10.1 / 19.2 / 28.5 / 38.5 / 59.3).  Long rows on long
    // sequences are bound by the arrival of K/V units and gain from fewer query blocks in progress; short rows
    // and short sequences (100 views: one pair is 5 to 10 % ahead at every row length) from more of them.
    if (a.kk >= 40 && a.n_blk >= 3000) return run_pipe<2, 2, 2, 3>(a, stream);
    return run_pipe<1, 2, 2, 3>(a, stream);
}

}  // namespace s3r
