// Selection attention + merge (Sec. 3.2 eq. 6, supplementary Alg. 2; eqs. 5, 7, 8) and dense
// attention (eq. 2 form) on bf16 MFMA for gfx950.
//
// Work layout.  A wave owns 32 query rows and keeps their Q operands in registers.  Keys are
// processed in UNITS of 64 tokens (one key block of 64, or half a key block of 128).  Per unit the
// wave computes the TRANSPOSED score tile S^T[key][query] = K Q^T with v_mfma_f32_32x32x16_bf16
// (A = K rows from LDS, B = Q^T registers), so a lane holds keys of ONE query: the online-softmax
// row max / row sum are in-lane reductions plus one exchange with the lane 32 positions away, and
// the probabilities already sit in the register order of the B operand of the next MFMA,
// O^T = V^T P^T (A = V^T from LDS).
//
// Data movement.  K and V units come from the operand-order copies written by the pooling kernel:
// each unit is two contiguous 8 KiB runs in HBM.  They are copied HBM -> LDS by the LDS-direct
// load (global_load_lds_dwordx4: lane L's 16 bytes land at M0 + 16 L, so one instruction moves one
// contiguous KiB and the LDS image is already in ds_read_b128 operand order); no registers and no
// ds_write are spent on staging.  A ring of NS LDS stages keeps NS - 1 units in flight per
// workgroup, paced by explicit s_waitcnt vmcnt counts (loads return in order) and one barrier per
// unit.  This matters because the gather of 16 KiB pieces is latency-bound otherwise.
//
// Bound.  At block 64 every (query block, selected block) pair moves 16 KiB for 1 MFLOP: the kernel
// runs at the rate at which the memory fabric delivers L2 misses (about 7 TB/s for scattered 16 KiB
// pieces on MI355X, whether they come from HBM or from the Infinity Cache), not at the MFMA rate.
// Letting one workgroup serve several neighbouring query blocks from a merged list was measured
// and brings nothing: the work mapping already runs neighbours on the same XCD at the same time,
// so their shared key blocks hit in that XCD's L2.
//
// Softmax.  The running row maximum is only raised when a unit exceeds it by more than
// kRescaleSlack (log2 units), so the rescale of the output accumulators is skipped for almost every
// unit; probabilities then range up to 2^kRescaleSlack, which fp32 sums and bf16 operands carry as
// well as values below 1, and the final normalisation uses the same maximum: plain softmax.
#include "s3r_device.h"
#include "s3r_attn_device.h"
#include "s3r_kernels.h"

namespace s3r {

// QW    : waves per workgroup = query rows / 32 (block / 32 for selection: one query block)
// DENSE : every key unit instead of an index list
// NS    : LDS stages of the unit ring
// SMALL : key blocks of 16 or 32 tokens (4 x 4 spatial windows and the like): a 64-key unit is put
//         together from 4 or 2 blocks, each lane of an LDS-direct load fetching its 16 bytes from the
//         block its unit row belongs to (the pooling kernel stores such blocks as small tiles in the
//         same operand order), and a query block fills only the first `block` of a wave's 32 query
//         columns.  At 16 FLOP per byte of K/V such blocks are bound by the gather alone, so the
//         empty MFMA columns cost nothing.
// EXTRA : the rarely used arguments of SelectExtras are honoured (a second instantiation, so that the plain
//         path carries none of their instructions: they cost the selection kernel 2.4 % when always compiled in)
// ASMQ  : Q is loaded by inline asm after the first unit requests instead of by plain loads (see below)
// PAIR  : selection with blocks of 64 tokens, QW = 4: one workgroup takes two neighbouring query blocks (two
//         waves each) and walks the union of their two index lists, merged on the fly; a key block both
//         lists hold is fetched into LDS once for both, and a pair of waves sits out the units only the
//         other pair's list holds.  For long lists that are mostly common to all query blocks (forced
//         blocks), where the traffic from the L2s into LDS is what binds.
// PROBE : measurement only.  The kernel walks its index list and moves every K/V unit into LDS exactly as the
//         real one does (same work mapping, ring, waits and barriers) but does no arithmetic on them; it
//         writes its Q rows to `out`, so Q is read and `out` written as well.  Its run time is what the data
//         movement of the selection stage costs by itself.
// F32   : fp32 q, gate, out and o_sel (the pointers below are then float pointers in disguise), K/V tiles in bf16
//         parts ([hi tiles | lo tiles | K only: lo2 tiles], lo_off elements apart), x = hi + lo (+ lo2).  Scores
//         take Q and K in three parts each and the six products whose weight is above 2^-24 (a logit's error
//         enters the result in absolute terms, so it must not grow with the size of the entries); P.V takes
//         two parts each, hi.hi + hi.lo + lo.hi (2^-17 relative, of values in [0, 1] times V).  All on the
//         bf16 matrix pipe with fp32 accumulation: fp32-grade results at nine MFMAs per tile step in place of two.
template <int QW, bool DENSE, int NS, bool SMALL, bool EXTRA, bool ASMQ, bool PAIR = false, bool PROBE = false,
          bool F32 = false>
__global__ __launch_bounds__(QW * 64, 2) void select_mfma_kernel(
    const bf16_t *__restrict__ q, const bf16_t *__restrict__ kb, const bf16_t *__restrict__ vb,
    const int32_t *__restrict__ idx, const float *__restrict__ o_comp, const bf16_t *__restrict__ gate,
    bf16_t *__restrict__ out, bf16_t *__restrict__ o_sel, float *__restrict__ lse, int64_t n_tok,
    int64_t n_blk, int heads, int block, int kk, float scale_log2, int64_t set_offset, int64_t n_sets,
    int map_mode, TokenMap qmap, int64_t n_keys, int64_t lse_stride, const bf16_t *__restrict__ kb2,
    const bf16_t *__restrict__ vb2, int64_t n_keys2, const int32_t *__restrict__ blk_len, SelectExtras x,
    int64_t lo_off, int64_t lo_off2)
{
    constexpr int NW = QW;             // waves per workgroup
    constexpr int NCH = F32 ? 40 : 16; // 1 KiB chunks of a unit: 8 K + 8 V (F32: then 8 K lo + 8 V lo + 8 K lo2)
    constexpr int CPW = NCH / NW;      // ... issued by each wave
    constexpr int D = NS - 1;          // units in flight
    static_assert(NCH % NW == 0 && 16 % NW == 0, "waves must split the chunks of a unit evenly");
    static_assert(CPW * D < 64, "vmcnt budget");
    static_assert(!F32 || (!PAIR && !PROBE), "operand parts: the plain and the dense kernels");
    // [stage][K 8 KiB | V 8 KiB] (F32: then [K lo 8 KiB | V lo 8 KiB | K lo2 8 KiB])
    constexpr int kStageParts = F32 ? 5 : 2;
    __shared__ __attribute__((aligned(1024))) bf16_t ring[NS][kStageParts * kUnitElems];
    constexpr int kLoElems = 2 * kUnitElems;  // from a hi part of a stage to its lo part, and on to K's lo2 part

    const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int h;
    int64_t set;    // query group (query block for selection) of this workgroup
    int split = 0;  // dense attention in key splits: which share of the key units
    {
        const int64_t bid = blockIdx.x;
        if (map_mode == 0) {  // head fastest
            h = static_cast<int>(bid % heads);
            set = bid / heads;
            if constexpr (EXTRA && DENSE) {  // then the key splits of a query group
                if (x.n_split > 1) {
                    split = static_cast<int>(set % x.n_split);
                    set /= x.n_split;
                }
            }
        } else {  // head-major, each XCD (workgroup id mod 8) takes a contiguous range of sets
            const int64_t per = (n_sets + 7) / 8;
            h = static_cast<int>(bid / (8 * per));
            const int64_t r = bid % (8 * per);
            set = (r % 8) * per + r / 8;
            if (set >= n_sets) return;
        }
        set += set_offset;
    }
    const int upb_shift = SMALL ? 0 : block / kUnitKeys - 1;  // units per key block: 1 or 2, as a shift
    const int upb_mask = (1 << upb_shift) - 1;
    const int bpu_shift = SMALL ? (block == 16 ? 2 : 1) : 0;  // SMALL: blocks per unit: 4 or 2, as a shift
    const int64_t qgroup = set;
    int64_t t = qgroup * (32 * QW) + wave * 32 + (lane & 31);
    bool row_valid = t < n_tok;
    if constexpr (SMALL && !DENSE) {  // one query block of `block` rows per wave
        t = qgroup * block + (lane & 31);
        row_valid = (lane & 31) < block && t < n_tok;
    }
    if (!DENSE && !PAIR && blk_len != nullptr) row_valid = wave * 32 + (lane & 31) < blk_len[qgroup];  // spatial windows
    if constexpr (PAIR) {
        static_assert(!PAIR || (QW == 4 && !DENSE && !SMALL && ASMQ), "two query blocks of 64 rows, two waves each");
        const int64_t qblk = 2 * qgroup + (wave >> 1);
        t = qblk * 64 + (wave & 1) * 32 + (lane & 31);
        row_valid = t < n_tok;
        if (blk_len != nullptr) row_valid = qblk < n_blk && (wave & 1) * 32 + (lane & 31) < blk_len[qblk];
    }
    if constexpr (EXTRA && DENSE)
        if (x.q_blk_len != nullptr && row_valid) row_valid = t % x.q_block < x.q_blk_len[t / x.q_block];
    const int64_t trow = qmap.row(row_valid ? t : 0);  // the caller's row of this query
    // Q.  Dense attention (rings of three stages, two units on their way while one is worked on) loads it with
    // inline-asm loads that carry their wait in the same statement: the compiler does not count the LDS-direct
    // loads of the key units, so a wait of its own for a load it knows of comes out as vmcnt(0), and with Q
    // loaded in plain code that wait lands in front of the first MFMA of the loop, in every iteration, where it
    // holds each unit back until the requests for the units after it have landed too (3.6 % of the dense
    // kernel's time).  That load is issued once the first units have been requested (its wait covers them as
    // well); rows that do not exist read row 0.  The selection kernels wait for every load at the head of
    // each step anyway (two stages), and a plain early load of Q is 1 % faster there, except on long index
    // rows (ASMQ chooses).
    bf16x8 qb[4];
    bf16x8 ql[F32 ? 4 : 1], ql2[F32 ? 4 : 1];   // F32: the lo and lo2 parts of Q
    constexpr bool kAsmQ = ASMQ && !F32;
    if constexpr (F32) {
        const float *qf = reinterpret_cast<const float *>(q);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            float f[8];
            if (row_valid) {
                const int64_t qo = EXTRA ? x.in.at(trow, h, heads) : (trow * heads + h) * 64;
                const floatx4 a = *reinterpret_cast<const floatx4 *>(qf + qo + 16 * s + 8 * g);
                const floatx4 b = *reinterpret_cast<const floatx4 *>(qf + qo + 16 * s + 8 * g + 4);
#pragma unroll
                for (int i = 0; i < 4; ++i) { f[i] = a[i]; f[4 + i] = b[i]; }
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) f[i] = 0.f;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                qb[s][i] = static_cast<bf16_t>(f[i]);
                const float r1 = f[i] - static_cast<float>(qb[s][i]);
                ql[s][i] = static_cast<bf16_t>(r1);
                ql2[s][i] = static_cast<bf16_t>(r1 - static_cast<float>(ql[s][i]));
            }
        }
    } else if constexpr (!kAsmQ) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (row_valid) {
                const int64_t qo = EXTRA ? x.in.at(trow, h, heads) : (trow * heads + h) * 64;
                qb[s] = *reinterpret_cast<const bf16x8 *>(q + qo + 16 * s + 8 * g);
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) qb[s][i] = static_cast<bf16_t>(0.f);
            }
        }
    }
    auto load_q_dense = [&]() __attribute__((always_inline)) {
        typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
        u32x4 q0, q1, q2, q3;
        const int64_t qo = EXTRA ? x.in.at(trow, h, heads) : (trow * heads + h) * 64;
        const bf16_t *qrow = q + qo + 8 * g;
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
    };
    const int64_t n_units1 = SMALL ? (n_blk + (1 << bpu_shift) - 1) >> bpu_shift
                                   : (n_keys + kUnitKeys - 1) / kUnitKeys;  // units of the first key segment
    const int64_t n_units2 = (n_keys2 + kUnitKeys - 1) / kUnitKeys;    // dense only: second segment

    // ---- the list of key blocks this workgroup visits ---------------------------------------
    int n_steps;  // units to process (host side keeps this below 2^31)
    int u_begin = 0;  // dense attention: first unit
    const int32_t *sel = nullptr;
    if constexpr (DENSE) {
        n_steps = static_cast<int>(n_units1 + n_units2);
        if constexpr (EXTRA && !SMALL) {  // key splits: units [u_begin, u_begin + n_steps)
            if (x.n_split > 1) {
                const int64_t u_all = n_units1 + n_units2;
                u_begin = static_cast<int>(u_all * split / x.n_split);
                n_steps = static_cast<int>(u_all * (split + 1) / x.n_split) - u_begin;
            }
        }
    } else {
        sel = idx + (static_cast<int64_t>(h) * n_blk + (PAIR ? 2 * qgroup : qgroup)) * kk;
        n_steps = SMALL ? (kk + (1 << bpu_shift) - 1) >> bpu_shift : kk << upb_shift;
    }
    // An entry of the index list, held into [0, n_blk): the lists of the library's own TopK are always in range,
    // a caller's (speed3r_select_attn) are not trusted with the address arithmetic.
    auto sel_at = [&](const int32_t *list, int pos) -> int {
        const int j = list[pos];
        return j < 0 ? 0 : (j >= static_cast<int>(n_blk) ? static_cast<int>(n_blk) - 1 : j);
    };
    // SMALL: the c-th key block of unit s, or -1 past the end of the list
    auto block_at = [&](int s, int c) -> int {
        const int pos = (s << bpu_shift) + c;
        if constexpr (DENSE) return pos < n_blk ? pos : -1;
        else return pos < kk ? sel_at(sel, pos) : -1;
    };
    auto block_tokens = [&](int j) -> int {  // tokens of key block j (j >= 0)
        if (blk_len != nullptr) return blk_len[j];
        const int64_t left = n_keys - static_cast<int64_t>(j) * block;
        return static_cast<int>(left < block ? left : block);
    };

    const int64_t kv_head_stride = (EXTRA && x.kv_head_stride != 0) ? x.kv_head_stride : n_blk * block * 64;
    const bf16_t *kb_h = kb + static_cast<int64_t>(h) * kv_head_stride;
    const bf16_t *vb_h = vb + static_cast<int64_t>(h) * kv_head_stride;
    const bf16_t *kb2_h = DENSE ? kb2 + static_cast<int64_t>(h) * n_units2 * kUnitElems : nullptr;
    const bf16_t *vb2_h = DENSE ? vb2 + static_cast<int64_t>(h) * n_units2 * kUnitElems : nullptr;
    const unsigned ring_base = static_cast<unsigned>(reinterpret_cast<size_t>(&ring[0][0]));
    const bool wave_k = wave * CPW < 8;              // plain units: this wave copies K chunks (else V chunks)
    const bf16_t *seg1 = wave_k ? kb_h : vb_h;       // ... of the first key segment
    const bf16_t *seg2 = wave_k ? kb2_h : vb2_h;     // ... of the second (dense only)

    // step s -> key unit (global unit index); 32-bit arithmetic: these run once per step on the scalar unit
    auto unit_of = [&](int s) -> int {
        if constexpr (DENSE) return (EXTRA && !SMALL) ? s + u_begin : s;
        else return (sel_at(sel, s >> upb_shift) << upb_shift) + (s & upb_mask);
    };
    // SMALL: the blocks a 64-key unit is put together from; missing ones (short last unit) point at the
    // first, and are masked
    struct UnitBlocks { int b0, b1, b2, b3; };
    auto blocks_of = [&](int s) -> UnitBlocks {
        const int f0 = block_at(s, 0);
        int b1 = block_at(s, 1), b2 = -1, b3 = -1;
        if (bpu_shift == 2) { b2 = block_at(s, 2); b3 = block_at(s, 3); }
        return UnitBlocks{f0, b1 >= 0 ? b1 : f0, b2 >= 0 ? b2 : f0, b3 >= 0 ? b3 : f0};
    };
    auto issue = [&](int s, int stage) {  // this wave's share of unit s -> LDS stage `stage`
        const unsigned stage_byte = ring_base + static_cast<unsigned>(stage) * (kStageParts * kUnitElems * 2);
        if constexpr (SMALL) {
            // (dense: the second key segment is stored as plain 64-key units)
            const bool small = !(DENSE && s >= n_units1);
            const UnitBlocks b = blocks_of(small ? s : 0);
            const int64_t tile = static_cast<int64_t>(block) * 64;  // elements of a block's K (or V) tile
            // Chunk c * QW + wave for c = 0 .. CPW - 1: the tile half mt a chunk belongs to is then a
            // compile-time constant (chunks 0..7 = K (mt, channel step), 8..15 = V (v = 2 mt + hw, dt)),
            // which keeps the block numbers in registers.
            static_assert(QW == 1 || QW == 2 || QW == 4, "chunk distribution");
#pragma unroll
            for (int c = 0; c < CPW; ++c) {
                const int base = c * QW;                 // compile time
                const int chunk = base + wave;           // base .. base + QW - 1, all in the same mt
                const int mt = (base & 7) >> 2;          // compile time
                const bool is_k = (base & 15) < 8;       // compile time (F32: 16 chunks per operand part, K only in the third)
                const int64_t part = F32 ? (base >> 4) * (small ? lo_off : lo_off2) : 0;
                const bf16_t *src;
                if (small) {
                    const int lo = mt == 0 ? b.b0 : (bpu_shift == 2 ? b.b2 : b.b1);   // first block of tile half mt
                    const int hi = mt == 0 ? b.b1 : b.b3;                              // block 16 only: its second block
                    if (is_k) {
                        const int cs = chunk & 3;
                        if (bpu_shift == 1) {  // block 32: the 32-row tile of block mt
                            src = kb_h + lo * tile + cs * 512 + lane * 8;
                        } else {               // block 16: rows 0..15 of the tile from its first block, rows 16..31 from its second
                            const int blk = ((lane >> 4) & 1) ? hi : lo;
                            src = kb_h + blk * tile + ((cs * 2 + (lane >> 5)) * 16 + (lane & 15)) * 8;
                        }
                    } else {
                        const int hw = ((chunk & 7) >> 1) & 1, dt = chunk & 1;
                        if (bpu_shift == 1) src = vb_h + lo * tile + ((hw * 2 + dt) * 64 + lane) * 8;
                        else src = vb_h + (hw ? hi : lo) * tile + (dt * 64 + lane) * 8;
                    }
                } else {
                    const int64_t w2 = s - n_units1;
                    src = (is_k ? kb2_h : vb2_h) + w2 * kUnitElems + (chunk & 7) * 512 + lane * 8;
                }
                lds_dma_16(src + part, __builtin_amdgcn_readfirstlane(stage_byte + chunk * 1024));
            }
            return;
        }
        const int64_t w = unit_of(s);
        if constexpr (F32) {  // chunk = 16 * part + (0..7: K, 8..15: V), part 0 = hi, 1 = lo, 2 = lo2 (K only)
            const bool second = DENSE && w >= n_units1;
            const int64_t wu = second ? w - n_units1 : w;
#pragma unroll
            for (int c = 0; c < CPW; ++c) {
                const int chunk = wave * CPW + c;
                const bf16_t *arr = (chunk & 8) ? (second ? vb2_h : vb_h) : (second ? kb2_h : kb_h);
                const int64_t part = (chunk >> 4) * (second ? lo_off2 : lo_off);
                lds_dma_16(arr + part + wu * kUnitElems + (chunk & 7) * 512 + lane * 8,
                           __builtin_amdgcn_readfirstlane(stage_byte + chunk * 1024));
            }
            return;
        }
        // all chunks of a wave are of one kind (K or V) here
        static_assert(SMALL || F32 || CPW <= 8, "a wave's chunks must be all K or all V");
        const bf16_t *unit = (DENSE && w >= n_units1) ? seg2 + (w - n_units1) * kUnitElems : seg1 + w * kUnitElems;
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            const int chunk = wave * CPW + c;  // 0..7: K, 8..15: V
            lds_dma_16(unit + (chunk & 7) * 512 + lane * 8, __builtin_amdgcn_readfirstlane(stage_byte + chunk * 1024));
        }
    };

    floatx16 oacc[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
    float m_run = -1e30f, l_run = 0.f;

    // which of unit s's 64 keys exist (wave-uniform)
    auto unit_mask = [&](int s) -> unsigned long long {
        if (SMALL && !(DENSE && s >= n_units1)) {
            unsigned long long vm = 0ull;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (c < (1 << bpu_shift)) {
                    const int j = block_at(s, c);
                    const int len = j >= 0 ? block_tokens(j) : 0;
                    vm |= ((1ull << len) - 1ull) << (c * block);
                }
            return vm;
        }
        const int64_t w = unit_of(s);
        int64_t left;
        if (DENSE && w >= n_units1) left = n_keys2 - (w - n_units1) * kUnitKeys;
        else if (blk_len != nullptr) left = blk_len[w >> upb_shift] - (static_cast<int>(w) & upb_mask) * kUnitKeys;  // wave-uniform load
        else left = n_keys - w * kUnitKeys;
        return left >= kUnitKeys ? ~0ull : left <= 0 ? 0ull : (1ull << left) - 1ull;
    };

    floatx16 sacc[2];
    bf16x8 pb[4];  // probabilities of one unit as MFMA operands
    bf16x8 pl[F32 ? 4 : 1];  // F32: their lo parts
    const floatx16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // S^T = K Q^T of the unit whose K sits in `ks`.  Selection: the two 32-key tiles take turns, so that
    // no MFMA waits for the one issued just before it (3 % faster at 64 blocks per row, 7 % at 288).
    // Dense attention: one tile after the other; alternating takes a few registers more there, which
    // costs a workgroup per CU (15 % slower), and with the register count capped the two orders tie.
    auto scores = [&](const bf16_t *ks) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int mt = DENSE ? i >> 2 : i & 1, c = DENSE ? i & 3 : i >> 1;
            const bf16x8 ka = *reinterpret_cast<const bf16x8 *>(ks + ((mt * 4 + c) * 64 + lane) * 8);
            sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qb[c], c == 0 ? zero16 : sacc[mt], 0, 0, 0);
            if constexpr (F32) {
                const bf16x8 kl = *reinterpret_cast<const bf16x8 *>(ks + kLoElems + ((mt * 4 + c) * 64 + lane) * 8);
                const bf16x8 kl2 = *reinterpret_cast<const bf16x8 *>(ks + 2 * kLoElems + ((mt * 4 + c) * 64 + lane) * 8);
                sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, ql[c], sacc[mt], 0, 0, 0);
                sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kl, qb[c], sacc[mt], 0, 0, 0);
                sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, ql2[c], sacc[mt], 0, 0, 0);
                sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kl, ql[c], sacc[mt], 0, 0, 0);
                sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kl2, qb[c], sacc[mt], 0, 0, 0);
            }
        }
    };
    // keys past the end of a block or of the sequence do not exist
    auto mask_scores = [&](unsigned long long vmask) __attribute__((always_inline)) {
        asm volatile("" ::: "memory");    // keep this rare path a real branch
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (!((vmask >> (mt * 32 + acc_row(lane, r))) & 1ull)) sacc[mt][r] = -INFINITY;
    };
    // the running maximum after a unit whose largest score (per lane) is mx
    auto raise_max = [&](float mx) __attribute__((always_inline)) {
        const float m_tile = max_with_other_half(mx) * scale_log2;
        const bool grow = m_tile > m_run + kRescaleSlack;
        if (__any(grow)) {  // rare after the first unit: raise the maximum, rescale the accumulators
            const float m_new = grow ? m_tile : m_run;
            const float alpha = fast_exp2(m_run - m_new);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
        }
    };
    // online softmax of sacc[X] -> pb[X]
    auto softmax = [&](unsigned long long vmask) __attribute__((always_inline)) {
        if (vmask != ~0ull) mask_scores(vmask);
        float mx = sacc[0][0];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[mt][r]);
        raise_max(mx);
        // The row sum adds the probabilities as the MFMA will see them (rounded to bf16), two per
        // v_dot2_f32_bf16 with a vector of ones: half the instructions of fp32 adds, and numerator and
        // denominator of the softmax then carry the same rounding.
        float lsum[4] = {0.f, 0.f, 0.f, 0.f};
        if constexpr (F32) {  // probabilities in fp32, split into operand pairs; the row sum adds the fp32 values
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int mt = v >> 1, r = 8 * (v & 1) + i;
                    const float p = fast_exp2(sacc[mt][r] * scale_log2 - m_run);
                    lsum[i & 3] += p;
                    pb[v][i] = static_cast<bf16_t>(p);
                    pl[v][i] = static_cast<bf16_t>(p - static_cast<float>(pb[v][i]));
                }
            l_run += (lsum[0] + lsum[1]) + (lsum[2] + lsum[3]);
            return;
        }
        const bf16x2 ones = {static_cast<bf16_t>(1.f), static_cast<bf16_t>(1.f)};
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int i = 0; i < 8; i += 2) {
                const int mt = v >> 1, r = 8 * (v & 1) + i;
                const bf16x2 pr = {static_cast<bf16_t>(fast_exp2(sacc[mt][r] * scale_log2 - m_run)),
                                   static_cast<bf16_t>(fast_exp2(sacc[mt][r + 1] * scale_log2 - m_run))};
                lsum[(i >> 1) & 3] = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, lsum[(i >> 1) & 3], false);
                pb[v][i] = pr[0];
                pb[v][i + 1] = pr[1];
            }
        l_run += (lsum[0] + lsum[1]) + (lsum[2] + lsum[3]);
    };
    // O^T += V^T P^T for the unit whose V sits in `vs`
    auto accumulate = [&](const bf16_t *vs) __attribute__((always_inline)) {
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                const bf16x8 va = *reinterpret_cast<const bf16x8 *>(vs + ((v * 2 + dt) * 64 + lane) * 8);
                oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[v], oacc[dt], 0, 0, 0);
                if constexpr (F32) {
                    const bf16x8 vl = *reinterpret_cast<const bf16x8 *>(vs + kLoElems + ((v * 2 + dt) * 64 + lane) * 8);
                    oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pl[v], oacc[dt], 0, 0, 0);
                    oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vl, pb[v], oacc[dt], 0, 0, 0);
                }
            }
    };

    if constexpr (PAIR) {
        // Two ascending lists -> their ascending union.  A cursor holds the position and the entry it looks
        // at in either list; one cursor runs D units ahead and requests the loads, the other consumes.
        constexpr int kEnd = 0x7fffffff;
        const int32_t *sel_b = sel + kk;
        const bool has_b = 2 * qgroup + 1 < n_blk;
        struct Cursor { int ia, ib, ja, jb; };
        auto start = [&]() -> Cursor {
            return Cursor{0, 0, kk > 0 ? sel_at(sel, 0) : kEnd, (has_b && kk > 0) ? sel_at(sel_b, 0) : kEnd};
        };
        // next unit of the union (kEnd when done); ua / ub: list A / B holds it
        auto next = [&](Cursor &c, bool &ua, bool &ub) -> int {
            const int j = c.ja < c.jb ? c.ja : c.jb;
            ua = c.ja == j;
            ub = c.jb == j;
            if (j == kEnd) return kEnd;
            if (ua) { ++c.ia; c.ja = c.ia < kk ? sel_at(sel, c.ia) : kEnd; }
            if (ub) { ++c.ib; c.jb = c.ib < kk ? sel_at(sel_b, c.ib) : kEnd; }
            return j;
        };
        auto issue_unit = [&](int64_t w, int stage) {  // this wave's share of unit w -> LDS stage `stage`
            const unsigned stage_byte = ring_base + static_cast<unsigned>(stage) * (2 * kUnitElems * 2);
            const bf16_t *unit = seg1 + w * kUnitElems;
#pragma unroll
            for (int c = 0; c < CPW; ++c) {
                const int chunk = wave * CPW + c;  // 0..7: K, 8..15: V
                lds_dma_16(unit + (chunk & 7) * 512 + lane * 8, __builtin_amdgcn_readfirstlane(stage_byte + chunk * 1024));
            }
        };
        auto unit_mask_of = [&](int64_t w) -> unsigned long long {  // which of unit w's 64 keys exist
            const int64_t left = blk_len != nullptr ? blk_len[w] : n_keys - w * kUnitKeys;
            return left >= kUnitKeys ? ~0ull : left <= 0 ? 0ull : (1ull << left) - 1ull;
        };
        Cursor ahead = start(), here = start();
        bool ua, ub;
        int in_flight = 0;  // units requested and not yet consumed
        for (int d = 0; d < D; ++d) {
            const int j = next(ahead, ua, ub);
            if (j == kEnd) break;
            issue_unit(j, d);
            ++in_flight;
        }
        load_q_dense();
        int stage = NS - 1, stage_ahead = D - 1;
        for (;;) {
            const int j = next(here, ua, ub);
            if (j == kEnd) break;
            const bool mine = (wave >> 1) ? ub : ua;
            stage = (stage + 1 == NS) ? 0 : stage + 1;
            stage_ahead = (stage_ahead + 1 == NS) ? 0 : stage_ahead + 1;
            // this unit's loads done (up to D - 1 later units may still be on their way), then everybody's
            if (in_flight == D) wait_vmcnt<CPW *(D - 1)>(); else wait_vmcnt<0>();
            lds_barrier();
            bool ta, tb;
            const int jn = next(ahead, ta, tb);
            if (jn != kEnd) issue_unit(jn, stage_ahead); else --in_flight;
            if (!mine) continue;
            const unsigned long long vmask = unit_mask_of(j);
            if (vmask == 0ull) continue;
            scores(&ring[stage][0]);
            softmax(vmask);
            accumulate(&ring[stage][kUnitElems]);
        }
    } else {
    for (int s = 0; s < D && s < n_steps; ++s) issue(s, s);  // D < NS: stage = s
    if constexpr (kAsmQ) load_q_dense();

    int stage = NS - 1, stage_ahead = D - 1;  // stages of unit s and of unit s + D, stepped at the loop head
    for (int s = 0; s < n_steps; ++s) {
        stage = (stage + 1 == NS) ? 0 : stage + 1;
        stage_ahead = (stage_ahead + 1 == NS) ? 0 : stage_ahead + 1;
        // unit s: this wave's loads done, then everybody's (barrier); the barrier also says every wave
        // has finished unit s - 1, whose stage the next request overwrites
        if (s + D <= n_steps) wait_vmcnt<CPW *(D - 1)>(); else wait_vmcnt<0>();
        lds_barrier();
        if (s + D < n_steps) issue(s + D, stage_ahead);
        if constexpr (PROBE) continue;
        const unsigned long long vmask = unit_mask(s);
        if (vmask == 0ull) continue;  // second half of a short last block
        scores(&ring[stage][0]);
        softmax(vmask);
        accumulate(&ring[stage][kUnitElems]);
    }
    }

    if (!row_valid) return;
    if constexpr (PROBE) {
        static_assert(!PROBE || (!DENSE && !PAIR && !SMALL && !EXTRA), "probe of the plain selection kernels only");
#pragma unroll
        for (int s = 0; s < 4; ++s) *reinterpret_cast<bf16x8 *>(out + (trow * heads + h) * 64 + 16 * s + 8 * g) = qb[s];
        return;
    }
    const float l_tot = sum_with_other_half(l_run);
    const float inv = (EXTRA && DENSE && l_tot == 0.f) ? 0.f : 1.f / l_tot;  // (a key split of empty units only)
    if (lse != nullptr && g == 0)
        lse[static_cast<int64_t>(h) * lse_stride + trow] = (m_run + __builtin_log2f(l_tot)) * kLn2;
    const int64_t o = (trow * heads + h) * 64;
    const float *oc = (o_comp != nullptr) ? o_comp + (static_cast<int64_t>(h) * n_blk + t / block) * 64 : nullptr;
    if constexpr (EXTRA)
        if (x.o_comp_tok != nullptr) oc = x.o_comp_tok + (t * heads + h) * 64;  // this query's own compressed output
    if (EXTRA && DENSE && x.out_f32 != nullptr) {  // fp32, by (key split and) query slot
        const int64_t slot = (static_cast<int64_t>(split) * n_tok + t) * heads + h;
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                floatx4 o4;
#pragma unroll
                for (int i = 0; i < 4; ++i) o4[i] = oacc[dt][4 * r4 + i] * inv;
                *reinterpret_cast<floatx4 *>(x.out_f32 + slot * 64 + 32 * dt + 8 * r4 + 4 * g) = o4;
            }
        // base-2 logarithm of the split's sum of exponentials: what weighs it against the other splits
        if (x.part_lse != nullptr && g == 0) x.part_lse[slot] = l_tot > 0.f ? m_run + __builtin_log2f(l_tot) : -INFINITY;
        return;
    }
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
                    float gl[4];
                    if constexpr (F32) {
                        const floatx4 g4 = *reinterpret_cast<const floatx4 *>(reinterpret_cast<const float *>(gate) + o + d0);
#pragma unroll
                        for (int i = 0; i < 4; ++i) gl[i] = g4[i];
                    } else {
                        const bf16x4 g4 = *reinterpret_cast<const bf16x4 *>(gate + o + d0);
#pragma unroll
                        for (int i = 0; i < 4; ++i) gl[i] = static_cast<float>(g4[i]);
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) gt[i] = 1.f / (1.f + __expf(-gl[i]));
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) res[i] = gt[i] * c4[i] + (1.f - gt[i]) * os[i];
            }
            if constexpr (F32) {
                *reinterpret_cast<floatx4 *>(reinterpret_cast<float *>(out) + o + d0) = floatx4{res[0], res[1], res[2], res[3]};
                if (o_sel != nullptr)
                    *reinterpret_cast<floatx4 *>(reinterpret_cast<float *>(o_sel) + o + d0) = floatx4{os[0], os[1], os[2], os[3]};
            } else {
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

template <int QW, bool DENSE, int NS, bool SMALL, bool EXTRA, bool ASMQ, bool PAIR, bool PROBE = false, bool F32 = false>
static hipError_t run_select_x(const SelectArgs &a, hipStream_t stream)
{
    // The load probe can hold the number of workgroups per CU down: unused dynamic LDS on top of the ring makes
    // each workgroup take 1 / probe_wg_per_cu of a CU's 160 KiB.
    unsigned pad_bytes = 0;
    if (PROBE && a.probe_wg_per_cu > 0) {
        const int ring = NS * 2 * kUnitElems * 2, share = (160 * 1024 / a.probe_wg_per_cu) & ~1023;
        if (share < ring) return hipErrorInvalidValue;
        pad_bytes = static_cast<unsigned>(share - ring);
        const hipError_t e = hipFuncSetAttribute(
            reinterpret_cast<const void *>(&select_mfma_kernel<QW, DENSE, NS, SMALL, EXTRA, ASMQ, PAIR, PROBE, F32>),
            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(pad_bytes));
        if (e != hipSuccess) return e;
    }
    const int64_t rows_per_group = 32 * QW;
    const int64_t groups = DENSE ? (a.n_tok + rows_per_group - 1) / rows_per_group : PAIR ? (a.n_blk + 1) / 2 : a.n_blk;
    const int64_t sets = groups;
    // Dense attention is quadratic: keep each launch to roughly 2e14 FLOP (a fraction of a second)
    // so that no single kernel occupies the GPU for seconds.
    int64_t per_launch = sets;
    if (DENSE) {
        const double flops_per_set = 4.0 * 64.0 * rows_per_group * static_cast<double>(a.n_keys + a.n_keys2) * a.heads;
        per_launch = static_cast<int64_t>(2e14 / flops_per_set);
        if (per_launch < 1) per_launch = 1;
        if (per_launch > sets) per_launch = sets;
    }
    if ((per_launch + 8) * a.heads * (a.x.n_split > 1 ? a.x.n_split : 1) > 0x7fffffffLL) return hipErrorInvalidValue;
    if (a.x.n_split > 1 && (!DENSE || SMALL || a.x.out_f32 == nullptr || a.x.part_lse == nullptr)) return hipErrorInvalidValue;
    const int map_mode = DENSE ? 0 : 2;
    for (int64_t s0 = 0; s0 < sets; s0 += per_launch) {
        const int64_t ns = (sets - s0 < per_launch) ? sets - s0 : per_launch;
        const int64_t n_split = (DENSE && a.x.n_split > 1) ? a.x.n_split : 1;
        const int64_t grid = (map_mode == 2) ? (ns + 7) / 8 * 8 * a.heads : ns * n_split * a.heads;
        hipLaunchKernelGGL((select_mfma_kernel<QW, DENSE, NS, SMALL, EXTRA, ASMQ, PAIR, PROBE, F32>), dim3(static_cast<unsigned>(grid)),
                           dim3(QW * 64), pad_bytes, stream, static_cast<const bf16_t *>(a.q),
                           static_cast<const bf16_t *>(a.kb), static_cast<const bf16_t *>(a.vb), a.idx,
                           a.o_comp, static_cast<const bf16_t *>(a.gate), static_cast<bf16_t *>(a.out),
                           static_cast<bf16_t *>(a.o_sel), a.lse, a.n_tok, a.n_blk, a.heads, a.block,
                           a.kk, a.scale * kLog2e, s0, ns, map_mode, a.qmap, a.n_keys, a.lse_stride,
                           static_cast<const bf16_t *>(a.kb2), static_cast<const bf16_t *>(a.vb2), a.n_keys2,
                           a.blk_len, a.x, a.lo_off, a.lo_off2);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

template <int QW, bool DENSE, int NS, bool SMALL = false, bool ASMQ = DENSE, bool PAIR = false, bool F32 = false>
static hipError_t run_select(const SelectArgs &a, hipStream_t stream)
{
    const SelectExtras &x = a.x;
    const bool extra = x.o_comp_tok != nullptr || x.out_f32 != nullptr || x.kv_head_stride != 0 ||
                       x.q_blk_len != nullptr || x.in.tok != 0;
    return extra ? run_select_x<QW, DENSE, NS, SMALL, true, ASMQ, PAIR, false, F32>(a, stream)
                 : run_select_x<QW, DENSE, NS, SMALL, false, ASMQ, PAIR, false, F32>(a, stream);
}

hipError_t launch_select_mfma(const SelectArgs &a, hipStream_t stream)
{
    if (a.kb == nullptr || a.vb == nullptr) return hipErrorInvalidValue;
    if (!a.is_bf16) {
        // fp32 problems: K/V tiles in bf16 operand parts
        if (a.lo_off <= 0 || a.loads_only) return hipErrorInvalidValue;
        const bool small = a.block == 16 || a.block == 32;
        if (!small && a.block != 64 && a.block != 128) return hipErrorInvalidValue;
        if (a.qmap.period != 0 && a.n_tok > 0x7fffffffLL) return hipErrorInvalidValue;
        if (a.idx == nullptr) {
            if (a.n_keys2 > 0 && (a.kb2 == nullptr || a.vb2 == nullptr || a.lo_off2 <= 0)) return hipErrorInvalidValue;
            return small ? run_select<4, true, 3, true, true, false, true>(a, stream)
                         : run_select<4, true, 3, false, true, false, true>(a, stream);
        }
        if (a.n_keys != a.n_tok || a.n_keys2 != 0) return hipErrorInvalidValue;
        return small          ? run_select<1, false, 2, true, false, false, true>(a, stream)
               : a.block == 64 ? run_select<2, false, 2, false, false, false, true>(a, stream)
                               : run_select<4, false, 2, false, false, false, true>(a, stream);
    }
    // One query block per workgroup, two LDS stages: measured best on MI355X.  A third stage is slower even
    // where it costs no occupancy (blocks of 128 tokens: 18.2 against 16.8 ms on 300 views, top-64): the fabric
    // is saturated already, and the units on their way (3 workgroups x 2 units x 16 KiB on each of an XCD's 32
    // CUs) then take up most of that XCD's 4 MiB of L2.
    if (a.qmap.period != 0 && a.n_tok > 0x7fffffffLL) return hipErrorInvalidValue;
    if (a.idx == nullptr) {
        if (a.n_keys2 > 0 && (a.kb2 == nullptr || a.vb2 == nullptr)) return hipErrorInvalidValue;
        if (a.block == 64 || a.block == 128) return run_select<4, true, 3>(a, stream);
        if (a.block == 16 || a.block == 32) return run_select<4, true, 3, true>(a, stream);
        return hipErrorInvalidValue;
    }
    if (a.n_keys != a.n_tok || a.n_keys2 != 0) return hipErrorInvalidValue;  // selection: keys = the query sequence
    // plain rows of at most 128 blocks of 64 tokens: the software-pipelined kernel of select_pipe.hip (rows that
    // are mostly forced blocks stay with the PAIR variant below)
    if (a.block == 64 && !a.loads_only && a.kk <= 128 && !(a.kk > 96 && 2 * a.n_common >= a.kk) &&
        a.x.o_comp_tok == nullptr && a.x.in.tok == 0)
        return launch_select_pipe(a, stream);
    if (a.loads_only) {  // the data movement of the plain kernels for blocks of 64 and 128 tokens, no arithmetic
        if (a.x.o_comp_tok != nullptr || a.x.in.tok != 0 || a.qmap.period != 0 || a.blk_len != nullptr) return hipErrorInvalidValue;
        const int ns = a.probe_stages == 0 ? 2 : a.probe_stages;
        if (a.block == 64) {
            if (ns == 2) return run_select_x<2, false, 2, false, false, false, false, true>(a, stream);
            if (ns == 3) return run_select_x<2, false, 3, false, false, false, false, true>(a, stream);
            if (ns == 4) return run_select_x<2, false, 4, false, false, false, false, true>(a, stream);
        }
        if (a.block == 128) {
            if (ns == 2) return run_select_x<4, false, 2, false, false, true, false, true>(a, stream);
            if (ns == 3) return run_select_x<4, false, 3, false, false, true, false, true>(a, stream);
            if (ns == 4) return run_select_x<4, false, 4, false, false, true, false, true>(a, stream);
        }
        return hipErrorInvalidValue;
    }
    // Long index rows (forced blocks, which every query block shares and the L2s keep) are bound by the loop
    // and by the traffic from the L2s into LDS rather than by the memory fabric: two neighbouring query blocks
    // per workgroup, each common unit fetched once for both (PAIR), with each unit's arithmetic overlapping
    // the next unit's loads (ASMQ): 135 against 149 ms with 224 forced + 64 selected blocks at 1000 views.  On
    // rows without common blocks, where neighbours share a third of their blocks, PAIR is 5 % slower; long
    // ones still gain from ASMQ alone.
    if (a.block == 64)
        return (a.kk > 96 && 2 * a.n_common >= a.kk) ? run_select<4, false, 2, false, true, true>(a, stream)
               : a.kk > 96                            ? run_select<2, false, 2, false, true>(a, stream)
                                                      : run_select<2, false, 2>(a, stream);
    // measured: the inline-asm Q load is 2 % faster for blocks of 128 and 32 tokens, 2 % slower for 16
    if (a.block == 128) return run_select<4, false, 2, false, true>(a, stream);
    if (a.block == 32) return run_select<1, false, 2, true, true>(a, stream);
    if (a.block == 16) return run_select<1, false, 2, true>(a, stream);
    return hipErrorInvalidValue;
}

// One thread per (query slot, head, 4 channels).
template <typename T>
__global__ __launch_bounds__(256) void dense_combine_kernel(const float *__restrict__ part_o,
                                                            const float *__restrict__ part_lse, int n_split,
                                                            int64_t n_tok, int heads, TokenMap qmap,
                                                            T *__restrict__ out)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= n_tok * heads * 16) return;
    const int c4 = static_cast<int>(i & 15);
    const int64_t th = i >> 4;  // t * heads + h
    const int64_t share = n_tok * heads;
    float top = -INFINITY;
    for (int j = 0; j < n_split; ++j) top = fmaxf(top, part_lse[j * share + th]);
    float den = 0.f;
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int j = 0; j < n_split; ++j) {
        const float l = part_lse[j * share + th];
        if (l == -INFINITY) continue;  // a share without keys
        const float w = exp2f(l - top);
        const floatx4 o = *reinterpret_cast<const floatx4 *>(part_o + (j * share + th) * 64 + c4 * 4);
        den += w;
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] += w * o[c];
    }
    const int64_t t = th / heads;
    const int h = static_cast<int>(th - t * heads);
    T *dst = out + (qmap.row(t) * heads + h) * 64 + c4 * 4;
    if constexpr (sizeof(T) == 4) {
        floatx4 r;
#pragma unroll
        for (int c = 0; c < 4; ++c) r[c] = acc[c] / den;
        *reinterpret_cast<floatx4 *>(dst) = r;
    } else {
        bf16x4 r;
#pragma unroll
        for (int c = 0; c < 4; ++c) r[c] = static_cast<bf16_t>(acc[c] / den);
        *reinterpret_cast<bf16x4 *>(dst) = r;
    }
}

hipError_t launch_dense_combine(const float *part_o, const float *part_lse, int n_split, int64_t n_tok, int heads,
                                TokenMap qmap, void *out, bool is_bf16, hipStream_t stream)
{
    const int64_t threads = n_tok * heads * 16;
    if (n_split < 1 || threads <= 0 || (threads + 255) / 256 > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid(static_cast<unsigned>((threads + 255) / 256));
    if (is_bf16)
        hipLaunchKernelGGL(dense_combine_kernel<bf16_t>, grid, dim3(256), 0, stream, part_o, part_lse, n_split, n_tok,
                           heads, qmap, static_cast<bf16_t *>(out));
    else
        hipLaunchKernelGGL(dense_combine_kernel<float>, grid, dim3(256), 0, stream, part_o, part_lse, n_split, n_tok,
                           heads, qmap, static_cast<float *>(out));
    return hipGetLastError();
}

}  // namespace s3r
