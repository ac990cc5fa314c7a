// C ABI of the library (see include/speed3r.h): argument checks, workspace carving, launch
// sequencing, optional per-stage event timing.  No kernel code here.
#include "../../include/speed3r.h"
#include "s3r_kernels.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <mutex>
#include <vector>

// Scratch of speed3r_sparse_global_attn_noalloc: device memory that exists from the moment the code object
// is loaded, one copy per GPU, so that entry point never allocates.  In host code this name only stands for
// the symbol; the device address comes from hipGetSymbolAddress (static_scratch below).
constexpr size_t kStaticScratchBytes = S3R_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local char g_err[512] = "no error";
thread_local bool t_no_events = false;  // set while an entry point that must not create HIP events runs

s3r_status fail(s3r_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

s3r_status hip_fail(hipError_t e, const char *what)
{
    return fail(S3R_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

#define S3R_HIP(call, what)                                  \
    do {                                                     \
        hipError_t e_ = (call);                              \
        if (e_ != hipSuccess) return hip_fail(e_, what);     \
    } while (0)

constexpr size_t kAlign = 256;
constexpr size_t kScoreBytesCap = size_t(8) << 30;  // S_guide is processed in head chunks of at most this size

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int g_kernel_choice = 0;  // 0 auto, 1 generic attention kernels only, 2 TopK from scores written to memory

// every supported block size, bf16 and fp32 (the latter with K/V in bf16 operand parts)
bool mfma_ok(s3r_dtype dtype, int block) { (void)dtype; (void)block; return g_kernel_choice != 1; }
// copies of a K (or V) tile array the MFMA kernels read: fp32 problems keep bf16 parts hi, lo and (K) lo2
size_t tile_parts(s3r_dtype dtype) { return dtype == S3R_BF16 ? 1 : 3; }

// Dense attention of few query rows (the special tokens) in key splits: as many as make the workgroups fill
// the CUs most evenly (MI355X: 256 CUs x 3 workgroups of the dense kernel each), at least 4 key units each.
constexpr int kDenseSlots = 256 * 3;
constexpr int kMaxDenseSplit = 8;
int dense_splits(int64_t n_rows, int heads, int64_t n_units)
{
    const int64_t wgs = (n_rows + 127) / 128 * heads;
    if (wgs >= 4 * kDenseSlots) return 1;
    int best = 1;
    double best_fill = 0.0;
    for (int s = 1; s <= kMaxDenseSplit && (s == 1 || s * 4 <= n_units); ++s) {
        const double rounds = static_cast<double>(wgs) * s / kDenseSlots;
        const double fill = rounds / static_cast<double>(static_cast<int64_t>(rounds + 0.999999));
        if (fill > best_fill + 1e-9) { best_fill = fill; best = s; }
    }
    return best;
}

constexpr int kCandCap = 256;  // candidate slots per list of the TopK-in-the-sweep path (two lists per row)

s3r_status check_shape(int64_t n_tok, int heads, int head_dim, int block, int topk, int dtype)
{
    if (n_tok <= 0 || heads <= 0 || topk <= 0)
        return fail(S3R_ERR_INVALID_ARG, "n_tok (%lld), heads (%d) and topk (%d) must be positive",
                    static_cast<long long>(n_tok), heads, topk);
    if (dtype != S3R_F32 && dtype != S3R_BF16) return fail(S3R_ERR_UNSUPPORTED, "unknown dtype %d", dtype);
    if (head_dim != 64) return fail(S3R_ERR_UNSUPPORTED, "head_dim %d unsupported (must be 64)", head_dim);
    if (block != 16 && block != 32 && block != 64 && block != 128)
        return fail(S3R_ERR_UNSUPPORTED, "block %d unsupported (must be 16, 32, 64 or 128)", block);
    if (heads > 65535) return fail(S3R_ERR_UNSUPPORTED, "heads %d unsupported (max 65535)", heads);
    const int64_t n_blk = (n_tok + block - 1) / block;
    if (n_blk * heads > 0x7fffffffLL) return fail(S3R_ERR_UNSUPPORTED, "n_blk * heads exceeds 2^31 - 1");
    return S3R_OK;
}

// ---- workspace layout of the full path -------------------------------------------------------
struct Layout {
    int64_t n_blk, tiles, ld_s;
    int kk;      // blocks TopK picks per row (among the non-forced ones)
    int width;   // blocks attended per row: kk + n_forced
    int head_chunk;
    size_t qc, kc, vc, oc, tile[8], idx, idx_merged, forced_clean, forced_words, s, kb, vb, kb_spec, vb_spec;
    size_t stat_slots, head_stats, thr, cand, cand_count, overflow, blk_len, oc_tok, spec_part_o, spec_part_lse, total;
    int spec_split;  // key splits of the special rows' dense attention (1: none)
};

// n_tok: tokens on the sparse path (the image tokens); n_spec: special tokens (dense rows).
Layout make_layout(int64_t n_tok, int heads, int block, int topk, int n_forced, s3r_dtype dtype,
                   int64_t n_spec = 0, bool token_queries = false)
{
    Layout L{};
    L.n_blk = (n_tok + block - 1) / block;
    const int64_t free_blk = L.n_blk - n_forced;
    L.kk = static_cast<int>(topk < free_blk ? topk : free_blk);
    L.width = L.kk + n_forced;
    L.tiles = s3r::pooled_tiles_padded(L.n_blk);
    L.ld_s = (L.n_blk + 63) / 64 * 64;
    const size_t per_head_s = static_cast<size_t>(L.n_blk) * L.ld_s * sizeof(float);
    int64_t hc = static_cast<int64_t>(kScoreBytesCap / per_head_s);
    if (hc < 1) hc = 1;
    if (hc > heads) hc = heads;
    L.head_chunk = static_cast<int>(hc);
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += align_up(bytes); return o; };
    const size_t pooled = static_cast<size_t>(heads) * L.n_blk * 64 * sizeof(float);
    L.qc = take(pooled);
    L.kc = take(pooled);
    L.vc = take(pooled);
    L.oc = take(pooled);
    for (int a = 0; a < 8; ++a) L.tile[a] = take(static_cast<size_t>(heads) * L.tiles * 32 * 64 * 2);
    L.idx = take(static_cast<size_t>(heads) * L.n_blk * L.kk * sizeof(int32_t));
    L.idx_merged = take(n_forced > 0 ? static_cast<size_t>(heads) * L.n_blk * L.width * sizeof(int32_t) : 0);
    L.forced_clean = take(static_cast<size_t>(n_forced) * sizeof(int32_t));
    L.forced_words = take(n_forced > 0 ? static_cast<size_t>((L.n_blk + 63) / 64) * sizeof(unsigned long long) : 0);
    L.s = take(per_head_s * L.head_chunk);
    const size_t blocked = mfma_ok(dtype, block) ? static_cast<size_t>(heads) * L.n_blk * block * 64 * 2 * tile_parts(dtype) : 0;
    L.kb = take(blocked);
    L.vb = take(blocked);
    const size_t spec_tiles = mfma_ok(dtype, block) ? static_cast<size_t>(heads) * ((n_spec + 63) / 64) * 64 * 64 * 2 * tile_parts(dtype) : 0;
    L.kb_spec = take(spec_tiles);
    L.vb_spec = take(spec_tiles);
    // TopK-in-the-sweep buffers, for all heads at once (the sweeps are not chunked)
    const size_t chunk_rows = static_cast<size_t>(heads) * L.n_blk;
    L.stat_slots = take(static_cast<size_t>(heads) * 3 * s3r::kStatSlots * sizeof(unsigned));
    L.head_stats = take(static_cast<size_t>(heads) * sizeof(s3r::HeadStats));
    L.thr = take(chunk_rows * sizeof(float));
    L.cand = take(chunk_rows * 2 * kCandCap * sizeof(int32_t));
    L.cand_count = take(chunk_rows * 2 * sizeof(int));
    L.overflow = take(sizeof(int));
    L.blk_len = take(static_cast<size_t>(L.n_blk) * sizeof(int32_t));
    // compression branch with unpooled queries: fp32 compressed output per query slot
    L.oc_tok = take(token_queries ? static_cast<size_t>(L.n_blk) * block * heads * 64 * sizeof(float) : 0);
    // special rows in key splits: normalised partial results and their log-sums
    L.spec_split = 1;
    if (n_spec > 0 && mfma_ok(dtype, block) && block >= 64)
        L.spec_split = dense_splits(n_spec, heads, L.n_blk * (block / 64) + (n_spec + 63) / 64);
    const size_t part_rows = L.spec_split > 1 ? static_cast<size_t>(L.spec_split) * n_spec * heads : 0;
    L.spec_part_o = take(part_rows * 64 * sizeof(float));
    L.spec_part_lse = take(part_rows * sizeof(float));
    L.total = off;
    return L;
}

// ---- library-held scratch --------------------------------------------------------------------
std::mutex g_mu;
constexpr int kMaxDevices = 64;
void *g_scratch[kMaxDevices] = {};
size_t g_scratch_bytes[kMaxDevices] = {};

s3r_status scratch_get(size_t bytes, void **out)
{
    int dev = 0;
    S3R_HIP(hipGetDevice(&dev), "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(S3R_ERR_UNSUPPORTED, "device ordinal %d unsupported", dev);
    std::lock_guard<std::mutex> lock(g_mu);
    if (bytes > g_scratch_bytes[dev]) {
        S3R_HIP(hipDeviceSynchronize(), "hipDeviceSynchronize before growing scratch");
        if (g_scratch[dev]) {
            S3R_HIP(hipFree(g_scratch[dev]), "hipFree(scratch)");
            g_scratch[dev] = nullptr;
            g_scratch_bytes[dev] = 0;
        }
        void *p = nullptr;
        hipError_t e = hipMalloc(&p, bytes);
        if (e != hipSuccess) return fail(S3R_ERR_WORKSPACE, "hipMalloc of %zu scratch bytes failed: %s", bytes, hipGetErrorString(e));
        g_scratch[dev] = p;
        g_scratch_bytes[dev] = bytes;
    }
    *out = g_scratch[dev];
    return S3R_OK;
}

// Device address of this GPU's copy of `scratch`, looked up once per device with that device current.
void *g_static_ptr[kMaxDevices] = {};

s3r_status static_scratch(void **out)
{
    int dev = 0;
    S3R_HIP(hipGetDevice(&dev), "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(S3R_ERR_UNSUPPORTED, "device ordinal %d unsupported", dev);
    std::lock_guard<std::mutex> lock(g_mu);
    if (g_static_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        S3R_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
        if (ptr == nullptr || (reinterpret_cast<uintptr_t>(ptr) & (kAlign - 1)) != 0)
            return fail(S3R_ERR_HIP, "static scratch has no usable device address (%p)", ptr);
        g_static_ptr[dev] = ptr;
    }
    *out = g_static_ptr[dev];
    return S3R_OK;
}

// ---- per-stage event timing ------------------------------------------------------------------
bool g_profiling = false;
struct Span { int stage; hipEvent_t start, stop; };
std::vector<Span> g_spans;        // spans recorded since the last speed3r_get_stage_ms
std::vector<hipEvent_t> g_pool;   // recycled events

hipEvent_t event_take()
{
    if (!g_pool.empty()) { hipEvent_t e = g_pool.back(); g_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

struct StageTimer {
    hipStream_t stream;
    Span span{};
    bool on = false;
    StageTimer(int stage, hipStream_t st) : stream(st)
    {
        if (!g_profiling || t_no_events) return;
        std::lock_guard<std::mutex> lock(g_mu);
        span.stage = stage;
        span.start = event_take();
        span.stop = event_take();
        on = span.start && span.stop;
        if (on) on = hipEventRecord(span.start, stream) == hipSuccess;
    }
    ~StageTimer()
    {
        if (!on) return;
        if (hipEventRecord(span.stop, stream) != hipSuccess) return;
        std::lock_guard<std::mutex> lock(g_mu);
        g_spans.push_back(span);
    }
};

char *at(void *base, size_t off) { return static_cast<char *>(base) + off; }

// Buffers of the TopK-in-the-sweep path (all null: TopK from scores written to s_buf).
struct FusedBufs {
    void *stat_slots = nullptr;             // scratch of launch_pooled_stats
    s3r::HeadStats *head_stats = nullptr;   // [heads]
    float *thr = nullptr;
    int32_t *cand = nullptr;
    int *cand_count = nullptr;
    int *overflow = nullptr;
};

// pooled fp32 -> operand tiles -> S_guide / Oc' -> TopK, in head chunks bounded by the S buffer
s3r_status run_compress_topk(const float *qc, const float *kc, const float *vc, void *const tile[8],
                             float *s_buf, int64_t ld_s, int head_chunk, float *o_comp, int32_t *idx,
                             int64_t n_blk, int64_t tiles, int heads, int kk, float scale,
                             bool accurate_pv, bool want_topk, const unsigned long long *forced_words,
                             const FusedBufs &fb, hipStream_t stream)
{
    // Without S_guide in memory when k allows it.  Should a candidate list run over (long runs of
    // equal scores), the overflow word makes the two plain launches that follow redo the chunk;
    // otherwise they return at once.
    const bool fused = want_topk && fb.thr != nullptr && kk >= 1 && kk <= s3r::kFusedTopkMaxK && g_kernel_choice != 2;
    {
        StageTimer tm(S3R_STAGE_SPLIT, stream);
        if (fused)
            S3R_HIP(s3r::launch_pooled_stats(qc, kc, n_blk, heads, fb.stat_slots, fb.head_stats, stream),
                    "pooled statistics kernel launch");
        S3R_HIP(s3r::launch_split(qc, kc, vc, tile[0], tile[1], tile[2], tile[3], tile[4],
                                  accurate_pv ? tile[5] : nullptr, fused ? tile[6] : nullptr, fused ? tile[7] : nullptr,
                                  fused ? fb.head_stats : nullptr, n_blk, heads, stream),
                "split kernel launch");
    }
    const size_t tile_head = static_cast<size_t>(tiles) * 32 * 64 * 2;  // bytes per head per array
    if (fused) {
        // all heads in one launch each: nothing here is as large as S
        {
            StageTimer tm(S3R_STAGE_COMPRESS, stream);
            S3R_HIP(s3r::launch_compress_threshold(tile[0], tile[1], tile[2], tile[3], tile[4],
                                                   accurate_pv ? tile[5] : nullptr, tile[6], tile[7], o_comp, n_blk, heads, scale,
                                                   forced_words, kk, fb.head_stats, fb.thr, fb.overflow, stream),
                    "compress (threshold) kernel launch");
        }
        StageTimer tm(S3R_STAGE_TOPK, stream);
        S3R_HIP(s3r::launch_compress_filter(tile[6], tile[7], n_blk, heads, forced_words, fb.thr,
                                            fb.cand, fb.cand_count, kCandCap, fb.overflow, stream),
                "compress (filter) kernel launch");
        S3R_HIP(s3r::launch_topk_candidates(qc, kc, fb.cand, fb.cand_count, kCandCap, idx, n_blk, heads, kk, stream),
                "candidate topk kernel launch");
    }
    const int *run_flag = fused ? fb.overflow : nullptr;
    for (int h0 = 0; h0 < heads; h0 += head_chunk) {
        const int hc = (heads - h0 < head_chunk) ? heads - h0 : head_chunk;
        {
            StageTimer tm(S3R_STAGE_COMPRESS, stream);
            S3R_HIP(s3r::launch_compress(at(tile[0], h0 * tile_head), at(tile[1], h0 * tile_head),
                                         at(tile[2], h0 * tile_head), at(tile[3], h0 * tile_head),
                                         at(tile[4], h0 * tile_head),
                                         accurate_pv ? at(tile[5], h0 * tile_head) : nullptr, s_buf, ld_s,
                                         o_comp + static_cast<size_t>(h0) * n_blk * 64, n_blk, hc, scale,
                                         forced_words, run_flag, stream),
                    "compress kernel launch");
        }
        if (want_topk && kk > 0) {
            StageTimer tm(S3R_STAGE_TOPK, stream);
            S3R_HIP(s3r::launch_topk(s_buf, ld_s, idx + static_cast<size_t>(h0) * n_blk * kk, n_blk,
                                     static_cast<int64_t>(hc) * n_blk, kk, run_flag, stream),
                    "topk kernel launch");
        }
    }
    return S3R_OK;
}

// Special / image token split of a sequence of `n_tok` rows in views of `period` rows whose first
// `special` rows are special tokens (0, 0: no special tokens).
struct Split {
    int64_t n_img;   // slots of the sequence the sparse path works on (with windows: n_blk * block, edge
                     // windows leaving slots empty)
    int64_t n_spec;
    bool windows;
    s3r::TokenMap img, spec;
};

s3r_status make_split(int64_t n_tok, int period, int special, int grid_h, int grid_w, int window, int block,
                      Split *out)
{
    Split sp{};
    sp.n_img = n_tok;
    sp.n_spec = 0;
    sp.windows = false;
    if (window != 0 || grid_h != 0 || grid_w != 0) {
        if (window <= 0 || grid_h <= 0 || grid_w <= 0)
            return fail(S3R_ERR_INVALID_ARG, "window (%d), grid_h (%d) and grid_w (%d) must all be positive or all 0",
                        window, grid_h, grid_w);
        if (window * window != block)
            return fail(S3R_ERR_INVALID_ARG, "block (%d) must equal window * window (%d)", block, window * window);
        if (period <= 0 || special < 0 || period - special != grid_h * grid_w)
            return fail(S3R_ERR_INVALID_ARG, "tokens_per_view (%d) must equal special_per_view (%d) + grid_h * grid_w (%d)",
                        period, special, grid_h * grid_w);
    }
    if (period == 0 && special == 0) { *out = sp; return S3R_OK; }
    if (period <= 0 || special < 0 || special >= period)
        return fail(S3R_ERR_INVALID_ARG, "special_per_view (%d) must lie in [0, tokens_per_view = %d)", special, period);
    if (n_tok % period != 0)
        return fail(S3R_ERR_INVALID_ARG, "n_tok (%lld) is not a multiple of tokens_per_view (%d)",
                    static_cast<long long>(n_tok), period);
    if (n_tok > 0x7fffffffLL) return fail(S3R_ERR_UNSUPPORTED, "n_tok exceeds 2^31 - 1 with special tokens");
    if (special == 0 && window == 0) { *out = sp; return S3R_OK; }
    const int64_t views = n_tok / period;
    sp.n_spec = views * special;
    sp.n_img = n_tok - sp.n_spec;
    sp.img.period = period; sp.img.first = special; sp.img.count = period - special;
    sp.spec.period = period; sp.spec.first = 0; sp.spec.count = special;
    if (window != 0) {
        sp.windows = true;
        sp.img.win = window; sp.img.grid_h = grid_h; sp.img.grid_w = grid_w;
        sp.img.nwx = (grid_w + window - 1) / window;
        sp.img.nw = sp.img.nwx * ((grid_h + window - 1) / window);
        sp.n_img = views * sp.img.nw * block;
        if (sp.n_img > 0x7fffffffLL) return fail(S3R_ERR_UNSUPPORTED, "windowed sequence exceeds 2^31 - 1 slots");
    }
    *out = sp;
    return S3R_OK;
}

float resolve_scale(float s, int head_dim) { return s > 0.f ? s : 1.f / std::sqrt(static_cast<float>(head_dim)); }

}  // namespace

extern "C" {

const char *speed3r_last_error(void) { return g_err; }

s3r_status speed3r_set_profiling(int enable)
{
    std::lock_guard<std::mutex> lock(g_mu);
    g_profiling = enable != 0;
    return S3R_OK;
}

s3r_status speed3r_set_kernel_choice(int choice)
{
    if (choice < 0 || choice > 2) return fail(S3R_ERR_INVALID_ARG, "kernel choice %d unknown", choice);
    g_kernel_choice = choice;
    return S3R_OK;
}

s3r_status speed3r_get_stage_ms(float *ms, int *launches)
{
    if (!ms || !launches) return fail(S3R_ERR_INVALID_ARG, "ms and launches must be non-null host arrays");
    std::lock_guard<std::mutex> lock(g_mu);
    for (int i = 0; i < S3R_N_STAGES; ++i) { ms[i] = 0.f; launches[i] = 0; }
    for (auto &s : g_spans) {
        S3R_HIP(hipEventSynchronize(s.stop), "hipEventSynchronize");
        float t = 0.f;
        S3R_HIP(hipEventElapsedTime(&t, s.start, s.stop), "hipEventElapsedTime");
        ms[s.stage] += t;
        launches[s.stage] += 1;
    }
    for (auto &s : g_spans) { g_pool.push_back(s.start); g_pool.push_back(s.stop); }
    g_spans.clear();
    return S3R_OK;
}

s3r_status speed3r_release_scratch(void)
{
    int dev = 0;
    S3R_HIP(hipGetDevice(&dev), "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return S3R_OK;
    std::lock_guard<std::mutex> lock(g_mu);
    if (g_scratch[dev]) {
        S3R_HIP(hipDeviceSynchronize(), "hipDeviceSynchronize");
        S3R_HIP(hipFree(g_scratch[dev]), "hipFree(scratch)");
        g_scratch[dev] = nullptr;
        g_scratch_bytes[dev] = 0;
    }
    return S3R_OK;
}

size_t speed3r_workspace_bytes(int64_t n_tok, int heads, int head_dim, int block, int topk, int n_forced,
                               s3r_dtype dtype)
{
    if (check_shape(n_tok, heads, head_dim, block, topk, dtype) != S3R_OK) return 0;
    if (n_forced < 0 || n_forced > (n_tok + block - 1) / block) {
        fail(S3R_ERR_INVALID_ARG, "n_forced (%d) must lie in [0, n_blk]", n_forced);
        return 0;
    }
    return make_layout(n_tok, heads, block, topk, n_forced, dtype).total;
}

size_t speed3r_workspace_bytes_ex(const s3r_params *p)
{
    if (!p) { fail(S3R_ERR_INVALID_ARG, "params is null"); return 0; }
    if (check_shape(p->n_tok, p->heads, p->head_dim, p->block, p->topk, p->dtype) != S3R_OK) return 0;
    Split sp{};
    if (make_split(p->n_tok, p->tokens_per_view, p->special_per_view, p->grid_h, p->grid_w, p->window, p->block,
                   &sp) != S3R_OK)
        return 0;
    if (p->n_forced < 0 || p->n_forced > (sp.n_img + p->block - 1) / p->block) {
        fail(S3R_ERR_INVALID_ARG, "n_forced (%d) must lie in [0, n_blk]", p->n_forced);
        return 0;
    }
    if (p->compress_queries != 0 && p->compress_queries != 1) {
        fail(S3R_ERR_INVALID_ARG, "compress_queries (%d) must be 0 or 1", p->compress_queries);
        return 0;
    }
    return make_layout(sp.n_img, p->heads, p->block, p->topk, p->n_forced, p->dtype, sp.n_spec, p->compress_queries == 1).total;
}

int64_t speed3r_num_blocks(const s3r_params *p)
{
    if (!p) { fail(S3R_ERR_INVALID_ARG, "params is null"); return -1; }
    if (check_shape(p->n_tok, p->heads, p->head_dim, p->block, p->topk, p->dtype) != S3R_OK) return -1;
    Split sp{};
    if (make_split(p->n_tok, p->tokens_per_view, p->special_per_view, p->grid_h, p->grid_w, p->window, p->block,
                   &sp) != S3R_OK)
        return -1;
    return (sp.n_img + p->block - 1) / p->block;
}

int speed3r_selected_per_row(int64_t n_tok, int block, int topk, int n_forced)
{
    if (n_tok <= 0 || block <= 0 || topk <= 0 || n_forced < 0) return -1;
    const int64_t n_blk = (n_tok + block - 1) / block;
    if (n_forced > n_blk) return -1;
    const int64_t free_blk = n_blk - n_forced;
    return static_cast<int>(n_forced + (topk < free_blk ? topk : free_blk));
}

s3r_status speed3r_sparse_global_attn_ex(const s3r_params *p)
{
    if (!p) return fail(S3R_ERR_INVALID_ARG, "params is null");
    s3r_status st = check_shape(p->n_tok, p->heads, p->head_dim, p->block, p->topk, p->dtype);
    if (st != S3R_OK) return st;
    if (!p->q || !p->k || !p->v || !p->out) return fail(S3R_ERR_INVALID_ARG, "q, k, v and out must be non-null");
    if (!aligned16(p->q) || !aligned16(p->k) || !aligned16(p->v) || !aligned16(p->out) ||
        !aligned16(p->gate_logits) || !aligned16(p->o_sel) || !aligned16(p->o_comp) ||
        !aligned16(p->topk_idx) || !aligned16(p->lse_sel) || (reinterpret_cast<uintptr_t>(p->status) & 3u) != 0)
        return fail(S3R_ERR_INVALID_ARG, "device pointers must be 16-byte aligned");
    if (p->out == p->q || p->out == p->k || p->out == p->v) return fail(S3R_ERR_INVALID_ARG, "out must not alias an input");
    // 16-byte vector loads: rows and heads of q, k, v must start on 16-byte boundaries
    if (p->stride_tok < 0 || p->stride_head < 0 || p->stride_tok % 8 != 0 || p->stride_head % 8 != 0)
        return fail(S3R_ERR_INVALID_ARG, "stride_tok (%lld) and stride_head (%lld) must be non-negative multiples of 8 elements",
                    static_cast<long long>(p->stride_tok), static_cast<long long>(p->stride_head));
    s3r::InStride in{};  // {0, 0} = packed
    if (p->stride_tok != 0 || p->stride_head != 0) {
        in.tok = p->stride_tok != 0 ? p->stride_tok : static_cast<int64_t>(p->heads) * 64;
        in.head = p->stride_head != 0 ? p->stride_head : 64;
    }
    const int n_forced = p->forced_blocks ? p->n_forced : 0;
    if (p->n_forced < 0 || (p->n_forced > 0 && !p->forced_blocks) || (p->forced_blocks && p->n_forced == 0))
        return fail(S3R_ERR_INVALID_ARG, "forced_blocks and n_forced (%d) must be given together", p->n_forced);
    Split sp{};
    st = make_split(p->n_tok, p->tokens_per_view, p->special_per_view, p->grid_h, p->grid_w, p->window, p->block, &sp);
    if (st != S3R_OK) return st;
    if (n_forced > (sp.n_img + p->block - 1) / p->block)
        return fail(S3R_ERR_INVALID_ARG, "n_forced (%d) exceeds the number of blocks", n_forced);
    if (p->compress_queries != 0 && p->compress_queries != 1)
        return fail(S3R_ERR_INVALID_ARG, "compress_queries (%d) must be 0 or 1", p->compress_queries);
    const bool token_queries = p->compress_queries == 1;
    if (token_queries && p->dtype == S3R_BF16 && !mfma_ok(p->dtype, p->block))
        return fail(S3R_ERR_UNSUPPORTED, "compress_queries = 1 on bf16 data needs the MFMA kernels (kernel choice 1 is set)");
    const Layout L = make_layout(sp.n_img, p->heads, p->block, p->topk, n_forced, p->dtype, sp.n_spec, token_queries);
    if (!p->workspace) return fail(S3R_ERR_WORKSPACE, "workspace is null (%zu bytes needed)", L.total);
    if ((reinterpret_cast<uintptr_t>(p->workspace) & (kAlign - 1)) != 0)
        return fail(S3R_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    if (p->workspace_bytes < L.total)
        return fail(S3R_ERR_WORKSPACE, "workspace too small: %zu bytes given, %zu needed", p->workspace_bytes, L.total);

    hipStream_t stream = static_cast<hipStream_t>(p->stream);
    const bool is_bf16 = p->dtype == S3R_BF16;
    const bool mfma = mfma_ok(p->dtype, p->block);
    const float scale = resolve_scale(p->softmax_scale, p->head_dim);
    void *ws = p->workspace;
    float *qc = reinterpret_cast<float *>(at(ws, L.qc));
    float *kc = reinterpret_cast<float *>(at(ws, L.kc));
    float *vc = reinterpret_cast<float *>(at(ws, L.vc));
    float *oc = p->o_comp ? p->o_comp : reinterpret_cast<float *>(at(ws, L.oc));
    // idx_sel: what the selection kernel reads ([heads][n_blk][width]); idx_dyn: what TopK writes.
    int32_t *idx_sel = p->topk_idx ? p->topk_idx
                                   : reinterpret_cast<int32_t *>(at(ws, n_forced > 0 ? L.idx_merged : L.idx));
    int32_t *idx_dyn = n_forced > 0 ? reinterpret_cast<int32_t *>(at(ws, L.idx)) : idx_sel;
    int32_t *forced_clean = reinterpret_cast<int32_t *>(at(ws, L.forced_clean));
    unsigned long long *forced_words =
        n_forced > 0 ? reinterpret_cast<unsigned long long *>(at(ws, L.forced_words)) : nullptr;
    void *tile[8];
    for (int a = 0; a < 8; ++a) tile[a] = at(ws, L.tile[a]);
    void *kb = mfma ? at(ws, L.kb) : nullptr;
    void *vb = mfma ? at(ws, L.vb) : nullptr;

    int32_t *blk_len = nullptr;
    {
        StageTimer tm(S3R_STAGE_POOL, stream);
        if (sp.windows) {
            blk_len = reinterpret_cast<int32_t *>(at(ws, L.blk_len));
            S3R_HIP(s3r::launch_block_lens(sp.img, p->block, sp.n_img, L.n_blk, blk_len, stream), "block length kernel launch");
        }
        S3R_HIP(s3r::launch_pool(p->q, p->k, p->v, qc, kc, vc, kb, vb, sp.n_img, p->heads, p->block, is_bf16,
                                 sp.img, in, stream),
                "pool kernel launch");
    }
    FusedBufs fb;
    fb.stat_slots = at(ws, L.stat_slots);
    fb.head_stats = reinterpret_cast<s3r::HeadStats *>(at(ws, L.head_stats));
    fb.thr = reinterpret_cast<float *>(at(ws, L.thr));
    fb.cand = reinterpret_cast<int32_t *>(at(ws, L.cand));
    fb.cand_count = reinterpret_cast<int *>(at(ws, L.cand_count));
    fb.overflow = reinterpret_cast<int *>(at(ws, L.overflow));
    if (n_forced > 0 || p->status != nullptr) {
        StageTimer tm(S3R_STAGE_TOPK, stream);
        S3R_HIP(s3r::launch_forced_prepare(p->forced_blocks, n_forced, L.n_blk, forced_clean, forced_words, p->status, stream),
                "forced-block prepare kernel launch");
    }
    st = run_compress_topk(qc, kc, vc, tile, reinterpret_cast<float *>(at(ws, L.s)), L.ld_s, L.head_chunk, oc,
                           idx_dyn, L.n_blk, L.tiles, p->heads, L.kk, scale, !is_bf16, true, forced_words, fb, stream);
    if (st != S3R_OK) return st;
    if (n_forced > 0) {
        StageTimer tm(S3R_STAGE_TOPK, stream);
        S3R_HIP(s3r::launch_merge_forced(idx_dyn, L.kk, forced_clean, n_forced, idx_sel,
                                         static_cast<int64_t>(p->heads) * L.n_blk, stream),
                "forced-block merge kernel launch");
    }

    float *oc_tok = nullptr;
    if (token_queries) {
        // Compression branch with unpooled queries: every image row's own query against the pooled keys,
        // i.e. dense attention over the pooled tensors (n_blk keys per head), result in fp32 per query
        // slot.  bf16 problems: the bf16 hi tiles of Kc, Vc written by the split kernel are already in
        // the unit layout of the MFMA kernel; fp32 problems: the generic kernel on Kc, Vc themselves.
        oc_tok = reinterpret_cast<float *>(at(ws, L.oc_tok));
        s3r::SelectArgs c{};
        c.q = p->q; c.qmap = sp.img; c.n_tok = sp.n_img; c.lse_stride = p->n_tok;
        c.n_keys = L.n_blk; c.n_blk = (L.n_blk + 63) / 64; c.block = 64; c.heads = p->heads;
        c.scale = scale; c.is_bf16 = is_bf16;
        c.x.out_f32 = oc_tok; c.x.q_blk_len = blk_len; c.x.q_block = p->block; c.x.in = in;
        StageTimer tm(S3R_STAGE_COMPRESS, stream);
        if (mfma && is_bf16) {
            c.kb = tile[2]; c.vb = tile[4];
            c.x.kv_head_stride = L.tiles * 32 * 64;
            S3R_HIP(s3r::launch_select_mfma(c, stream), "compression branch (unpooled queries) kernel launch");
        } else {
            c.k = kc; c.v = vc;
            c.x.k_row_stride = 64; c.x.k_head_stride = L.n_blk * 64;
            S3R_HIP(s3r::launch_select_generic(c, stream), "compression branch (unpooled queries) kernel launch");
        }
    }

    s3r::SelectArgs a{};
    a.x.o_comp_tok = oc_tok; a.x.in = in;
    a.n_common = n_forced;
    a.q = p->q; a.k = p->k; a.v = p->v; a.kb = kb; a.vb = vb; a.idx = idx_sel; a.o_comp = oc;
    a.gate = p->gate_logits; a.out = p->out; a.o_sel = p->o_sel; a.lse = p->lse_sel;
    a.n_tok = sp.n_img; a.n_keys = sp.n_img; a.n_blk = L.n_blk; a.lse_stride = p->n_tok;
    a.qmap = sp.img; a.kmap = sp.img; a.blk_len = blk_len;
    a.heads = p->heads; a.block = p->block; a.kk = L.width;
    a.scale = scale; a.is_bf16 = is_bf16;
    a.lo_off = (mfma && !is_bf16) ? static_cast<int64_t>(p->heads) * L.n_blk * p->block * 64 : 0;
    {
        StageTimer tm(S3R_STAGE_SELECT, stream);
        S3R_HIP(mfma ? s3r::launch_select_mfma(a, stream) : s3r::launch_select_generic(a, stream),
                "select kernel launch");
    }
    if (sp.n_spec > 0) {
        // Special tokens (Sec. 3.2 eq. 2): plain attention of those rows over every token.
        s3r::SelectArgs d{};
        d.q = p->q; d.k = p->k; d.v = p->v; d.idx = nullptr; d.o_comp = nullptr; d.gate = nullptr;
        d.out = p->out; d.o_sel = nullptr; d.lse = nullptr;
        d.n_tok = sp.n_spec; d.qmap = sp.spec; d.lse_stride = p->n_tok;
        d.heads = p->heads; d.block = p->block; d.kk = 0; d.scale = scale; d.is_bf16 = is_bf16;
        d.x.in = in;
        if (mfma) {
            void *kb_s = at(ws, L.kb_spec), *vb_s = at(ws, L.vb_spec);
            {
                StageTimer tm(S3R_STAGE_POOL, stream);
                S3R_HIP(s3r::launch_pool(p->q, p->k, p->v, nullptr, nullptr, nullptr, kb_s, vb_s, sp.n_spec, p->heads,
                                         64, is_bf16, sp.spec, in, stream),
                        "pool kernel launch (special tokens)");
            }
            d.kb = kb; d.vb = vb; d.n_keys = sp.n_img; d.n_blk = L.n_blk;      // image keys, then special keys
            d.blk_len = blk_len;
            d.kb2 = kb_s; d.vb2 = vb_s; d.n_keys2 = sp.n_spec;
            if (!is_bf16) {
                d.lo_off = a.lo_off;
                d.lo_off2 = static_cast<int64_t>(p->heads) * ((sp.n_spec + 63) / 64) * 64 * 64;
            }
            if (L.spec_split > 1) {
                d.x.n_split = L.spec_split;
                d.x.out_f32 = reinterpret_cast<float *>(at(ws, L.spec_part_o));
                d.x.part_lse = reinterpret_cast<float *>(at(ws, L.spec_part_lse));
            }
        } else {
            d.n_keys = p->n_tok; d.n_blk = (p->n_tok + p->block - 1) / p->block;  // every row, in place
        }
        StageTimer tm(S3R_STAGE_DENSE, stream);
        S3R_HIP(mfma ? s3r::launch_select_mfma(d, stream) : s3r::launch_select_generic(d, stream),
                "dense kernel launch (special tokens)");
        if (d.x.n_split > 1)
            S3R_HIP(s3r::launch_dense_combine(d.x.out_f32, d.x.part_lse, d.x.n_split, sp.n_spec, p->heads, sp.spec,
                                              p->out, is_bf16, stream),
                    "dense combine kernel launch (special tokens)");
    }
    return S3R_OK;
}

int speed3r_sparse_global_attn(const void *q, const void *k, const void *v, void *out, int64_t n_tok,
                               int heads, int head_dim, int block, int topk, void *stream)
{
    s3r_status st = check_shape(n_tok, heads, head_dim, block, topk, S3R_BF16);
    if (st != S3R_OK) return st;
    s3r_params p{};
    p.q = q; p.k = k; p.v = v; p.out = out;
    p.n_tok = n_tok; p.heads = heads; p.head_dim = head_dim; p.block = block; p.topk = topk;
    p.dtype = S3R_BF16; p.softmax_scale = 0.f; p.stream = stream;
    p.workspace_bytes = speed3r_workspace_bytes(n_tok, heads, head_dim, block, topk, 0, S3R_BF16);
    st = scratch_get(p.workspace_bytes, &p.workspace);
    if (st != S3R_OK) return st;
    return speed3r_sparse_global_attn_ex(&p);
}

int speed3r_sparse_global_attn_noalloc(const void *q, const void *k, const void *v, void *out, int64_t n_tok,
                                       int heads, int head_dim, int block, int topk, void *stream)
{
    s3r_status st = check_shape(n_tok, heads, head_dim, block, topk, S3R_BF16);
    if (st != S3R_OK) return st;
    const size_t need = speed3r_workspace_bytes(n_tok, heads, head_dim, block, topk, 0, S3R_BF16);
    if (need == 0 || need > kStaticScratchBytes)
        return fail(S3R_ERR_WORKSPACE,
                    "problem needs %zu bytes of scratch, the static scratch of this entry point holds %zu: "
                    "use speed3r_sparse_global_attn_ex with a caller workspace",
                    need, kStaticScratchBytes);
    s3r_params p{};
    p.q = q; p.k = k; p.v = v; p.out = out;
    p.n_tok = n_tok; p.heads = heads; p.head_dim = head_dim; p.block = block; p.topk = topk;
    p.dtype = S3R_BF16; p.softmax_scale = 0.f; p.stream = stream;
    p.workspace_bytes = kStaticScratchBytes;
    st = static_scratch(&p.workspace);
    if (st != S3R_OK) return st;
    // nothing of the previous call's scratch contents is relied on: every flag and counter the kernels
    // read is cleared by a kernel of this call
    t_no_events = true;
    st = speed3r_sparse_global_attn_ex(&p);
    t_no_events = false;
    return st;
}

s3r_status speed3r_pool_blocks(const void *q, const void *k, const void *v, float *qc, float *kc, float *vc,
                               int64_t n_tok, int heads, int head_dim, int block, s3r_dtype dtype, void *stream)
{
    s3r_status st = check_shape(n_tok, heads, head_dim, block, 1, dtype);
    if (st != S3R_OK) return st;
    if (!q || !k || !v || !qc || !kc || !vc) return fail(S3R_ERR_INVALID_ARG, "all six tensors must be non-null");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v)) return fail(S3R_ERR_INVALID_ARG, "device pointers must be 16-byte aligned");
    StageTimer tm(S3R_STAGE_POOL, static_cast<hipStream_t>(stream));
    S3R_HIP(s3r::launch_pool(q, k, v, qc, kc, vc, nullptr, nullptr, n_tok, heads, block, dtype == S3R_BF16,
                             s3r::TokenMap{}, s3r::InStride{}, static_cast<hipStream_t>(stream)),
            "pool kernel launch");
    return S3R_OK;
}

s3r_status speed3r_compress_attn_scores(const float *qc, const float *kc, const float *vc, float *s_guide,
                                        int64_t ld_s, float *o_comp, int64_t n_blk, int heads, int head_dim,
                                        float softmax_scale, int accurate_pv, void *stream)
{
    if (n_blk <= 0 || heads <= 0 || heads > 65535) return fail(S3R_ERR_INVALID_ARG, "n_blk and heads must be positive");
    if (head_dim != 64) return fail(S3R_ERR_UNSUPPORTED, "head_dim %d unsupported (must be 64)", head_dim);
    if (!qc || !kc || !vc || !s_guide || !o_comp) return fail(S3R_ERR_INVALID_ARG, "all five tensors must be non-null");
    if (ld_s < n_blk || ld_s % 4 != 0) return fail(S3R_ERR_INVALID_ARG, "ld_s must be >= n_blk and a multiple of 4");
    if (!aligned16(s_guide) || !aligned16(o_comp)) return fail(S3R_ERR_INVALID_ARG, "s_guide and o_comp must be 16-byte aligned");
    const int64_t tiles = s3r::pooled_tiles_padded(n_blk);
    const size_t arr = align_up(static_cast<size_t>(heads) * tiles * 32 * 64 * 2);
    void *ws = nullptr;
    s3r_status st = scratch_get(8 * arr, &ws);
    if (st != S3R_OK) return st;
    void *tile[8];
    for (int a = 0; a < 8; ++a) tile[a] = at(ws, a * arr);
    return run_compress_topk(qc, kc, vc, tile, s_guide, ld_s, heads, o_comp, nullptr, n_blk, tiles, heads, 0,
                             resolve_scale(softmax_scale, head_dim), accurate_pv != 0, false, nullptr, FusedBufs{},
                             static_cast<hipStream_t>(stream));
}

s3r_status speed3r_compress_attn_topk(const float *qc, const float *kc, const float *vc, float *o_comp, int32_t *idx,
                                      int64_t n_blk, int heads, int head_dim, int topk, float softmax_scale,
                                      int accurate_pv, void *stream)
{
    if (n_blk <= 0 || heads <= 0 || heads > 65535 || topk <= 0)
        return fail(S3R_ERR_INVALID_ARG, "n_blk, heads and topk must be positive");
    if (head_dim != 64) return fail(S3R_ERR_UNSUPPORTED, "head_dim %d unsupported (must be 64)", head_dim);
    if (!qc || !kc || !vc || !o_comp || !idx) return fail(S3R_ERR_INVALID_ARG, "all five tensors must be non-null");
    if (!aligned16(qc) || !aligned16(kc) || !aligned16(o_comp))
        return fail(S3R_ERR_INVALID_ARG, "qc, kc and o_comp must be 16-byte aligned");
    if (n_blk * heads > 0x7fffffffLL) return fail(S3R_ERR_UNSUPPORTED, "n_blk * heads exceeds 2^31 - 1");
    const int kk = static_cast<int>(topk < n_blk ? topk : n_blk);
    if (kk > s3r::kFusedTopkMaxK) return fail(S3R_ERR_UNSUPPORTED, "k = %d exceeds %d", kk, s3r::kFusedTopkMaxK);
    if (g_kernel_choice == 2) return fail(S3R_ERR_UNSUPPORTED, "TopK inside the sweep is switched off (kernel choice 2)");
    // scratch: six operand tile arrays, bounds, candidate lists and counts, overflow word, and S for the
    // fallback in head chunks
    const int64_t tiles = s3r::pooled_tiles_padded(n_blk);
    const size_t arr = align_up(static_cast<size_t>(heads) * tiles * 32 * 64 * 2);
    const size_t rows = static_cast<size_t>(heads) * n_blk;
    const int64_t ld_s = (n_blk + 63) / 64 * 64;
    const size_t per_head_s = static_cast<size_t>(n_blk) * ld_s * sizeof(float);
    int64_t hc = static_cast<int64_t>(kScoreBytesCap / per_head_s);
    if (hc < 1) hc = 1;
    if (hc > heads) hc = heads;
    size_t off = 8 * arr;
    auto take = [&](size_t bytes) { const size_t o = off; off += align_up(bytes); return o; };
    const size_t o_slots = take(static_cast<size_t>(heads) * 3 * s3r::kStatSlots * sizeof(unsigned));
    const size_t o_stats = take(static_cast<size_t>(heads) * sizeof(s3r::HeadStats));
    const size_t o_thr = take(rows * sizeof(float));
    const size_t o_cand = take(rows * 2 * kCandCap * sizeof(int32_t));
    const size_t o_cnt = take(rows * 2 * sizeof(int));
    const size_t o_ovf = take(sizeof(int));
    const size_t o_s = take(per_head_s * hc);
    void *ws = nullptr;
    s3r_status st = scratch_get(off, &ws);
    if (st != S3R_OK) return st;
    void *tile[8];
    for (int a = 0; a < 8; ++a) tile[a] = at(ws, a * arr);
    FusedBufs fb;
    fb.stat_slots = at(ws, o_slots);
    fb.head_stats = reinterpret_cast<s3r::HeadStats *>(at(ws, o_stats));
    fb.thr = reinterpret_cast<float *>(at(ws, o_thr));
    fb.cand = reinterpret_cast<int32_t *>(at(ws, o_cand));
    fb.cand_count = reinterpret_cast<int *>(at(ws, o_cnt));
    fb.overflow = reinterpret_cast<int *>(at(ws, o_ovf));
    return run_compress_topk(qc, kc, vc, tile, reinterpret_cast<float *>(at(ws, o_s)), ld_s, static_cast<int>(hc), o_comp,
                             idx, n_blk, tiles, heads, kk, resolve_scale(softmax_scale, head_dim), accurate_pv != 0, true,
                             nullptr, fb, static_cast<hipStream_t>(stream));
}

s3r_status speed3r_topk_blocks(const float *s_guide, int64_t ld_s, int32_t *idx, int64_t n_blk, int heads,
                               int topk, void *stream)
{
    if (n_blk <= 0 || heads <= 0 || topk <= 0) return fail(S3R_ERR_INVALID_ARG, "n_blk, heads and topk must be positive");
    if (!s_guide || !idx) return fail(S3R_ERR_INVALID_ARG, "s_guide and idx must be non-null");
    if (ld_s < n_blk) return fail(S3R_ERR_INVALID_ARG, "ld_s must be >= n_blk");
    if (n_blk * heads > 0x7fffffffLL) return fail(S3R_ERR_UNSUPPORTED, "n_blk * heads exceeds 2^31 - 1");
    const int kk = static_cast<int>(topk < n_blk ? topk : n_blk);
    StageTimer tm(S3R_STAGE_TOPK, static_cast<hipStream_t>(stream));
    S3R_HIP(s3r::launch_topk(s_guide, ld_s, idx, n_blk, n_blk * heads, kk, nullptr, static_cast<hipStream_t>(stream)),
            "topk kernel launch");
    return S3R_OK;
}

s3r_status speed3r_select_attn(const void *q, const void *k, const void *v, const int32_t *idx,
                               const float *o_comp, const void *gate_logits, void *out, void *o_sel,
                               float *lse, int64_t n_tok, int heads, int head_dim, int block, int kk,
                               s3r_dtype dtype, float softmax_scale, void *stream)
{
    s3r_status st = check_shape(n_tok, heads, head_dim, block, kk, dtype);
    if (st != S3R_OK) return st;
    if (!q || !k || !v || !idx || !out) return fail(S3R_ERR_INVALID_ARG, "q, k, v, idx and out must be non-null");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(gate_logits) ||
        !aligned16(o_sel) || !aligned16(o_comp))
        return fail(S3R_ERR_INVALID_ARG, "device pointers must be 16-byte aligned");
    const int64_t n_blk = (n_tok + block - 1) / block;
    if (kk > n_blk) return fail(S3R_ERR_INVALID_ARG, "k (%d) exceeds the number of blocks (%lld)", kk, static_cast<long long>(n_blk));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool mfma = mfma_ok(dtype, block);
    s3r::SelectArgs a{};
    if (mfma) {
        const size_t blocked = align_up(static_cast<size_t>(heads) * n_blk * block * 64 * 2 * tile_parts(dtype));
        void *ws = nullptr;
        st = scratch_get(2 * blocked, &ws);
        if (st != S3R_OK) return st;
        a.kb = ws;
        a.vb = at(ws, blocked);
        a.lo_off = dtype == S3R_BF16 ? 0 : static_cast<int64_t>(heads) * n_blk * block * 64;
        StageTimer tm(S3R_STAGE_POOL, s);
        S3R_HIP(s3r::launch_pool(q, k, v, nullptr, nullptr, nullptr, const_cast<void *>(a.kb),
                                 const_cast<void *>(a.vb), n_tok, heads, block, dtype == S3R_BF16, s3r::TokenMap{},
                                 s3r::InStride{}, s),
                "pool kernel launch");
    }
    a.q = q; a.k = k; a.v = v; a.idx = idx; a.o_comp = o_comp; a.gate = gate_logits; a.out = out;
    a.o_sel = o_sel; a.lse = lse; a.n_tok = n_tok; a.n_keys = n_tok; a.lse_stride = n_tok; a.n_blk = n_blk;
    a.heads = heads; a.block = block;
    a.kk = kk; a.scale = resolve_scale(softmax_scale, head_dim); a.is_bf16 = dtype == S3R_BF16;
    StageTimer tm(S3R_STAGE_SELECT, s);
    S3R_HIP(mfma ? s3r::launch_select_mfma(a, s) : s3r::launch_select_generic(a, s), "select kernel launch");
    return S3R_OK;
}

s3r_status speed3r_probe_select_loads(const void *q, const void *k, const void *v, const int32_t *idx, void *out,
                                      int64_t n_tok, int heads, int head_dim, int block, int kk, int ring_stages,
                                      int wg_per_cu, void *stream)
{
    s3r_status st = check_shape(n_tok, heads, head_dim, block, kk, S3R_BF16);
    if (st != S3R_OK) return st;
    if (block != 64 && block != 128) return fail(S3R_ERR_UNSUPPORTED, "the load probe covers blocks of 64 and 128 tokens");
    if (ring_stages != 0 && (ring_stages < 2 || ring_stages > 4))
        return fail(S3R_ERR_INVALID_ARG, "ring_stages (%d) must be 0 or 2..4", ring_stages);
    if (wg_per_cu < 0 || wg_per_cu > 5 || (wg_per_cu > 0 && 160 / wg_per_cu < 16 * (ring_stages ? ring_stages : 2)))
        return fail(S3R_ERR_INVALID_ARG, "wg_per_cu (%d) must be 0 or 1..5 and leave each workgroup room for a ring of %d stages of 16 KiB",
                    wg_per_cu, ring_stages ? ring_stages : 2);
    if (!q || !k || !v || !idx || !out) return fail(S3R_ERR_INVALID_ARG, "q, k, v, idx and out must be non-null");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out))
        return fail(S3R_ERR_INVALID_ARG, "device pointers must be 16-byte aligned");
    const int64_t n_blk = (n_tok + block - 1) / block;
    if (kk > n_blk) return fail(S3R_ERR_INVALID_ARG, "k (%d) exceeds the number of blocks (%lld)", kk, static_cast<long long>(n_blk));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t blocked = align_up(static_cast<size_t>(heads) * n_blk * block * 64 * 2);
    void *ws = nullptr;
    st = scratch_get(2 * blocked, &ws);
    if (st != S3R_OK) return st;
    s3r::SelectArgs a{};
    a.kb = ws;
    a.vb = at(ws, blocked);
    {
        StageTimer tm(S3R_STAGE_POOL, s);
        S3R_HIP(s3r::launch_pool(q, k, v, nullptr, nullptr, nullptr, const_cast<void *>(a.kb), const_cast<void *>(a.vb),
                                 n_tok, heads, block, true, s3r::TokenMap{}, s3r::InStride{}, s),
                "pool kernel launch");
    }
    a.q = q; a.k = k; a.v = v; a.idx = idx; a.out = out;
    a.n_tok = n_tok; a.n_keys = n_tok; a.lse_stride = n_tok; a.n_blk = n_blk;
    a.heads = heads; a.block = block; a.kk = kk; a.scale = 1.f; a.is_bf16 = true; a.loads_only = true;
    a.probe_stages = ring_stages; a.probe_wg_per_cu = wg_per_cu;
    StageTimer tm(S3R_STAGE_SELECT, s);
    S3R_HIP(s3r::launch_select_mfma(a, s), "select (loads only) kernel launch");
    return S3R_OK;
}

s3r_status speed3r_dense_attn(const void *q, const void *k, const void *v, void *out, float *lse, int64_t n_tok,
                              int heads, int head_dim, s3r_dtype dtype, float softmax_scale, void *stream)
{
    const int block = 64;
    s3r_status st = check_shape(n_tok, heads, head_dim, block, 1, dtype);
    if (st != S3R_OK) return st;
    if (!q || !k || !v || !out) return fail(S3R_ERR_INVALID_ARG, "q, k, v and out must be non-null");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out))
        return fail(S3R_ERR_INVALID_ARG, "device pointers must be 16-byte aligned");
    const int64_t n_blk = (n_tok + block - 1) / block;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool mfma = mfma_ok(dtype, block);
    s3r::SelectArgs a{};
    if (mfma) {
        const size_t blocked = align_up(static_cast<size_t>(heads) * n_blk * block * 64 * 2 * tile_parts(dtype));
        void *ws = nullptr;
        st = scratch_get(2 * blocked, &ws);
        if (st != S3R_OK) return st;
        a.kb = ws;
        a.vb = at(ws, blocked);
        a.lo_off = dtype == S3R_BF16 ? 0 : static_cast<int64_t>(heads) * n_blk * block * 64;
        StageTimer tm(S3R_STAGE_POOL, s);
        S3R_HIP(s3r::launch_pool(q, k, v, nullptr, nullptr, nullptr, const_cast<void *>(a.kb),
                                 const_cast<void *>(a.vb), n_tok, heads, block, dtype == S3R_BF16, s3r::TokenMap{},
                                 s3r::InStride{}, s),
                "pool kernel launch");
    }
    a.q = q; a.k = k; a.v = v; a.idx = nullptr; a.o_comp = nullptr; a.gate = nullptr; a.out = out;
    a.o_sel = nullptr; a.lse = lse; a.n_tok = n_tok; a.n_keys = n_tok; a.lse_stride = n_tok; a.n_blk = n_blk;
    a.heads = heads; a.block = block;
    a.kk = 0; a.scale = resolve_scale(softmax_scale, head_dim); a.is_bf16 = dtype == S3R_BF16;
    StageTimer tm(S3R_STAGE_DENSE, s);
    S3R_HIP(mfma ? s3r::launch_select_mfma(a, s) : s3r::launch_select_generic(a, s), "dense kernel launch");
    return S3R_OK;
}

}  // extern "C"
