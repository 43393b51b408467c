// libslimdp host side: the C ABI of include/slimdp.h.  Argument checks, workspace carving
// and kernel launches only; every step of the path runs in the kernels of slimdp_kernels.h.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "slimdp.h"
#include "slimdp_kernels.h"

using namespace slimdp;

namespace {

thread_local std::string g_create_error;

struct Tiling {
    std::vector<uint32_t> tile_start;      // T+1
    std::vector<uint32_t> tile_seg;        // T
    std::vector<uint32_t> seg_first_tile;  // n_seg+1
    bool word_aligned = true;              // every tile starts on a bitmap word
    bool quad_aligned = true;              // every tile starts on a Philox block (index divisible by 4)
};

bool valid_shape(uint64_t n, uint32_t n_seg, const uint64_t* seg_off)
{
    if (n == 0 || n > SLIMDP_MAX_N || n_seg == 0 || n_seg > SLIMDP_MAX_SEGMENTS || !seg_off) return false;
    if (seg_off[0] != 0 || seg_off[n_seg] != n) return false;
    for (uint32_t s = 0; s < n_seg; ++s)
        if (seg_off[s + 1] <= seg_off[s]) return false;
    return true;
}

Tiling make_tiling(uint64_t n, uint32_t n_seg, const uint64_t* seg_off)
{
    Tiling tl;
    tl.seg_first_tile.resize(n_seg + 1);
    for (uint32_t s = 0; s < n_seg; ++s) {
        tl.seg_first_tile[s] = (uint32_t)tl.tile_seg.size();
        for (uint64_t a = seg_off[s]; a < seg_off[s + 1]; a += TILE) {
            tl.tile_start.push_back((uint32_t)a);
            tl.tile_seg.push_back(s);
            if (a & 31u) tl.word_aligned = false;
            if (a & 3u) tl.quad_aligned = false;
        }
    }
    tl.seg_first_tile[n_seg] = (uint32_t)tl.tile_seg.size();
    tl.tile_start.push_back((uint32_t)n);   // n <= 2^31
    return tl;
}

uint64_t count_tiles(uint64_t n, uint32_t n_seg, const uint64_t* seg_off)
{
    (void)n;
    uint64_t T = 0;
    for (uint32_t s = 0; s < n_seg; ++s) T += (seg_off[s + 1] - seg_off[s] + TILE - 1) / TILE;
    return T;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// One linear pass hands out the workspace; run once with base == nullptr to size it.
struct Carver {
    char* base;
    size_t pos = 0;
    explicit Carver(char* b) : base(b) {}
    template <class Tp> Tp* take(size_t count)
    {
        pos = align_up(pos, 256);
        Tp* p = base ? reinterpret_cast<Tp*>(base + pos) : nullptr;
        pos += count * sizeof(Tp);
        return p;
    }
};

}  // namespace

struct slimdp_ctx {
    uint64_t n = 0;
    uint32_t maxW = 0, n_seg = 0, T = 0;
    uint64_t seed = 0;
    hipStream_t stream = nullptr;
    // an announced explorer draw can run beside the caller's stream: pure integer work that fills the
    // arithmetic units the memory-bound kernels leave idle
    hipStream_t side = nullptr;
    hipEvent_t ev_consumed = nullptr;      // main stream: everything enqueued before a side-stream draw (readers of its buffers)
    hipEvent_t ev_drawn = nullptr;         // side stream: the announced draw is complete
    bool side_pending = false;             // a side draw was launched and the main stream has not waited for it yet
    // asynchronous slimdp_sample_explore requests (option "explore_async") that the main stream has not waited for yet:
    // their completion events on the side stream and the address ranges they write
    static constexpr int N_PENDING = 4;
    struct PendingExplore {
        hipEvent_t ev = nullptr;
        bool live = false;
        uint64_t seq = 0;
        uint32_t nw = 0;
        uintptr_t idx[MAXW] = {}, off[MAXW] = {};
        uint64_t idx_bytes = 0, off_bytes = 0;
    } pend[N_PENDING];
    uint64_t pend_seq = 0;
    int64_t opt_explore_async = 0;
    int device = 0, cus = 256;
    std::vector<uint64_t> seg_off;
    Tiling tl;
    char* ws = nullptr;
    size_t ws_bytes = 0;
    uint64_t keys_stride = 0;
    // device tables
    uint32_t *d_tile_start = nullptr, *d_tile_seg = nullptr, *d_seg_first_tile = nullptr, *d_flags = nullptr;
    // core selection
    SegState* c_state = nullptr;
    uint32_t *c_hist = nullptr, *c_gt_bits = nullptr, *c_cand_bits = nullptr, *c_cand_keys = nullptr;
    uint32_t* c_chunk_sum = nullptr;
    uint32_t *c_pred = nullptr, *c_skip = nullptr, *c_used = nullptr;   // predicted level-0 threshold bin per segment; "the scoring pass classified against the right bin"
    bool cls_by_score = false;                       // the last scoring pass classified whole tiles against c_pred
    uint32_t *c_cnt_gt = nullptr, *c_cnt_cand = nullptr, *c_cnt_sel = nullptr, *c_cnt_tie = nullptr, *c_tie_pre = nullptr;
    // explorer selection (batch = worker)
    SegState* e_state = nullptr;
    SegState* e_draw_state = nullptr;      // zone bounds of the announced draw (side stream)
    uint32_t *e_hist = nullptr, *e_sure_bits = nullptr, *e_cand_bits = nullptr;
    uint32_t* e_pair_keys = nullptr;       // narrow zones: per sub-tile a slot of (key, offset) pairs
    uint64_t pair_stride = 0;              // words per worker of the pair slots
    uint32_t* e_cand_keys = nullptr;       // wide zones: candidate keys compacted per sub-tile over the whole index range;
                                           // its own allocation, made by the first request that needs it
    uint32_t *e_cnt_gt = nullptr, *e_nsure = nullptr, *e_list_count = nullptr, *e_chunk_sum = nullptr, *e_tie_list = nullptr;
    uint4* e_list = nullptr;
    uint64_t list_cap = 0;
    uint32_t n_chunks = 0;
    uint32_t *e_cnt_cand = nullptr, *e_cnt_sel = nullptr, *e_cnt_tie = nullptr, *e_tie_pre = nullptr;
    // host state
    uint64_t epoch = 0;
    bool hist_pending = false;
    const float* hist_score = nullptr;
    int64_t opt_force_fallback = 0;
    int64_t opt_per_tile_tail = 0;
    int64_t opt_strided = 1;               // flat model: persistent blocks take every P-th tile
    int64_t opt_side_blocks = 2;           // blocks per compute unit of a side-stream draw
    int64_t opt_hint_mode = 0;             // 0: the announced draw rides inside slimdp_score; 1: side stream
    // speculative packing: its own allocation, made when the option is switched on
    struct Spec {
        bool on = false;
        char* mem = nullptr;
        uint32_t* lo[2] = {nullptr, nullptr};   // capture bound per segment: [cur] read by the scoring pass, the other written by the selection
        uint32_t* fail = nullptr;               // per segment: the selection's threshold fell below the capture bound
        uint2* bits = nullptr;
        float* vals = nullptr;
        int cur = 0;
        bool next_written = false;              // a selection has refreshed lo[cur ^ 1] since the last capture
        bool bound_valid = false;               // lo[cur] comes from a selection (else: nothing, or a sampled estimate)
        uint32_t* sample = nullptr;             // keys of the sampled significances (flat model)
        // the capture made by the last slimdp_score, and the selection that used that score
        bool captured = false;
        const float* score = nullptr;
        const float* g[MAXW] = {};
        uint32_t W = 0;
        int vec_ok = 0;
        uint64_t core_epoch = 0;                // 0: no selection on the captured score yet
    } spec;
    int64_t opt_pack_nbuf = 2;
    int64_t opt_pack_kernel = 1;           // general pack: 1 = loading and storing waves apart, 0 = one set of waves
    int64_t opt_pull_kernel = 1;           // local overwrite of a pull: 1 = a pass that streams the local models, 0 = scattered writes
    int64_t opt_build_blocks = 4;
    int64_t opt_pack_core_blocks = 0;      // blocks per compute unit of the pack from the capture (0: one per 1024 list entries)
    int64_t opt_core_predict = 1;          // the flat scoring kernel sorts whole tiles against the predicted threshold bin (0: never; 2: test, a wrong bin)          // blocks per compute unit of the core candidate pass
    int64_t opt_score_pipeline = 1;        // flat aligned models: the scoring kernel with two rounds of loads in flight
    int64_t opt_expected_core = -1;        // core size the next selection will ask for (flat model), if the caller says
    int64_t opt_estimate_bias = 0;         // test switch: added to a sampled capture bound
    uint64_t last_K = 0;                   // core size of the last selection
    bool have_last_K = false;
    // explorer draw announced by slimdp_explore_hint (hint) / already drawn inside slimdp_score (pre)
    struct Draw {
        bool valid = false;
        uint64_t iteration = 0;
        uint32_t worker0 = 0, n_workers = 0;
        std::vector<uint64_t> k_seg, m_seg;
        bool pairs = false;          // drawn in the short-list format
        bool same(uint64_t it, uint32_t w0, uint32_t nw, const uint64_t* k, const uint64_t* m, uint32_t n_seg) const
        {
            if (!valid || it != iteration || w0 != worker0 || nw != n_workers) return false;
            for (uint32_t s = 0; s < n_seg; ++s)
                if (k[s] != k_seg[s] || m[s] != m_seg[s]) return false;
            return true;
        }
    } hint, pre;
    std::string err;
};

namespace {

// Tables and the buffers of the core selection (all that a selection without explorers needs).
void carve_core(slimdp_ctx* c, Carver& cv)
{
    const size_t T = c->T, S = c->n_seg;
    c->d_tile_start = cv.take<uint32_t>(T + 1);
    c->d_tile_seg = cv.take<uint32_t>(T);
    c->d_seg_first_tile = cv.take<uint32_t>(S + 1);
    c->d_flags = cv.take<uint32_t>(64);
    c->c_state = cv.take<SegState>(S);
    c->c_hist = cv.take<uint32_t>(S * H_STRIDE);
    c->c_gt_bits = cv.take<uint32_t>(T * TILE_WORDS);
    c->c_cand_bits = cv.take<uint32_t>(T * TILE_WORDS);
    c->c_cand_keys = cv.take<uint32_t>(c->keys_stride);
    c->c_cnt_gt = cv.take<uint32_t>(T * SUBS);
    c->c_cnt_cand = cv.take<uint32_t>(T * SUBS);
    c->c_cnt_sel = cv.take<uint32_t>(T);
    c->c_cnt_tie = cv.take<uint32_t>(T);
    c->c_tie_pre = cv.take<uint32_t>(T + 1);
    c->c_chunk_sum = cv.take<uint32_t>(2 * c->n_chunks);
    c->c_pred = cv.take<uint32_t>(S);
    c->c_skip = cv.take<uint32_t>(S);
    c->c_used = cv.take<uint32_t>(S);
}

void carve(slimdp_ctx* c, Carver& cv)
{
    const size_t T = c->T, S = c->n_seg, B = c->maxW;
    carve_core(c, cv);
    c->e_state = cv.take<SegState>(B * S);
    c->e_draw_state = cv.take<SegState>(B * S);
    c->e_hist = cv.take<uint32_t>(B * S * H_STRIDE);
    c->e_sure_bits = cv.take<uint32_t>(B * T * TILE_WORDS);
    c->e_cand_bits = cv.take<uint32_t>(B * T * TILE_WORDS);
    c->e_cnt_gt = cv.take<uint32_t>(B * T * SUBS);
    c->e_nsure = cv.take<uint32_t>(B * S);
    c->e_list_count = cv.take<uint32_t>(64);          // [0] candidates listed, [1] ties listed
    c->e_tie_list = cv.take<uint32_t>(TIE_CAP);
    c->e_chunk_sum = cv.take<uint32_t>(2 * B * c->n_chunks);   // tie sums, then offset sums
    c->e_list = cv.take<uint4>(c->list_cap);
    c->e_pair_keys = cv.take<uint32_t>(B * c->pair_stride);
    c->e_cnt_cand = cv.take<uint32_t>(B * T * SUBS);
    c->e_cnt_sel = cv.take<uint32_t>(B * T);
    c->e_cnt_tie = cv.take<uint32_t>(B * T);
    c->e_tie_pre = cv.take<uint32_t>(B * (T + 1));
}

int fail(slimdp_ctx* c, int code, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c) c->err = buf; else g_create_error = buf;
    return code;
}

int hip_fail(slimdp_ctx* c, hipError_t e, const char* what)
{
    return fail(c, SLIMDP_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

#define SLIMDP_HIP(c, call)                                        \
    do {                                                           \
        hipError_t e__ = (call);                                   \
        if (e__ != hipSuccess) return hip_fail((c), e__, #call);   \
    } while (0)

#define SLIMDP_LAUNCHED(c, name)                                   \
    do {                                                           \
        hipError_t e__ = hipGetLastError();                        \
        if (e__ != hipSuccess) return hip_fail((c), e__, name);    \
    } while (0)

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

uint32_t fill_grid(uint64_t count) { uint64_t g = (count + 255) / 256; return (uint32_t)(g < 1 ? 1 : (g > 4096 ? 4096 : g)); }

int fill(slimdp_ctx* c, uint32_t* p, uint64_t count, uint32_t v)
{
    if (count == 0) return SLIMDP_OK;
    hipLaunchKernelGGL(k_fill_u32, dim3(fill_grid(count)), dim3(256), 0, c->stream, p, count, v);
    SLIMDP_LAUNCHED(c, "k_fill_u32");
    return SLIMDP_OK;
}

int init_states(slimdp_ctx* c, SegState* st, const std::vector<SegInit>& init, uint32_t nbatch, int core,
                hipStream_t stream = nullptr)
{
    if (!stream) stream = c->stream;
    for (uint32_t s0 = 0; s0 < c->n_seg; s0 += INIT_CHUNK) {
        SegInitChunk chunk;
        const uint32_t cnt = (c->n_seg - s0 < (uint32_t)INIT_CHUNK) ? c->n_seg - s0 : (uint32_t)INIT_CHUNK;
        memset(&chunk, 0, sizeof chunk);
        for (uint32_t j = 0; j < cnt; ++j) chunk.s[j] = init[s0 + j];
        const uint32_t threads = cnt * nbatch;
        hipLaunchKernelGGL(k_init_state, dim3((threads + 255) / 256), dim3(256), 0, stream, st, chunk, s0, cnt,
                           c->n_seg, nbatch, core);
        SLIMDP_LAUNCHED(c, "k_init_state");
    }
    return SLIMDP_OK;
}

uint32_t persistent_blocks(const slimdp_ctx* c, uint32_t per_cu, uint32_t nbatch)
{
    uint64_t p = (uint64_t)c->cus * per_cu / (nbatch ? nbatch : 1);
    if (p < 32) p = 32;
    if (p > c->T) p = c->T;
    return (uint32_t)p;
}

// Levels 1, 2, per-tile counts, scan over tiles and ordered emission, shared by the core
// (after k_core_build, which already filled the level-1 histogram) and the explorer.
template <int KPL, int BPW>
int finish_selection(slimdp_ctx* c, uint32_t nbatch, SegState* st, uint32_t* hist, const uint32_t* gt_bits,
                     const uint32_t* cand_bits, const uint32_t* cand_keys, const uint32_t* cnt_gt,
                     const uint32_t* cnt_cand, uint32_t* cnt_sel, uint32_t* cnt_tie, uint32_t* tie_pre,
                     uint64_t keys_stride, bool level1_done, const MutPtrTab& out_off, const MutPtrTab& out_idx,
                     uint32_t expected, uint32_t* pub_bits, const uint32_t* excl_bits, const uint32_t* gate,
                     uint32_t* chunk_sum, SpecTau sp = SpecTau{nullptr, nullptr, nullptr},
                     CorePred cp = CorePred{nullptr, nullptr, nullptr, 0}, hipStream_t stream = nullptr)
{
    if (!stream) stream = c->stream;
    const uint32_t T = c->T, S = c->n_seg;
    const dim3 wave_grid((T + 3) / 4, (nbatch + BPW - 1) / BPW);     // a wave serves its tile for BPW batches
    if (!level1_done) {
        hipLaunchKernelGGL((k_list_hist<KPL, BPW>), wave_grid, dim3(BLOCK), 0, stream, c->n, c->d_tile_start,
                           c->d_tile_seg, T, S, nbatch, st, hist, (uint32_t)H_L1, 1, cand_keys, cnt_cand, keys_stride, gate);
        SLIMDP_LAUNCHED(c, "k_list_hist(1)");
    }
    hipLaunchKernelGGL(k_threshold, dim3(S, nbatch), dim3(256), 0, stream, st, hist, 1, (uint32_t)H_L1, S, 0, c->d_flags,
                       nullptr, gate ? 1 : 0, SpecTau{nullptr, nullptr, nullptr}, CorePred{nullptr, nullptr, nullptr, 0});
    SLIMDP_LAUNCHED(c, "k_threshold(1)");
    hipLaunchKernelGGL((k_list_hist<KPL, BPW>), wave_grid, dim3(BLOCK), 0, stream, c->n, c->d_tile_start, c->d_tile_seg,
                       T, S, nbatch, st, hist, (uint32_t)H_L2, 2, cand_keys, cnt_cand, keys_stride, gate);
    SLIMDP_LAUNCHED(c, "k_list_hist(2)");
    hipLaunchKernelGGL(k_threshold, dim3(S, nbatch), dim3(256), 0, stream, st, hist, 2, (uint32_t)H_L2, S, 0, c->d_flags,
                       nullptr, gate ? 1 : 0, sp, cp);
    SLIMDP_LAUNCHED(c, "k_threshold(2)");
    hipLaunchKernelGGL((k_count<KPL, BPW>), wave_grid, dim3(BLOCK), 0, stream, c->n, c->d_tile_start, c->d_tile_seg, T, S,
                       nbatch, st, cand_keys, cnt_cand, cnt_gt, keys_stride, cnt_sel, cnt_tie, gate);
    SLIMDP_LAUNCHED(c, "k_count");
    const dim3 scan_grid(c->n_chunks, nbatch);
    hipLaunchKernelGGL(k_tile_scan<0>, scan_grid, dim3(1024), 0, stream, c->d_tile_seg, c->d_seg_first_tile, T, S, st, cnt_sel,
                       cnt_tie, tie_pre, chunk_sum, out_off, chunk_sum + (size_t)nbatch * c->n_chunks, gate);
    SLIMDP_LAUNCHED(c, "k_tile_scan(ties)");
    hipLaunchKernelGGL(k_tile_scan<1>, scan_grid, dim3(1024), 0, stream, c->d_tile_seg, c->d_seg_first_tile, T, S, st, cnt_sel,
                       cnt_tie, tie_pre, chunk_sum, out_off, chunk_sum + (size_t)nbatch * c->n_chunks, gate);
    SLIMDP_LAUNCHED(c, "k_tile_scan(offsets)");
    hipLaunchKernelGGL((k_emit<KPL, BPW>), wave_grid, dim3(BLOCK), 0, stream, c->n, c->d_tile_start, c->d_tile_seg,
                       c->d_seg_first_tile, T, S, nbatch, st, gt_bits, cand_bits, cand_keys, keys_stride, tie_pre, out_off,
                       out_idx, expected, pub_bits, excl_bits, (uint32_t)((c->n + 31) / 32), gate, chunk_sum,
                       chunk_sum + (size_t)nbatch * c->n_chunks, c->n_chunks, c->d_flags);
    SLIMDP_LAUNCHED(c, "k_emit");
    return SLIMDP_OK;
}

template <class P> bool table_ok(P const* tab, uint32_t nw, bool allow_null_entries = false)
{
    if (!tab) return false;
    if (!allow_null_entries)
        for (uint32_t q = 0; q < nw; ++q)
            if (!tab[q]) return false;
    return true;
}

template <class Tab, class P> Tab make_tab(P const* tab, uint32_t nw)
{
    Tab t;
    for (int q = 0; q < MAXW; ++q) t.p[q] = nullptr;
    if (tab)
        for (uint32_t q = 0; q < nw; ++q) t.p[q] = (decltype(t.p[0]))tab[q];
    return t;
}

// The context's stream waits for whatever the side stream still has in flight (an announced draw, asynchronous
// explorer requests) before it touches what that work reads or writes.
int wait_for_side(slimdp_ctx* c)
{
    int last = -1;
    for (int j = 0; j < slimdp_ctx::N_PENDING; ++j)
        if (c->pend[j].live && (last < 0 || c->pend[j].seq > c->pend[last].seq)) last = j;
    if (last >= 0) {                     // the side stream runs in order: the newest request's event covers all
        SLIMDP_HIP(c, hipStreamWaitEvent(c->stream, c->pend[last].ev, 0));
        for (int j = 0; j < slimdp_ctx::N_PENDING; ++j) c->pend[j].live = false;
        c->side_pending = false;         // a draw that preceded it on the same stream is done as well
    }
    if (c->side_pending) {
        SLIMDP_HIP(c, hipStreamWaitEvent(c->stream, c->ev_drawn, 0));
        c->side_pending = false;
    }
    return SLIMDP_OK;
}

// A call that reads explorer lists waits for the asynchronous requests that write any of them (address ranges
// compared, so views into the same allocation count), and with them for every older request; requests whose
// arrays it does not touch keep running beside it.
int wait_for_lists(slimdp_ctx* c, uint32_t nw, const uint32_t* const* expl_idx, const uint32_t* const* expl_off,
                   const uint64_t* m_w)
{
    int hit = -1;
    for (int j = 0; j < slimdp_ctx::N_PENDING; ++j) {
        const slimdp_ctx::PendingExplore& p = c->pend[j];
        if (!p.live) continue;
        bool touches = false;
        for (uint32_t a = 0; a < nw && !touches; ++a)
            for (uint32_t b = 0; b < p.nw && !touches; ++b) {
                const uintptr_t i0 = reinterpret_cast<uintptr_t>(expl_idx ? expl_idx[a] : nullptr);
                const uintptr_t o0 = reinterpret_cast<uintptr_t>(expl_off ? expl_off[a] : nullptr);
                if (i0 && i0 < p.idx[b] + p.idx_bytes && p.idx[b] < i0 + (m_w ? m_w[a] : 0) * 4 + 4) touches = true;
                if (o0 && o0 < p.off[b] + p.off_bytes && p.off[b] < o0 + p.off_bytes) touches = true;
            }
        if (touches && (hit < 0 || p.seq > c->pend[hit].seq)) hit = j;
    }
    if (hit < 0) return SLIMDP_OK;
    SLIMDP_HIP(c, hipStreamWaitEvent(c->stream, c->pend[hit].ev, 0));
    const uint64_t upto = c->pend[hit].seq;
    for (int j = 0; j < slimdp_ctx::N_PENDING; ++j)
        if (c->pend[j].live && c->pend[j].seq <= upto) c->pend[j].live = false;
    return SLIMDP_OK;
}

int check_epoch(slimdp_ctx* c, uint64_t core_epoch)
{
    if (c->epoch == 0 || core_epoch != c->epoch)
        return fail(c, SLIMDP_ERR_STALE_CORE, "core_epoch %llu is not the context's current core epoch %llu",
                    (unsigned long long)core_epoch, (unsigned long long)c->epoch);
    return SLIMDP_OK;
}

// Explorer requests whose zones are not narrow compact their candidate keys over the whole index range: that buffer
// (4 bytes per parameter and worker) is allocated by the first such request and kept.
int ensure_wide_keys(slimdp_ctx* c)
{
    if (c->e_cand_keys) return SLIMDP_OK;
    const size_t bytes = (size_t)c->maxW * c->keys_stride * sizeof(uint32_t);
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&c->e_cand_keys), bytes);
    if (e != hipSuccess) {
        c->e_cand_keys = nullptr;
        return fail(c, SLIMDP_ERR_WORKSPACE, "explorer with wide zones: hipMalloc(%zu bytes): %s", bytes, hipGetErrorString(e));
    }
    return SLIMDP_OK;
}

// Probability that one sub-tile holds more than PAIR_CAP candidates of one draw when lambda are expected (the draw
// marks each of its up to 1024 words independently: Poisson tail, summed directly so that tiny values keep their digits).
double pair_overflow_prob(double lambda)
{
    if (lambda <= 0.0) return 0.0;
    const int j0 = (int)PAIR_CAP + 1;
    double term = std::exp(-lambda + j0 * std::log(lambda) - std::lgamma((double)j0 + 1.0)), sum = 0.0;
    for (int j = j0; j < j0 + 4096; ++j) {
        sum += term;
        term *= lambda / (double)(j + 1);
        if (term < 1e-18 * sum && (double)j > lambda) break;
    }
    return sum < 1.0 ? sum : 1.0;
}

// Per-segment start of the explorer's radix descent.  The m-th smallest Philox word of the
// avail = n_s - k_s parameters outside the core lies, with overwhelming probability, between
// the words that m - 6 sqrt(m) - 32 and m + 6 sqrt(m) + 32 of them are expected to stay below:
// words up to the first are taken without ranking (sure zone), only the words between the two
// become candidates.  The exact rerun with every word a candidate catches a miss on either
// side.  Returns an error code for impossible requests; *narrow is set when every segment
// got a narrow candidate zone; *short_list when the zones are so narrow that the candidates
// of n_workers draws fit the unordered list of the short-list path with room to spare and no
// sub-tile is likely to see more of them than its pair slot holds (small segments have
// relatively wide zones: twelve standard deviations of a small m are a large share of it).
int explorer_init(slimdp_ctx* ctx, const char* who, const uint64_t* k_seg, const uint64_t* m_seg, uint32_t n_workers,
                  std::vector<SegInit>& init, uint64_t* M_out, bool* narrow, bool* short_list)
{
    uint64_t M = 0;
    bool all_narrow = true, all_short = true;
    double expect = 0.0;           // candidates of one draw
    double overflows = 0.0;        // expected number of sub-tiles of the request with more candidates than a pair slot holds
    init.resize(ctx->n_seg);
    for (uint32_t s = 0; s < ctx->n_seg; ++s) {
        const uint64_t ns = ctx->seg_off[s + 1] - ctx->seg_off[s];
        if (k_seg[s] > ns || m_seg[s] > ns - k_seg[s])
            return fail(ctx, SLIMDP_ERR_OUT_OF_RANGE, "%s: segment %u: m=%llu exceeds the %llu parameters outside the core",
                        who, s, (unsigned long long)m_seg[s], (unsigned long long)(k_seg[s] > ns ? 0 : ns - k_seg[s]));
        const uint64_t m = m_seg[s];
        M += m;
        SegInit in{(uint32_t)m, 0u, 0u, 0u, 0u};
        if (m > 0) {
            const double avail = (double)(ns - k_seg[s]);
            const double slack = 6.0 * std::sqrt((double)m) + 32.0;
            double hi = ((double)m + slack) / avail, lo = ((double)m - slack) / avail;
            if (ctx->opt_force_fallback == 1) { hi = 0.25 * (double)m / avail; lo = 0.5 * hi; }     // too few candidates
            if (ctx->opt_force_fallback == 2) { hi = 2.0 * (double)m / avail; lo = 0.75 * hi; }     // sure zone too large
            uint64_t width = 1ull << 32;                     // number of distinct candidate words
            if (hi >= 0.25) all_short = false;
            expect += (hi - (lo > 0.0 ? lo : 0.0)) * avail;
            overflows += pair_overflow_prob((hi - (lo > 0.0 ? lo : 0.0)) * (double)SUB) * ((double)ns / SUB + 2.0) * n_workers;
            if (hi >= 0.95) {
                in.bound_m1 = 0xFFFFFFFFu;
                all_narrow = false;
            } else {
                uint64_t B1 = (uint64_t)std::ceil(hi * 4294967296.0);
                if (B1 < 1) B1 = 1;
                if (B1 > (1ull << 32)) B1 = 1ull << 32;
                in.bound_m1 = (uint32_t)(B1 - 1);
                width = B1;
                const uint64_t B0 = lo > 0.0 ? (uint64_t)std::floor(lo * 4294967296.0) : 0;
                if (B0 >= 1 && B0 < B1) {                    // words 0 .. B0-1 are sure, B0 .. B1-1 candidates
                    in.sure_m1 = (uint32_t)(B0 - 1);
                    in.has_gt = 1;
                    width = B1 - B0;
                }
            }
            uint32_t bitlen = 0;
            while (bitlen < 33 && ((width - 1) >> bitlen) != 0) ++bitlen;
            in.shift0 = bitlen > 12 ? bitlen - 12 : 0;
        }
        init[s] = in;
    }
    *M_out = M;
    *narrow = all_narrow;
    // an overflowing slot costs the exact rerun (about a thousand times the per-tile tail): taken only if that is unlikely
    *short_list = all_narrow && all_short && !ctx->opt_per_tile_tail && (uint64_t)ctx->T * TILE <= 0xFFFFFFFFull &&
                  1.25 * expect * (double)n_workers + 4096.0 <= (double)ctx->list_cap && overflows <= 1e-5;
    return SLIMDP_OK;
}

}  // namespace

extern "C" {

uint64_t slimdp_num_tiles(uint64_t n, uint32_t n_seg, const uint64_t* seg_off)
{
    if (!valid_shape(n, n_seg, seg_off)) return 0;
    return count_tiles(n, n_seg, seg_off);
}

uint64_t slimdp_workspace_bytes(uint64_t n, uint32_t max_workers, uint32_t n_seg, const uint64_t* seg_off)
{
    if (!valid_shape(n, n_seg, seg_off) || max_workers == 0 || max_workers > SLIMDP_MAX_WORKERS) return 0;
    slimdp_ctx tmp;
    tmp.n = n; tmp.maxW = max_workers; tmp.n_seg = n_seg;
    tmp.T = (uint32_t)count_tiles(n, n_seg, seg_off);
    tmp.keys_stride = align_up(n, TILE) + TILE;
    tmp.pair_stride = (uint64_t)tmp.T * SUBS * PAIR_SLOT;
    tmp.n_chunks = (tmp.T + SCAN_CHUNK - 1) / SCAN_CHUNK;
    tmp.list_cap = (uint64_t)tmp.maxW * (64ull * tmp.T + 8192ull);
    if (tmp.list_cap > 0x40000000ull) tmp.list_cap = 0x40000000ull;
    Carver cv(nullptr);
    carve(&tmp, cv);
    return align_up(cv.pos, 256);
}

uint64_t slimdp_capture_bytes(uint64_t n, uint32_t max_workers, uint32_t n_seg, const uint64_t* seg_off)
{
    if (!valid_shape(n, n_seg, seg_off) || max_workers == 0 || max_workers > SLIMDP_MAX_WORKERS) return 0;
    const uint64_t T = count_tiles(n, n_seg, seg_off);
    Carver cv(nullptr);
    cv.take<uint32_t>(n_seg); cv.take<uint32_t>(n_seg); cv.take<uint32_t>(n_seg);
    cv.take<uint2>((size_t)T * TILE_WORDS);
    cv.take<float>((size_t)max_workers * T * SUBS * SPEC_CAP);
    cv.take<uint32_t>((size_t)T * SAMPLE_PER);
    return align_up(cv.pos, 256);
}

const char* slimdp_last_error(const slimdp_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

int slimdp_create(slimdp_ctx** out, uint64_t n, uint32_t max_workers, uint32_t n_seg, const uint64_t* seg_off,
                  uint64_t seed, void* hip_stream)
{
    if (!out) return fail(nullptr, SLIMDP_ERR_INVALID_ARG, "slimdp_create: out is NULL");
    *out = nullptr;
    if (n == 0 || n > SLIMDP_MAX_N) return fail(nullptr, SLIMDP_ERR_INVALID_ARG, "slimdp_create: n must be in [1, 2^31]");
    if (max_workers == 0 || max_workers > SLIMDP_MAX_WORKERS)
        return fail(nullptr, SLIMDP_ERR_INVALID_ARG, "slimdp_create: max_workers must be in [1, %u]", SLIMDP_MAX_WORKERS);
    if (!valid_shape(n, n_seg, seg_off))
        return fail(nullptr, SLIMDP_ERR_INVALID_ARG,
                    "slimdp_create: seg_off must be %u+1 strictly increasing offsets from 0 to n", n_seg);
    slimdp_ctx* c = new (std::nothrow) slimdp_ctx;
    if (!c) return fail(nullptr, SLIMDP_ERR_WORKSPACE, "slimdp_create: out of host memory");
    c->n = n; c->maxW = max_workers; c->n_seg = n_seg; c->seed = seed;
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->seg_off.assign(seg_off, seg_off + n_seg + 1);
    c->tl = make_tiling(n, n_seg, seg_off);
    c->T = (uint32_t)c->tl.tile_seg.size();
    c->keys_stride = align_up(n, TILE) + TILE;
    c->pair_stride = (uint64_t)c->T * SUBS * PAIR_SLOT;
    c->n_chunks = (c->T + SCAN_CHUNK - 1) / SCAN_CHUNK;
    c->list_cap = (uint64_t)c->maxW * (64ull * c->T + 8192ull);
    if (c->list_cap > 0x40000000ull) c->list_cap = 0x40000000ull;
    hipError_t e = hipGetDevice(&c->device);
    if (e != hipSuccess) { int rc = hip_fail(nullptr, e, "hipGetDevice (no usable GPU?)"); delete c; return rc; }
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, c->device);
    if (e != hipSuccess) { int rc = hip_fail(nullptr, e, "hipGetDeviceProperties"); delete c; return rc; }
    c->cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    Carver sizing(nullptr);
    carve(c, sizing);
    c->ws_bytes = align_up(sizing.pos, 256);
    e = hipMalloc(reinterpret_cast<void**>(&c->ws), c->ws_bytes);
    if (e != hipSuccess) {
        int rc = fail(nullptr, SLIMDP_ERR_WORKSPACE, "slimdp_create: hipMalloc(%zu bytes): %s", c->ws_bytes, hipGetErrorString(e));
        delete c;
        return rc;
    }
    Carver cv(c->ws);
    carve(c, cv);
    // tables are uploaded once; the copies are synchronous with respect to the host
    e = hipMemcpy(c->d_tile_start, c->tl.tile_start.data(), (c->T + 1) * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->d_tile_seg, c->tl.tile_seg.data(), c->T * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(c->d_seg_first_tile, c->tl.seg_first_tile.data(), (n_seg + 1) * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemset(c->d_flags, 0, 64 * 4);
    if (e == hipSuccess) e = hipMemset(c->c_pred, 0xFF, (size_t)n_seg * 4);      // no prediction yet
    if (e == hipSuccess) e = hipMemset(c->c_skip, 0, (size_t)n_seg * 4);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking);      // default priority
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_consumed, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_drawn, hipEventDisableTiming);
    for (int j = 0; j < slimdp_ctx::N_PENDING && e == hipSuccess; ++j)
        e = hipEventCreateWithFlags(&c->pend[j].ev, hipEventDisableTiming);
    if (e != hipSuccess) {
        int rc = hip_fail(nullptr, e, "slimdp_create: table upload, side stream");
        if (c->ev_consumed) (void)hipEventDestroy(c->ev_consumed);
        if (c->ev_drawn) (void)hipEventDestroy(c->ev_drawn);
        for (int j = 0; j < slimdp_ctx::N_PENDING; ++j)
            if (c->pend[j].ev) (void)hipEventDestroy(c->pend[j].ev);
        if (c->side) (void)hipStreamDestroy(c->side);
        (void)hipFree(c->ws);
        delete c;
        return rc;
    }
    *out = c;
    return SLIMDP_OK;
}

int slimdp_destroy(slimdp_ctx* ctx)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    (void)hipStreamSynchronize(ctx->side);
    (void)hipStreamSynchronize(ctx->stream);
    (void)hipEventDestroy(ctx->ev_consumed);
    (void)hipEventDestroy(ctx->ev_drawn);
    for (int j = 0; j < slimdp_ctx::N_PENDING; ++j) (void)hipEventDestroy(ctx->pend[j].ev);
    (void)hipStreamDestroy(ctx->side);
    hipError_t e = hipFree(ctx->ws);
    if (ctx->spec.mem) (void)hipFree(ctx->spec.mem);
    if (ctx->e_cand_keys) (void)hipFree(ctx->e_cand_keys);
    delete ctx;
    return e == hipSuccess ? SLIMDP_OK : SLIMDP_ERR_HIP;
}

int slimdp_tile_starts(const slimdp_ctx* ctx, uint32_t* tile_start)
{
    if (!ctx || !tile_start) return SLIMDP_ERR_INVALID_ARG;
    memcpy(tile_start, ctx->tl.tile_start.data(), (ctx->T + 1) * sizeof(uint32_t));
    return SLIMDP_OK;
}

int slimdp_set_option(slimdp_ctx* ctx, const char* name, int64_t value)
{
    if (!ctx || !name) return SLIMDP_ERR_INVALID_ARG;
    if (strcmp(name, "explore_force_fallback") == 0) { ctx->opt_force_fallback = value; return SLIMDP_OK; }
    if (strcmp(name, "explore_per_tile_tail") == 0) { ctx->opt_per_tile_tail = value; return SLIMDP_OK; }
    if (strcmp(name, "strided_tiles") == 0 && (value == 0 || value == 1)) { ctx->opt_strided = value; return SLIMDP_OK; }
    if (strcmp(name, "side_blocks") == 0 && value >= 1 && value <= 8) { ctx->opt_side_blocks = value; return SLIMDP_OK; }
    if (strcmp(name, "explore_async") == 0 && (value == 0 || value == 1)) { ctx->opt_explore_async = value; return SLIMDP_OK; }
    if (strcmp(name, "explore_hint_mode") == 0 && (value == 0 || value == 1)) { ctx->opt_hint_mode = value; return SLIMDP_OK; }
    if (strcmp(name, "core_predict") == 0 && value >= 0 && value <= 2) { ctx->opt_core_predict = value; return SLIMDP_OK; }
    if (strcmp(name, "pack_core_blocks") == 0 && value >= 0 && value <= 64) { ctx->opt_pack_core_blocks = value; return SLIMDP_OK; }
    if (strcmp(name, "build_blocks") == 0 && value >= 1 && value <= 64) { ctx->opt_build_blocks = value; return SLIMDP_OK; }
    if (strcmp(name, "pack_nbuf") == 0 && (value == 1 || value == 2)) { ctx->opt_pack_nbuf = value; return SLIMDP_OK; }
    if (strcmp(name, "pack_kernel") == 0 && (value == 0 || value == 1)) { ctx->opt_pack_kernel = value; return SLIMDP_OK; }
    if (strcmp(name, "pull_kernel") == 0 && (value == 0 || value == 1)) { ctx->opt_pull_kernel = value; return SLIMDP_OK; }
    if (strcmp(name, "expected_core") == 0 && value >= -1 && (value < 0 || (uint64_t)value <= ctx->n)) { ctx->opt_expected_core = value; return SLIMDP_OK; }
    if (strcmp(name, "score_pipeline") == 0 && (value == 0 || value == 1)) { ctx->opt_score_pipeline = value; return SLIMDP_OK; }
    if (strcmp(name, "capture_estimate_bias") == 0) { ctx->opt_estimate_bias = value; return SLIMDP_OK; }
    if (strcmp(name, "speculative_pack") == 0) {
        ctx->spec.captured = false;
        if (value && !ctx->spec.mem) {
            const size_t S = ctx->n_seg;
            Carver sizing(nullptr);
            auto carve_spec = [&](Carver& cv) {
                ctx->spec.lo[0] = cv.take<uint32_t>(S);
                ctx->spec.lo[1] = cv.take<uint32_t>(S);
                ctx->spec.fail = cv.take<uint32_t>(S);
                ctx->spec.bits = cv.take<uint2>((size_t)ctx->T * TILE_WORDS);
                ctx->spec.vals = cv.take<float>((size_t)ctx->maxW * ctx->T * SUBS * SPEC_CAP);
                ctx->spec.sample = cv.take<uint32_t>((size_t)ctx->T * SAMPLE_PER);
            };
            carve_spec(sizing);
            hipError_t e = hipMalloc(reinterpret_cast<void**>(&ctx->spec.mem), align_up(sizing.pos, 256));
            if (e != hipSuccess) {
                ctx->spec.mem = nullptr;
                return fail(ctx, SLIMDP_ERR_WORKSPACE, "slimdp_set_option(speculative_pack): hipMalloc(%zu bytes): %s",
                            align_up(sizing.pos, 256), hipGetErrorString(e));
            }
            Carver cv(ctx->spec.mem);
            carve_spec(cv);
            // nothing captured, nothing trusted until a selection has set a bound
            int rc = fill(ctx, ctx->spec.lo[0], S, NONE);
            if (!rc) rc = fill(ctx, ctx->spec.lo[1], S, NONE);
            if (!rc) rc = fill(ctx, ctx->spec.fail, S, 1u);
            if (rc) return rc;
            ctx->spec.cur = 0;
            ctx->spec.next_written = false;
            ctx->spec.bound_valid = false;
        }
        ctx->spec.on = value != 0;
        return SLIMDP_OK;
    }
    return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_set_option: unknown option '%s'", name);
}

int slimdp_synchronize(slimdp_ctx* ctx)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    SLIMDP_HIP(ctx, hipStreamSynchronize(ctx->stream));
    SLIMDP_HIP(ctx, hipStreamSynchronize(ctx->side));
    for (int j = 0; j < slimdp_ctx::N_PENDING; ++j) ctx->pend[j].live = false;
    ctx->side_pending = false;
    uint32_t flags[2] = {0, 0};
    SLIMDP_HIP(ctx, hipMemcpy(flags, ctx->d_flags, sizeof flags, hipMemcpyDeviceToHost));
    if (flags[1]) {
        SLIMDP_HIP(ctx, hipMemset(ctx->d_flags + 1, 0, 4));
        return fail(ctx, SLIMDP_ERR_DEVICE_STATUS, "device status 0x%x:%s%s", flags[1],
                    (flags[1] & 1u) ? " an emitted index list does not have the requested length;" : "",
                    (flags[1] & 2u) ? " a segment holds fewer eligible parameters than requested;" : "");
    }
    return SLIMDP_OK;
}

// ------------------------------------------------------------------------------------------
static int score_impl(slimdp_ctx* ctx, const float* w, const float* const* g, uint32_t W, float c, float* score, float* w_new,
                      float lr)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    if (!w || !score) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_score: NULL array");
    if (W == 0 || W > ctx->maxW) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_score: W=%u outside [1, %u]", W, ctx->maxW);
    if (!table_ok(g, W)) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_score: NULL update pointer");
    if (!(c >= 0.0f) || std::isinf(c)) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_score: c must be finite and >= 0");
    ctx->hist_pending = false;
    ctx->cls_by_score = false;
    int rc = fill(ctx, ctx->c_hist, (uint64_t)ctx->n_seg * H_STRIDE, 0u);
    if (rc) return rc;
    PtrTab gt = make_tab<PtrTab>(g, W);
    int vec_ok = aligned16(w) && aligned16(score);
    for (uint32_t q = 0; q < W; ++q) vec_ok = vec_ok && aligned16(g[q]);
    // an announced explorer draw rides along if every segment has a narrow candidate bound
    PreArgs pre{};
    bool presample = false, pairs = false;
    if (ctx->opt_hint_mode == 0) ctx->pre.valid = false;      // a draw made on the side stream stays valid
    if (ctx->hint.valid && ctx->opt_hint_mode == 0 && ctx->tl.quad_aligned) {
        std::vector<SegInit> init;
        uint64_t M = 0;
        bool narrow = false;
        if (explorer_init(ctx, "slimdp_score(hint)", ctx->hint.k_seg.data(), ctx->hint.m_seg.data(), ctx->hint.n_workers, init,
                          &M, &narrow, &pairs) == SLIMDP_OK && narrow && M > 0) {
            rc = wait_for_side(ctx);         // the draw's buffers may still be read by work on the side stream
            if (rc) return rc;
            rc = init_states(ctx, ctx->e_state, init, ctx->hint.n_workers, 0);
            if (rc) return rc;
            pre.nw = ctx->hint.n_workers; pre.worker0 = ctx->hint.worker0; pre.n_seg = ctx->n_seg;
            pre.states = ctx->e_state; pre.sure_bits = ctx->e_sure_bits; pre.cand_bits = ctx->e_cand_bits;
            if (!pairs) { rc = ensure_wide_keys(ctx); if (rc) return rc; }
            pre.cand_keys = pairs ? ctx->e_pair_keys : ctx->e_cand_keys; pre.cnt_cand = ctx->e_cnt_cand;
            pre.keys_stride = pairs ? ctx->pair_stride : ctx->keys_stride;
            pre.pk = PhiloxKey{(uint32_t)ctx->seed, (uint32_t)(ctx->seed >> 32), (uint32_t)ctx->hint.iteration,
                               (uint32_t)(ctx->hint.iteration >> 32)};
            presample = true;
        }
    }
    // speculative packing: keep the update values of the parameters at or above the previous threshold
    SpecArgs sa{};
    // (not after a dense update: the pack that follows it belongs to the next iteration's updates)
    const bool capture = ctx->spec.on && !w_new && (W == 1 || W == 2 || W == 4 || W == 8 || W == 16);
    ctx->spec.captured = false;
    if (capture) {
        if (ctx->spec.next_written) { ctx->spec.cur ^= 1; ctx->spec.next_written = false; ctx->spec.bound_valid = true; }
        sa.lo = ctx->spec.lo[ctx->spec.cur]; sa.bits = ctx->spec.bits; sa.vals = ctx->spec.vals;
        // No selection has set a bound yet (first iteration of a context): estimate the coming threshold from a sample of
        // the very significances this pass computes, if the size of the coming core is known (announced draw, option, or
        // the previous selection).  Flat model, whole aligned tiles.
        const uint32_t T_full = (uint32_t)(ctx->n / TILE);
        int64_t expect = ctx->opt_expected_core;
        if (expect < 0 && ctx->hint.valid && ctx->n_seg == 1) expect = (int64_t)ctx->hint.k_seg[0];
        if (expect < 0 && ctx->have_last_K) expect = (int64_t)ctx->last_K;
        if (!ctx->spec.bound_valid && ctx->n_seg == 1 && vec_ok && T_full >= 64 && expect >= 0) {
            const uint32_t N = T_full * SAMPLE_PER;
            // rank of the threshold inside the sample, rounded up
            const uint64_t need = ((uint64_t)expect * N + ctx->n - 1) / ctx->n;
            hipLaunchKernelGGL(k_sample_keys, dim3((N + 255) / 256), dim3(256), 0, ctx->stream, w, gt, (int)W, c, T_full,
                               ctx->spec.sample);
            SLIMDP_LAUNCHED(ctx, "k_sample_keys");
            hipLaunchKernelGGL(k_sample_bound, dim3(1), dim3(1024), 0, ctx->stream, ctx->spec.sample, N, (uint32_t)need,
                               (long long)ctx->opt_estimate_bias, ctx->spec.lo[ctx->spec.cur], ctx->c_pred);
            SLIMDP_LAUNCHED(ctx, "k_sample_bound");
        }
    }
    // flat model, aligned arrays, 1/2/4/8 workers: the pipelined kernel
    if (ctx->n_seg == 1 && vec_ok && ctx->opt_strided && ctx->opt_score_pipeline && ctx->n < (1ull << 30) &&
        (W == 1 || W == 2 || W == 4 || W == 8)) {
        const dim3 fgrid(persistent_blocks(ctx, SCOREF_MINB, 1)), fblock(BLOCK);
        const ClsArgs cls{ctx->c_pred, ctx->c_used, (int)ctx->opt_core_predict, ctx->c_gt_bits, ctx->c_cand_bits, ctx->c_cand_keys, ctx->c_cnt_gt, ctx->c_cnt_cand};
#define LAUNCH_FLAT_Q(WT, PRE, SPEC, DENSE)                                                                           \
    hipLaunchKernelGGL((k_score_flat<WT, PRE, SPEC, DENSE>), fgrid, fblock, 0, ctx->stream, w, gt, c, score, ctx->n,  \
                       ctx->c_hist, pre, sa, cls, w_new, lr)
#define LAUNCH_FLAT_S(WT, SPEC, DENSE)                                                                                \
    do {                                                                                                              \
        if (presample && pairs) LAUNCH_FLAT_Q(WT, 2, SPEC, DENSE);                                                    \
        else if (presample) LAUNCH_FLAT_Q(WT, 1, SPEC, DENSE);                                                        \
        else LAUNCH_FLAT_Q(WT, 0, SPEC, DENSE);                                                                       \
    } while (0)
#define LAUNCH_FLAT(WT)                                                                                               \
    do {                                                                                                              \
        if (w_new) LAUNCH_FLAT_S(WT, 0, 1);                                                                           \
        else if (capture) LAUNCH_FLAT_S(WT, 1, 0);                                                                    \
        else LAUNCH_FLAT_S(WT, 0, 0);                                                                                 \
    } while (0)
        switch (W) {
            case 1: LAUNCH_FLAT(1); break;
            case 2: LAUNCH_FLAT(2); break;
            case 4: LAUNCH_FLAT(4); break;
            default: LAUNCH_FLAT(8); break;
        }
#undef LAUNCH_FLAT
#undef LAUNCH_FLAT_S
#undef LAUNCH_FLAT_Q
        SLIMDP_LAUNCHED(ctx, "k_score_flat");
        ctx->cls_by_score = true;
        if (presample) { ctx->pre = ctx->hint; ctx->pre.pairs = pairs; }
        if (capture) {
            ctx->spec.captured = true; ctx->spec.score = score; ctx->spec.W = W; ctx->spec.vec_ok = vec_ok; ctx->spec.core_epoch = 0;
            for (uint32_t q = 0; q < W; ++q) ctx->spec.g[q] = g[q];
        }
        ctx->hint.valid = false;
        ctx->hist_pending = true;
        ctx->hist_score = score;
        return SLIMDP_OK;
    }
    const uint32_t P = persistent_blocks(ctx, SCORE_MINB, 1);
    const dim3 grid(P), block(BLOCK);
    // flat model, up to 8 workers: every P-th tile per block (measured: 8 workers 1.38 -> 1.34 ms; 16 workers slower)
    const bool strided = ctx->n_seg == 1 && ctx->opt_strided && W <= 8;
#define LAUNCH_SCORE_Q(WT, PRE, SPEC, DENSE, STRIDED)                                                                 \
    hipLaunchKernelGGL((k_score<WT, PRE, SPEC, DENSE, STRIDED>), grid, block, 0, ctx->stream, w, gt, (int)W, c, score, \
                       ctx->d_tile_start, ctx->d_tile_seg, ctx->T, ctx->c_hist, vec_ok, pre, sa, w_new, lr)
#define LAUNCH_SCORE_P(WT, PRE, SPEC, DENSE)                                                                          \
    do {                                                                                                              \
        if constexpr ((WT) >= 1 && (WT) <= 8) {                                                                       \
            if (strided) LAUNCH_SCORE_Q(WT, PRE, SPEC, DENSE, 1);                                                     \
            else LAUNCH_SCORE_Q(WT, PRE, SPEC, DENSE, 0);                                                             \
        } else LAUNCH_SCORE_Q(WT, PRE, SPEC, DENSE, 0);                                                               \
    } while (0)
#define LAUNCH_SCORE_S(WT, SPEC, DENSE)                                                                               \
    do {                                                                                                              \
        if (presample && pairs) LAUNCH_SCORE_P(WT, 2, SPEC, DENSE);                                                   \
        else if (presample) LAUNCH_SCORE_P(WT, 1, SPEC, DENSE);                                                       \
        else LAUNCH_SCORE_P(WT, 0, SPEC, DENSE);                                                                      \
    } while (0)
#define LAUNCH_SCORE(WT)                                                                                              \
    do {                                                                                                              \
        if (w_new) LAUNCH_SCORE_S(WT, 0, 1);                                                                          \
        else if (capture) LAUNCH_SCORE_S(WT, 1, 0);                                                                   \
        else LAUNCH_SCORE_S(WT, 0, 0);                                                                                \
    } while (0)
    switch (W) {
        case 1: LAUNCH_SCORE(1); break;
        case 2: LAUNCH_SCORE(2); break;
        case 4: LAUNCH_SCORE(4); break;
        case 8: LAUNCH_SCORE(8); break;
        case 16: LAUNCH_SCORE(16); break;
        default:
            if (w_new) LAUNCH_SCORE_S(0, 0, 1);
            else LAUNCH_SCORE_S(0, 0, 0);
            break;
    }
#undef LAUNCH_SCORE_P
#undef LAUNCH_SCORE_Q
#undef LAUNCH_SCORE_S
#undef LAUNCH_SCORE
    SLIMDP_LAUNCHED(ctx, "k_score");
    if (presample) { ctx->pre = ctx->hint; ctx->pre.pairs = pairs; }
    if (capture) {
        ctx->spec.captured = true; ctx->spec.score = score; ctx->spec.W = W; ctx->spec.vec_ok = vec_ok; ctx->spec.core_epoch = 0;
        for (uint32_t q = 0; q < W; ++q) ctx->spec.g[q] = g[q];
    }
    ctx->hint.valid = false;
    ctx->hist_pending = true;
    ctx->hist_score = score;
    return SLIMDP_OK;
}

int slimdp_score(slimdp_ctx* ctx, const float* w, const float* const* g, uint32_t W, float c, float* score)
{
    return score_impl(ctx, w, g, W, c, score, nullptr, 0.0f);
}

int slimdp_dense_update_score(slimdp_ctx* ctx, float* w, const float* const* g, uint32_t W, float lr, float c, float* score)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    if (!std::isfinite(lr)) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_dense_update_score: lr must be finite");
    if (w && score && static_cast<const void*>(w) == static_cast<const void*>(score))
        return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_dense_update_score: score aliases w");
    return score_impl(ctx, w, g, W, c, score, w, lr);
}

// The selection itself, for a context whose device pointers may also lie in the static scratch array.
static int select_core_impl(slimdp_ctx* ctx, const float* score, const uint64_t* k_seg, uint32_t flags, uint32_t* core_idx,
                            uint32_t* core_bits, uint32_t* core_off, uint64_t* core_epoch)
{
    if (!score || !k_seg || !core_bits || !core_off || !core_epoch)
        return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_select_core: NULL argument");
    uint64_t K = 0;
    std::vector<SegInit> init(ctx->n_seg);
    for (uint32_t s = 0; s < ctx->n_seg; ++s) {
        const uint64_t ns = ctx->seg_off[s + 1] - ctx->seg_off[s];
        if (k_seg[s] > ns)
            return fail(ctx, SLIMDP_ERR_OUT_OF_RANGE, "slimdp_select_core: k_seg[%u]=%llu exceeds the segment size %llu", s,
                        (unsigned long long)k_seg[s], (unsigned long long)ns);
        init[s] = SegInit{(uint32_t)k_seg[s], 0u, 0u, 0u, 1u};
        K += k_seg[s];
    }
    if (K > 0 && !core_idx) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_select_core: core_idx is NULL");
    const bool reuse = (flags & SLIMDP_SELECT_REUSE_HISTOGRAM) != 0;
    if (reuse && !(ctx->hist_pending && ctx->hist_score == score))
        return fail(ctx, SLIMDP_ERR_INVALID_ARG,
                    "slimdp_select_core: no histogram pending for this score buffer (call slimdp_score first)");
    ctx->hist_pending = false;
    const uint32_t T = ctx->T, S = ctx->n_seg;
    int rc = wait_for_side(ctx);             // an explorer request on the side stream may still read the bitmap this call rewrites
    if (rc) return rc;
    rc = init_states(ctx, ctx->c_state, init, 1, 1);
    if (rc) return rc;
    const uint32_t P = persistent_blocks(ctx, (uint32_t)ctx->opt_build_blocks, 1);
    if (!reuse) {
        rc = fill(ctx, ctx->c_hist, (uint64_t)S * H_STRIDE, 0u);
        if (rc) return rc;
        hipLaunchKernelGGL(k_core_hist0, dim3(P), dim3(BLOCK), 0, ctx->stream, score, ctx->d_tile_start, ctx->d_tile_seg, T,
                           ctx->c_hist);
        SLIMDP_LAUNCHED(ctx, "k_core_hist0");
    }
    // did the scoring pass that made this histogram already sort the whole tiles against a predicted bin?
    const bool classified = reuse && ctx->cls_by_score;
    ctx->cls_by_score = false;
    const CorePred cp{ctx->c_pred, ctx->c_skip, ctx->c_used, classified ? 1 : 0};
    hipLaunchKernelGGL(k_threshold, dim3(S, 1), dim3(256), 0, ctx->stream, ctx->c_state, ctx->c_hist, 0, (uint32_t)H_L0, S, 0,
                       ctx->d_flags, nullptr, 0, SpecTau{nullptr, nullptr, nullptr}, cp);
    SLIMDP_LAUNCHED(ctx, "k_threshold(0)");
    hipLaunchKernelGGL(k_core_build, dim3(P), dim3(BLOCK), 0, ctx->stream, score, ctx->d_tile_start, ctx->d_tile_seg, T,
                       ctx->c_state, ctx->c_skip, ctx->c_hist, ctx->c_gt_bits, ctx->c_cand_bits, ctx->c_cand_keys, ctx->c_cnt_gt,
                       ctx->c_cnt_cand, (int)aligned16(score), (int)(S == 1 && ctx->opt_strided));
    SLIMDP_LAUNCHED(ctx, "k_core_build");
    MutPtrTab off_tab = make_tab<MutPtrTab, uint32_t*>(&core_off, 1);
    MutPtrTab idx_tab = make_tab<MutPtrTab, uint32_t*>(&core_idx, 1);
    // speculative packing: this selection rates the capture of the scoring pass it reuses and sets the next bound
    const bool spec_sel = ctx->spec.on && ctx->spec.mem && ctx->spec.captured && reuse && ctx->spec.score == score;
    SpecTau sp{nullptr, nullptr, nullptr};
    if (spec_sel) sp = SpecTau{ctx->spec.lo[ctx->spec.cur], ctx->spec.lo[ctx->spec.cur ^ 1], ctx->spec.fail};
    uint32_t* pub = ctx->tl.word_aligned ? core_bits : nullptr;
    rc = finish_selection<CORE_KPL, 1>(ctx, 1, ctx->c_state, ctx->c_hist, ctx->c_gt_bits, ctx->c_cand_bits, ctx->c_cand_keys,
                          ctx->c_cnt_gt, ctx->c_cnt_cand, ctx->c_cnt_sel, ctx->c_cnt_tie, ctx->c_tie_pre, ctx->keys_stride,
                          true, off_tab, idx_tab, (uint32_t)K, pub, nullptr, nullptr, ctx->c_chunk_sum, sp,
                          CorePred{ctx->c_pred, nullptr, nullptr, 0});
    if (rc) return rc;
    if (!pub) {
        rc = fill(ctx, core_bits, (ctx->n + 31) / 32, 0u);
        if (rc) return rc;
        if (K) {
            hipLaunchKernelGGL(k_bits_from_idx, dim3(fill_grid(K)), dim3(256), 0, ctx->stream, core_idx, K, ctx->n, core_bits);
            SLIMDP_LAUNCHED(ctx, "k_bits_from_idx");
        }
    }
    *core_epoch = ++ctx->epoch;
    ctx->last_K = K; ctx->have_last_K = true;
    if (spec_sel) { ctx->spec.core_epoch = ctx->epoch; ctx->spec.next_written = true; }
    else ctx->spec.core_epoch = 0;
    return SLIMDP_OK;
}

int slimdp_select_core(slimdp_ctx* ctx, const float* score, const uint64_t* k_seg, uint32_t flags, uint32_t* core_idx,
                       uint32_t* core_bits, uint32_t* core_off, uint64_t* core_epoch)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    return select_core_impl(ctx, score, k_seg, flags, core_idx, core_bits, core_off, core_epoch);
}

// ------------------------------------------------------------------------------------------
// Core selection for callers that cannot allocate: no context, no hipMalloc.  The workspace is
// a file-scope array in device memory (one copy per GPU, held until the process ends); the
// host uses its per-device address obtained from the runtime, never the symbol itself.
// ------------------------------------------------------------------------------------------
#define SLIMDP_STATIC_SCRATCH_BYTES (5u << 20)
static __device__ __align__(256) unsigned char scratch[SLIMDP_STATIC_SCRATCH_BYTES];

namespace {
struct StaticDev { void* ptr = nullptr; int cus = 0; };
constexpr int STATIC_MAX_DEVICES = 64;
StaticDev g_static[STATIC_MAX_DEVICES];
std::mutex g_static_mu;
}  // namespace

int slimdp_select_core_static(const float* score, uint64_t n, uint64_t k, uint32_t* core_idx, uint32_t* core_bits,
                              uint32_t* core_off, void* hip_stream)
{
    if (!score || !core_bits || !core_off || (k && !core_idx))
        return fail(nullptr, SLIMDP_ERR_INVALID_ARG, "slimdp_select_core_static: NULL argument");
    if (n == 0 || n > SLIMDP_STATIC_MAX_N)
        return fail(nullptr, SLIMDP_ERR_OUT_OF_RANGE, "slimdp_select_core_static: n=%llu outside [1, %u] (the static workspace "
                    "serves at most SLIMDP_STATIC_MAX_N parameters; larger models need a context)",
                    (unsigned long long)n, (unsigned)SLIMDP_STATIC_MAX_N);
    if (k > n) return fail(nullptr, SLIMDP_ERR_OUT_OF_RANGE, "slimdp_select_core_static: k exceeds n");
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return hip_fail(nullptr, e, "hipGetDevice");
    if (device < 0 || device >= STATIC_MAX_DEVICES)
        return fail(nullptr, SLIMDP_ERR_INVALID_ARG, "slimdp_select_core_static: device %d not supported", device);
    StaticDev sdv;
    {
        std::lock_guard<std::mutex> lock(g_static_mu);
        if (!g_static[device].ptr) {          // once per device, with that device current: this GPU's copy of the array
            void* p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !p) return hip_fail(nullptr, e, "hipGetSymbolAddress(scratch)");
            int cus = 0;
            e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device);
            if (e != hipSuccess) return hip_fail(nullptr, e, "hipDeviceGetAttribute");
            g_static[device].cus = cus > 0 ? cus : 256;
            g_static[device].ptr = p;
        }
        sdv = g_static[device];
    }
    // a context on the stack whose device pointers lie inside this GPU's array (host members only, nothing allocated on the device)
    slimdp_ctx tmp;
    const uint64_t so[2] = {0, n};
    tmp.n = n; tmp.maxW = 1; tmp.n_seg = 1; tmp.seed = 0;
    tmp.stream = static_cast<hipStream_t>(hip_stream);
    tmp.device = device; tmp.cus = sdv.cus;
    tmp.seg_off.assign(so, so + 2);
    tmp.T = (uint32_t)count_tiles(n, 1, so);
    tmp.keys_stride = align_up(n, TILE) + TILE;
    tmp.n_chunks = (tmp.T + SCAN_CHUNK - 1) / SCAN_CHUNK;
    Carver cv(static_cast<char*>(sdv.ptr));
    carve_core(&tmp, cv);
    if (cv.pos > SLIMDP_STATIC_SCRATCH_BYTES)
        return fail(nullptr, SLIMDP_ERR_WORKSPACE, "slimdp_select_core_static: %zu bytes of workspace needed, %u available",
                    cv.pos, (unsigned)SLIMDP_STATIC_SCRATCH_BYTES);
    // the array keeps the previous call's contents: tables for this n, flags cleared (the histogram is cleared by the selection)
    hipLaunchKernelGGL(k_flat_tables, dim3((tmp.T + 1 + 255) / 256), dim3(256), 0, tmp.stream, tmp.d_tile_start, tmp.d_tile_seg,
                       tmp.d_seg_first_tile, tmp.d_flags, tmp.T, (uint32_t)n);
    e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(nullptr, e, "k_flat_tables");
    uint64_t epoch = 0;
    const int rc = select_core_impl(&tmp, score, &k, 0u, core_idx, core_bits, core_off, &epoch);
    if (rc) g_create_error = tmp.err;
    return rc;
}

int slimdp_import_core(slimdp_ctx* ctx, const uint32_t* core_idx, const uint64_t* k_seg, uint32_t* core_bits,
                       uint32_t* core_off, uint64_t* core_epoch)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    if (!k_seg || !core_bits || !core_off || !core_epoch) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_import_core: NULL argument");
    uint64_t K = 0;
    for (uint32_t s = 0; s < ctx->n_seg; ++s) {
        if (k_seg[s] > ctx->seg_off[s + 1] - ctx->seg_off[s])
            return fail(ctx, SLIMDP_ERR_OUT_OF_RANGE, "slimdp_import_core: k_seg[%u] exceeds the segment size", s);
        K += k_seg[s];
    }
    if (K && !core_idx) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_import_core: core_idx is NULL");
    int rc = wait_for_side(ctx);
    if (rc) return rc;
    rc = fill(ctx, core_bits, (ctx->n + 31) / 32, 0u);
    if (rc) return rc;
    if (K) {
        hipLaunchKernelGGL(k_bits_from_idx, dim3(fill_grid(K)), dim3(256), 0, ctx->stream, core_idx, K, ctx->n, core_bits);
        SLIMDP_LAUNCHED(ctx, "k_bits_from_idx");
    }
    hipLaunchKernelGGL(k_tile_offsets, dim3((ctx->T + 1 + 255) / 256), dim3(256), 0, ctx->stream, core_idx, K, ctx->d_tile_start,
                       ctx->T, ctx->n, core_off);
    SLIMDP_LAUNCHED(ctx, "k_tile_offsets");
    ctx->hist_pending = false;
    ctx->spec.core_epoch = 0;
    *core_epoch = ++ctx->epoch;
    ctx->last_K = K; ctx->have_last_K = true;
    return SLIMDP_OK;
}

int slimdp_sample_explore(slimdp_ctx* ctx, const uint32_t* core_bits, const uint64_t* k_seg, uint32_t worker0,
                          uint32_t n_workers, uint64_t iteration, const uint64_t* m_seg, uint32_t* const* expl_idx,
                          uint32_t* const* expl_off)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    if (!core_bits || !k_seg || !m_seg) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_sample_explore: NULL argument");
    if (n_workers == 0 || n_workers > ctx->maxW)
        return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_sample_explore: n_workers=%u outside [1, %u]", n_workers, ctx->maxW);
    if (!table_ok(expl_off, n_workers)) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_sample_explore: NULL expl_off entry");
    uint64_t M = 0;
    std::vector<SegInit> init;
    bool narrow = false, short_list = false;
    int rc = explorer_init(ctx, "slimdp_sample_explore", k_seg, m_seg, n_workers, init, &M, &narrow, &short_list);
    if (rc) return rc;
    if (M > 0 && !table_ok(expl_idx, n_workers)) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_sample_explore: NULL expl_idx entry");
    const uint32_t T = ctx->T, S = ctx->n_seg, B = n_workers;
    // zones already drawn inside slimdp_score for exactly this request, in the format this call wants?
    const bool cached = ctx->pre.same(iteration, worker0, n_workers, k_seg, m_seg, S) && ctx->pre.pairs == short_list;
    ctx->pre.valid = false;
    ctx->hint.valid = false;
    // Option "explore_async": the whole request runs on the library's side stream, beside whatever the caller enqueues
    // on the context's stream after this call; the calls that take the lists make the context's stream wait for them.
    const bool async = ctx->opt_explore_async != 0;
    hipStream_t st = async ? ctx->side : ctx->stream;
    if (async) {
        // everything enqueued so far comes first: the selection that wrote core_bits, readers of the output arrays
        SLIMDP_HIP(ctx, hipEventRecord(ctx->ev_consumed, ctx->stream));
        SLIMDP_HIP(ctx, hipStreamWaitEvent(ctx->side, ctx->ev_consumed, 0));
        ctx->side_pending = false;       // a draw on the side stream precedes this request in stream order
    } else {
        rc = wait_for_side(ctx);         // an announced draw, or an earlier asynchronous request: their buffers are theirs until done
        if (rc) return rc;
    }
    rc = init_states(ctx, ctx->e_state, init, B, 0, st);
    if (rc) return rc;
    {   // histograms, rerun flag, list counters
        FillJobs fj{};
        fj.p[0] = ctx->e_hist; fj.count[0] = (uint64_t)B * S * H_STRIDE;
        fj.p[1] = ctx->d_flags; fj.count[1] = 1;
        fj.p[2] = ctx->e_list_count; fj.count[2] = 2;
        hipLaunchKernelGGL(k_fill_multi, dim3(fill_grid(fj.count[0])), dim3(256), 0, st, fj);
        SLIMDP_LAUNCHED(ctx, "k_fill_multi");
    }
    const uint32_t P = persistent_blocks(ctx, 8, B);
    const uint32_t n_words = (uint32_t)((ctx->n + 31) / 32);
    const PhiloxKey pk{(uint32_t)ctx->seed, (uint32_t)(ctx->seed >> 32), (uint32_t)iteration, (uint32_t)(iteration >> 32)};
    MutPtrTab off_tab = make_tab<MutPtrTab>(expl_off, B);
    MutPtrTab idx_tab = make_tab<MutPtrTab>(expl_idx, B);
#define LAUNCH_DRAW(PAIRS)                                                                                               \
    do {                                                                                                                 \
        if (ctx->tl.quad_aligned)                                                                                        \
            hipLaunchKernelGGL((k_explore_keys<1, PAIRS>), dim3(P, B), dim3(BLOCK), 0, st, ctx->d_tile_start,   \
                               ctx->d_tile_seg, T, S, ctx->e_state, ctx->e_sure_bits, ctx->e_cand_bits,                  \
                               (PAIRS) ? ctx->e_pair_keys : ctx->e_cand_keys, ctx->e_cnt_cand,                           \
                               (PAIRS) ? ctx->pair_stride : ctx->keys_stride, worker0, pk);                              \
        else                                                                                                             \
            hipLaunchKernelGGL((k_explore_keys<0, PAIRS>), dim3(P, B), dim3(BLOCK), 0, st, ctx->d_tile_start,   \
                               ctx->d_tile_seg, T, S, ctx->e_state, ctx->e_sure_bits, ctx->e_cand_bits,                  \
                               (PAIRS) ? ctx->e_pair_keys : ctx->e_cand_keys, ctx->e_cnt_cand,                           \
                               (PAIRS) ? ctx->pair_stride : ctx->keys_stride, worker0, pk);                              \
        SLIMDP_LAUNCHED(ctx, "k_explore_keys");                                                                          \
    } while (0)
    if (short_list) {
        // the few candidates go through one unordered list; any irregularity raises the flag that
        // switches these kernels off and the exact rerun below on
        constexpr int SBPW = 8;
        if (!cached) LAUNCH_DRAW(1);
        hipLaunchKernelGGL(k_sure_count<SBPW>, dim3((T + 3) / 4, (B + SBPW - 1) / SBPW), dim3(BLOCK), 0, st, core_bits,
                           n_words, ctx->n, ctx->d_tile_start, ctx->d_tile_seg, T, S, B, ctx->e_sure_bits, ctx->e_cnt_sel);
        SLIMDP_LAUNCHED(ctx, "k_sure_count");
        hipLaunchKernelGGL(k_seg_sum, dim3(S, B), dim3(1024), 0, st, ctx->e_cnt_sel, 1u, ctx->d_seg_first_tile, T, S,
                           ctx->e_nsure);
        SLIMDP_LAUNCHED(ctx, "k_seg_sum");
        hipLaunchKernelGGL(k_cand_gather, dim3((uint32_t)(((uint64_t)B * T + 1023) / 1024)), dim3(1024), 0, st,
                           core_bits, ctx->n, ctx->d_tile_start, ctx->d_tile_seg, T, S, B, ctx->e_pair_keys, ctx->pair_stride,
                           ctx->e_cnt_cand, ctx->e_list, ctx->e_list_count, (uint32_t)ctx->list_cap, ctx->d_flags);
        SLIMDP_LAUNCHED(ctx, "k_cand_gather");
        const uint32_t hoff[3] = {H_L0, H_L1, H_L2};
        for (int level = 0; level < 3; ++level) {
            hipLaunchKernelGGL(k_short_hist, dim3(512), dim3(256), 0, st, ctx->e_list, ctx->e_list_count,
                               (uint32_t)ctx->list_cap, ctx->e_state, ctx->e_hist, hoff[level], level, ctx->d_flags);
            SLIMDP_LAUNCHED(ctx, "k_short_hist");
            hipLaunchKernelGGL(k_threshold, dim3(S, B), dim3(256), 0, st, ctx->e_state, ctx->e_hist, level, hoff[level],
                               S, level == 0 ? 1 : 0, ctx->d_flags, ctx->e_nsure, 1, SpecTau{nullptr, nullptr, nullptr}, CorePred{nullptr, nullptr, nullptr, 0});
            SLIMDP_LAUNCHED(ctx, "k_threshold");
        }
        hipLaunchKernelGGL(k_short_mark, dim3(512), dim3(256), 0, st, ctx->e_list, ctx->e_list_count,
                           (uint32_t)ctx->list_cap, ctx->e_state, T, ctx->e_sure_bits, ctx->e_cnt_sel, ctx->e_tie_list,
                           ctx->e_list_count + 1, ctx->d_flags);
        SLIMDP_LAUNCHED(ctx, "k_short_mark");
        hipLaunchKernelGGL(k_short_ties, dim3(1), dim3(1024), 0, st, ctx->e_list, ctx->e_state, T, ctx->e_sure_bits,
                           ctx->e_cnt_sel, ctx->e_tie_list, ctx->e_list_count + 1, ctx->d_flags);
        SLIMDP_LAUNCHED(ctx, "k_short_ties");
        hipLaunchKernelGGL(k_chunk_scan, dim3(ctx->n_chunks, B), dim3(1024), 0, st, T, ctx->e_cnt_sel, off_tab,
                           ctx->e_chunk_sum, ctx->d_flags);
        SLIMDP_LAUNCHED(ctx, "k_chunk_scan");
        constexpr int EBPW = 4;
        hipLaunchKernelGGL(k_emit_bits<EBPW>, dim3((T + 3) / 4, (B + EBPW - 1) / EBPW), dim3(BLOCK), 0, st, core_bits,
                           n_words, ctx->n, ctx->d_tile_start, ctx->d_tile_seg, T, S, B, ctx->e_sure_bits, ctx->e_chunk_sum,
                           ctx->n_chunks, off_tab, idx_tab, (uint32_t)M, ctx->d_flags);
        SLIMDP_LAUNCHED(ctx, "k_emit_bits");
    } else {
        // zones that are not narrow: the per-tile tail that the core selection uses
        rc = ensure_wide_keys(ctx);
        if (rc) return rc;
        if (!cached) LAUNCH_DRAW(0);
        hipLaunchKernelGGL(k_explore_filter, dim3(P, B), dim3(BLOCK), 0, st, core_bits, ctx->n, ctx->d_tile_start,
                           ctx->d_tile_seg, T, S, ctx->e_state, ctx->e_hist, ctx->e_sure_bits, ctx->e_cnt_gt, ctx->e_cand_bits,
                           ctx->e_cand_keys, ctx->e_cnt_cand, ctx->keys_stride, n_words);
        SLIMDP_LAUNCHED(ctx, "k_explore_filter");
        hipLaunchKernelGGL(k_seg_sum, dim3(S, B), dim3(1024), 0, st, ctx->e_cnt_gt, (uint32_t)SUBS, ctx->d_seg_first_tile,
                           T, S, ctx->e_nsure);
        SLIMDP_LAUNCHED(ctx, "k_seg_sum");
        hipLaunchKernelGGL(k_threshold, dim3(S, B), dim3(256), 0, st, ctx->e_state, ctx->e_hist, 0, (uint32_t)H_L0, S, 1,
                           ctx->d_flags, ctx->e_nsure, 0, SpecTau{nullptr, nullptr, nullptr}, CorePred{nullptr, nullptr, nullptr, 0});
        SLIMDP_LAUNCHED(ctx, "k_threshold(0)");
        rc = finish_selection<EXPL_KPL, 4>(ctx, B, ctx->e_state, ctx->e_hist, ctx->e_sure_bits, ctx->e_cand_bits,
                              ctx->e_cand_keys, ctx->e_cnt_gt, ctx->e_cnt_cand, ctx->e_cnt_sel, ctx->e_cnt_tie, ctx->e_tie_pre,
                              ctx->keys_stride, false, off_tab, idx_tab, (uint32_t)M, nullptr, core_bits, ctx->d_flags,
                              ctx->e_chunk_sum, SpecTau{nullptr, nullptr, nullptr}, CorePred{nullptr, nullptr, nullptr, 0}, st);
        if (rc) return rc;
    }
#undef LAUNCH_DRAW
    // zones missed (flag up): the whole request again, exactly, from the definition; idle otherwise
    hipLaunchKernelGGL(k_explore_exact, dim3(1, B), dim3(1024), 0, st, core_bits, ctx->n, ctx->d_tile_start,
                       ctx->d_seg_first_tile, T, S, ctx->e_state, worker0, pk, idx_tab, off_tab, (uint32_t)M, ctx->d_flags);
    SLIMDP_LAUNCHED(ctx, "k_explore_exact");
    if (async) {
        // a free slot, else the oldest one (the main stream then waits for that request first)
        int slot = -1;
        for (int j = 0; j < slimdp_ctx::N_PENDING && slot < 0; ++j)
            if (!ctx->pend[j].live) slot = j;
        if (slot < 0) {
            slot = 0;
            for (int j = 1; j < slimdp_ctx::N_PENDING; ++j)
                if (ctx->pend[j].seq < ctx->pend[slot].seq) slot = j;
            SLIMDP_HIP(ctx, hipStreamWaitEvent(ctx->stream, ctx->pend[slot].ev, 0));
        }
        slimdp_ctx::PendingExplore& p = ctx->pend[slot];
        SLIMDP_HIP(ctx, hipEventRecord(p.ev, ctx->side));
        p.live = true; p.seq = ++ctx->pend_seq; p.nw = B;
        p.idx_bytes = M * 4 + 4; p.off_bytes = ((uint64_t)T + 1) * 4;
        for (uint32_t q = 0; q < B; ++q) {
            p.idx[q] = reinterpret_cast<uintptr_t>(expl_idx ? expl_idx[q] : nullptr);
            p.off[q] = reinterpret_cast<uintptr_t>(expl_off[q]);
        }
    }
    return SLIMDP_OK;
}

int slimdp_explore_hint(slimdp_ctx* ctx, const uint64_t* k_seg, uint32_t worker0, uint32_t n_workers,
                        uint64_t iteration, const uint64_t* m_seg)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    ctx->hint.valid = false;
    if (!k_seg || !m_seg) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_explore_hint: NULL argument");
    if (n_workers == 0 || n_workers > ctx->maxW)
        return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_explore_hint: n_workers=%u outside [1, %u]", n_workers, ctx->maxW);
    std::vector<SegInit> init;
    uint64_t M = 0;
    bool narrow = false, short_list = false;
    int rc = explorer_init(ctx, "slimdp_explore_hint", k_seg, m_seg, n_workers, init, &M, &narrow, &short_list);
    if (rc) return rc;
    ctx->hint.iteration = iteration; ctx->hint.worker0 = worker0; ctx->hint.n_workers = n_workers;
    ctx->hint.k_seg.assign(k_seg, k_seg + ctx->n_seg);
    ctx->hint.m_seg.assign(m_seg, m_seg + ctx->n_seg);
    if (ctx->opt_hint_mode == 0) {           // slimdp_score will draw
        ctx->hint.valid = true;
        return SLIMDP_OK;
    }
    if (!narrow || M == 0) return SLIMDP_OK;  // nothing worth drawing ahead: slimdp_sample_explore draws itself
    if (!short_list) { rc = ensure_wide_keys(ctx); if (rc) return rc; }
    // the draw starts now on the side stream, once the previous draw's buffers have been read
    // (the event is recorded here, not after every slimdp_sample_explore: an event on a stream costs a gap between kernels)
    SLIMDP_HIP(ctx, hipEventRecord(ctx->ev_consumed, ctx->stream));
    SLIMDP_HIP(ctx, hipStreamWaitEvent(ctx->side, ctx->ev_consumed, 0));
    rc = init_states(ctx, ctx->e_draw_state, init, n_workers, 0, ctx->side);
    if (rc) return rc;
    // few waves keep the arithmetic units busy; the wave slots stay with the kernels of the main stream
    const uint32_t P = persistent_blocks(ctx, (uint32_t)ctx->opt_side_blocks, n_workers);
    const PhiloxKey pk{(uint32_t)ctx->seed, (uint32_t)(ctx->seed >> 32), (uint32_t)iteration, (uint32_t)(iteration >> 32)};
    const dim3 grid(P, n_workers), block(BLOCK);
#define LAUNCH_SIDE_DRAW(FAST, PAIRS)                                                                                   \
    hipLaunchKernelGGL((k_explore_keys<FAST, PAIRS>), grid, block, 0, ctx->side, ctx->d_tile_start, ctx->d_tile_seg,    \
                       ctx->T, ctx->n_seg, ctx->e_draw_state, ctx->e_sure_bits, ctx->e_cand_bits,                       \
                       (PAIRS) ? ctx->e_pair_keys : ctx->e_cand_keys, ctx->e_cnt_cand,                                  \
                       (PAIRS) ? ctx->pair_stride : ctx->keys_stride, worker0, pk)
    if (ctx->tl.quad_aligned) { if (short_list) LAUNCH_SIDE_DRAW(1, 1); else LAUNCH_SIDE_DRAW(1, 0); }
    else { if (short_list) LAUNCH_SIDE_DRAW(0, 1); else LAUNCH_SIDE_DRAW(0, 0); }
#undef LAUNCH_SIDE_DRAW
    SLIMDP_LAUNCHED(ctx, "k_explore_keys(side stream)");
    SLIMDP_HIP(ctx, hipEventRecord(ctx->ev_drawn, ctx->side));
    ctx->side_pending = true;
    ctx->pre = ctx->hint;
    ctx->pre.valid = true;
    ctx->pre.pairs = short_list;
    return SLIMDP_OK;
}

int slimdp_tile_offsets(slimdp_ctx* ctx, const uint32_t* idx, uint64_t count, uint32_t* off)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    if (!off || (count && !idx)) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_tile_offsets: NULL argument");
    if (count > ctx->n) return fail(ctx, SLIMDP_ERR_OUT_OF_RANGE, "slimdp_tile_offsets: count exceeds n");
    hipLaunchKernelGGL(k_tile_offsets, dim3((ctx->T + 1 + 255) / 256), dim3(256), 0, ctx->stream, idx, count,
                       ctx->d_tile_start, ctx->T, ctx->n, off);
    SLIMDP_LAUNCHED(ctx, "k_tile_offsets");
    return SLIMDP_OK;
}

static int check_lists(slimdp_ctx* ctx, const char* who, uint32_t n_workers, const uint32_t* core_idx,
                       const uint32_t* core_off, uint64_t k, const uint32_t* const* expl_idx,
                       const uint32_t* const* expl_off, const uint64_t* m_w)
{
    if (n_workers == 0 || n_workers > ctx->maxW)
        return fail(ctx, SLIMDP_ERR_INVALID_ARG, "%s: n_workers=%u outside [1, %u]", who, n_workers, ctx->maxW);
    if (!core_off || (k && !core_idx) || !m_w) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "%s: NULL argument", who);
    if (k > ctx->n) return fail(ctx, SLIMDP_ERR_OUT_OF_RANGE, "%s: k exceeds n", who);
    if (!table_ok(expl_off, n_workers)) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "%s: NULL expl_off entry", who);
    for (uint32_t q = 0; q < n_workers; ++q) {
        if (m_w[q] > ctx->n - k) return fail(ctx, SLIMDP_ERR_OUT_OF_RANGE, "%s: m_w[%u] exceeds n - k", who, q);
        if (m_w[q] && (!expl_idx || !expl_idx[q])) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "%s: NULL expl_idx entry", who);
    }
    return SLIMDP_OK;
}

int slimdp_pack(slimdp_ctx* ctx, uint32_t n_workers, const float* const* g, const uint32_t* core_idx,
                const uint32_t* core_off, uint64_t k, const uint32_t* const* expl_idx, const uint32_t* const* expl_off,
                const uint64_t* m_w, float* const* core_val, float* const* expl_val, uint64_t core_epoch, uint32_t flags)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    if (flags & ~SLIMDP_PACK_UPDATES_AS_SCORED) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_pack: unknown flag bits 0x%x", flags);
    int rc = check_lists(ctx, "slimdp_pack", n_workers, core_idx, core_off, k, expl_idx, expl_off, m_w);
    if (rc) return rc;
    if (!table_ok(g, n_workers)) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_pack: NULL update pointer");
    for (uint32_t q = 0; q < n_workers; ++q) {
        if (k && (!core_val || !core_val[q])) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_pack: NULL core_val entry");
        if (m_w[q] && (!expl_val || !expl_val[q])) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_pack: NULL expl_val entry");
    }
    rc = check_epoch(ctx, core_epoch);
    if (rc) return rc;
    // The caller states that g is what the last scoring pass read.  That the contents are unchanged cannot be
    // checked here; that it is the same table can.
    const bool as_scored = (flags & SLIMDP_PACK_UPDATES_AS_SCORED) != 0;
    if (as_scored && ctx->spec.captured) {
        bool same = ctx->spec.W == n_workers;
        for (uint32_t q = 0; same && q < n_workers; ++q) same = ctx->spec.g[q] == g[q];
        if (!same)
            return fail(ctx, SLIMDP_ERR_INVALID_ARG,
                        "slimdp_pack: SLIMDP_PACK_UPDATES_AS_SCORED, but g is not the table of arrays the last slimdp_score read");
    }
    // the scoring pass of this very selection kept the core's update values: no second pass over the updates
    const bool spec = as_scored && ctx->spec.on && ctx->spec.captured && ctx->spec.core_epoch == core_epoch;
    if (spec) {
        ctx->spec.captured = false;      // one capture serves one pack
        if (k && ctx->n_seg == 1) {
            // flat model: tile = index / 4096; all tiles but a ragged last one are full
            const uint32_t T_full = (uint32_t)(ctx->n / TILE);
            // many short blocks: work on the side stream (an asynchronous explorer request) gets its turn between them
            uint64_t blocks = (k + 1023) / 1024;
            if (blocks > 32768) blocks = 32768;
            // while an explorer request runs on the side stream: few resident blocks, so that its small kernels find free
            // slots at once (measured: 2.54 -> 2.48 ms per step with one block per compute unit)
            bool side_busy = false;
            for (int j = 0; j < slimdp_ctx::N_PENDING; ++j) side_busy = side_busy || ctx->pend[j].live;
            const uint64_t per_cu = ctx->opt_pack_core_blocks > 0 ? (uint64_t)ctx->opt_pack_core_blocks : (side_busy ? 1u : 0u);
            if (per_cu > 0 && blocks > (uint64_t)ctx->cus * per_cu) blocks = (uint64_t)ctx->cus * per_cu;
            hipLaunchKernelGGL(k_pack_core_flat, dim3((uint32_t)blocks), dim3(256), 0, ctx->stream, make_tab<PtrTab>(g, n_workers),
                               n_workers, ctx->n, T_full, core_idx, (uint32_t)k, ctx->spec.bits, ctx->spec.vals, ctx->spec.fail,
                               ctx->spec.vec_ok, make_tab<MutPtrTab>(core_val, n_workers));
            SLIMDP_LAUNCHED(ctx, "k_pack_core_flat");
        } else if (k) {
            hipLaunchKernelGGL(k_pack_core_spec, dim3((ctx->T + 3) / 4), dim3(BLOCK), 0, ctx->stream, make_tab<PtrTab>(g, n_workers),
                               n_workers, ctx->n, ctx->d_tile_start, ctx->d_tile_seg, ctx->T, core_idx, core_off, ctx->spec.bits,
                               ctx->spec.vals, ctx->spec.fail, ctx->spec.vec_ok,
                               make_tab<MutPtrTab>(core_val, n_workers));
            SLIMDP_LAUNCHED(ctx, "k_pack_core_spec");
        }
        CountTab mt{};
        uint64_t mmax = 0;
        for (uint32_t q = 0; q < n_workers; ++q) { mt.c[q] = (uint32_t)m_w[q]; if (m_w[q] > mmax) mmax = m_w[q]; }
        rc = wait_for_lists(ctx, n_workers, expl_idx, expl_off, m_w);    // the core values above did not need the explorer lists; these do
        if (rc) return rc;
        if (mmax) {
            uint64_t blocks = (mmax + 1023) / 1024;
            if (blocks > 2048) blocks = 2048;
            hipLaunchKernelGGL(k_pack_expl_gather, dim3((uint32_t)blocks, n_workers), dim3(256), 0, ctx->stream,
                               make_tab<PtrTab>(g, n_workers), ctx->n, make_tab<PtrTab>(expl_idx, n_workers), mt,
                               make_tab<MutPtrTab>(expl_val, n_workers));
            SLIMDP_LAUNCHED(ctx, "k_pack_expl_gather");
        }
        return SLIMDP_OK;
    }
    rc = wait_for_lists(ctx, n_workers, expl_idx, expl_off, m_w);
    if (rc) return rc;
    int vec_ok = 1;
    for (uint32_t q = 0; q < n_workers; ++q) vec_ok = vec_ok && aligned16(g[q]);
    if (ctx->opt_pack_kernel == 1) {
        hipLaunchKernelGGL(k_pack_stream_ws, dim3(8 * ((ctx->T + 7) / 8)), dim3(2 * BLOCK), 0, ctx->stream,
                           make_tab<PtrTab>(g, n_workers), n_workers, ctx->T, ctx->d_tile_start, core_idx, core_off,
                           make_tab<PtrTab>(expl_idx, n_workers), make_tab<PtrTab>(expl_off, n_workers),
                           make_tab<MutPtrTab>(core_val, n_workers), make_tab<MutPtrTab>(expl_val, n_workers), vec_ok);
        SLIMDP_LAUNCHED(ctx, "k_pack_stream_ws");
        return SLIMDP_OK;
    }
    if (ctx->opt_pack_nbuf == 2)
        hipLaunchKernelGGL(k_pack_stream<2>, dim3(ctx->T), dim3(BLOCK), 0, ctx->stream, make_tab<PtrTab>(g, n_workers),
                           n_workers, ctx->d_tile_start, core_idx, core_off, make_tab<PtrTab>(expl_idx, n_workers),
                           make_tab<PtrTab>(expl_off, n_workers), make_tab<MutPtrTab>(core_val, n_workers),
                           make_tab<MutPtrTab>(expl_val, n_workers), vec_ok);
    else
        hipLaunchKernelGGL(k_pack_stream<1>, dim3(ctx->T), dim3(BLOCK), 0, ctx->stream, make_tab<PtrTab>(g, n_workers),
                           n_workers, ctx->d_tile_start, core_idx, core_off, make_tab<PtrTab>(expl_idx, n_workers),
                           make_tab<PtrTab>(expl_off, n_workers), make_tab<MutPtrTab>(core_val, n_workers),
                           make_tab<MutPtrTab>(expl_val, n_workers), vec_ok);
    SLIMDP_LAUNCHED(ctx, "k_pack_stream");
    return SLIMDP_OK;
}

int slimdp_merge(slimdp_ctx* ctx, float* w, float lr, uint64_t core_epoch, uint32_t n_workers, const uint32_t* core_idx,
                 const uint32_t* core_off, uint64_t k, const float* const* core_val, const uint32_t* const* expl_idx,
                 const uint32_t* const* expl_off, const float* const* expl_val, const uint64_t* m_w)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    if (!w) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_merge: w is NULL");
    int rc = check_lists(ctx, "slimdp_merge", n_workers, core_idx, core_off, k, expl_idx, expl_off, m_w);
    if (rc) return rc;
    for (uint32_t q = 0; q < n_workers; ++q) {
        if (k && (!core_val || !core_val[q])) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_merge: NULL core_val entry");
        if (m_w[q] && (!expl_val || !expl_val[q])) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_merge: NULL expl_val entry");
    }
    rc = check_epoch(ctx, core_epoch);
    if (rc) return rc;
    rc = wait_for_lists(ctx, n_workers, expl_idx, expl_off, m_w);
    if (rc) return rc;
    hipLaunchKernelGGL(k_merge, dim3(ctx->T), dim3(BLOCK), 0, ctx->stream, w, lr, n_workers, ctx->d_tile_start, core_idx,
                       core_off, make_tab<PtrTab>(core_val, n_workers), make_tab<PtrTab>(expl_idx, n_workers),
                       make_tab<PtrTab>(expl_off, n_workers), make_tab<PtrTab>(expl_val, n_workers), (int)aligned16(w),
                       ctx->n, ctx->n_seg);
    SLIMDP_LAUNCHED(ctx, "k_merge");
    return SLIMDP_OK;
}

int slimdp_pull(slimdp_ctx* ctx, const float* w, uint64_t core_epoch, uint32_t n_workers, const uint32_t* core_idx,
                const uint32_t* core_off, uint64_t k, const uint32_t* const* expl_idx, const uint32_t* const* expl_off,
                const uint64_t* m_w, float* const* core_out, float* const* expl_out, float* const* w_local)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    if (!w) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_pull: w is NULL");
    int rc = check_lists(ctx, "slimdp_pull", n_workers, core_idx, core_off, k, expl_idx, expl_off, m_w);
    if (rc) return rc;
    for (uint32_t q = 0; q < n_workers; ++q) {
        if (k && (!core_out || !core_out[q])) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_pull: NULL core_out entry");
        if (m_w[q] && (!expl_out || !expl_out[q])) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_pull: NULL expl_out entry");
        if (w_local && w_local[q] == w) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_pull: w_local aliases w");
    }
    rc = check_epoch(ctx, core_epoch);
    if (rc) return rc;
    rc = wait_for_lists(ctx, n_workers, expl_idx, expl_off, m_w);
    if (rc) return rc;
    const float* src = w;
    bool any_local = false;
    for (uint32_t q = 0; w_local && q < n_workers; ++q) any_local = any_local || w_local[q] != nullptr;
    // the values at the communication sets; the local models are patched by a pass of their own that streams them (a
    // scattered 4-byte write per value would touch nearly every line of every local model, at a fraction of the rate)
    hipLaunchKernelGGL(k_gather, dim3(ctx->T), dim3(BLOCK), 0, ctx->stream, make_tab<PtrTab, const float*>(&src, 1), 1,
                       n_workers, ctx->n, core_idx, core_off, make_tab<PtrTab>(expl_idx, n_workers),
                       make_tab<PtrTab>(expl_off, n_workers), make_tab<MutPtrTab>(core_out, n_workers),
                       make_tab<MutPtrTab>(expl_out, n_workers),
                       make_tab<MutPtrTab>(w_local, (w_local && ctx->opt_pull_kernel == 0) ? n_workers : 0));
    SLIMDP_LAUNCHED(ctx, "k_gather(pull)");
    if (any_local && ctx->opt_pull_kernel == 1) {
        int vec_ok = aligned16(w);
        for (uint32_t q = 0; q < n_workers; ++q) vec_ok = vec_ok && (!w_local[q] || aligned16(w_local[q]));
        hipLaunchKernelGGL(k_pull_local_step<0>, dim3(ctx->T), dim3(BLOCK), 0, ctx->stream, w,
                           make_tab<MutPtrTab>(w_local, n_workers), PtrTab{}, MutPtrTab{}, 0.0f, 1, n_workers, ctx->d_tile_start,
                           core_idx, core_off, make_tab<PtrTab>(expl_idx, n_workers), make_tab<PtrTab>(expl_off, n_workers), vec_ok);
        SLIMDP_LAUNCHED(ctx, "k_pull_local_step<0>");
    }
    return SLIMDP_OK;
}

int slimdp_local_step(slimdp_ctx* ctx, uint32_t n_workers, float* const* w_local, const float* const* grad,
                      float* const* delta, float eta, uint32_t flags)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    if (flags & ~SLIMDP_LOCAL_FIRST) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_local_step: unknown flag bits 0x%x", flags);
    if (n_workers == 0 || n_workers > ctx->maxW)
        return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_local_step: n_workers=%u outside [1, %u]", n_workers, ctx->maxW);
    if (!table_ok(w_local, n_workers) || !table_ok(grad, n_workers) || !table_ok(delta, n_workers))
        return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_local_step: NULL array");
    if (!std::isfinite(eta)) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_local_step: eta must be finite");
    int vec_ok = 1;
    for (uint32_t q = 0; q < n_workers; ++q) {
        vec_ok = vec_ok && aligned16(w_local[q]) && aligned16(grad[q]) && aligned16(delta[q]);
        if (static_cast<const void*>(w_local[q]) == static_cast<const void*>(delta[q]) ||
            static_cast<const void*>(grad[q]) == static_cast<const void*>(delta[q]) ||
            static_cast<const void*>(grad[q]) == static_cast<const void*>(w_local[q]))
            return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_local_step: arrays of worker %u alias", q);
    }
    uint64_t blocks = (ctx->n / 4 + 511) / 512;
    const uint64_t cap = (uint64_t)ctx->cus * 16 / n_workers + 1;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(k_local_step, dim3((uint32_t)blocks, n_workers), dim3(256), 0, ctx->stream, make_tab<MutPtrTab>(w_local, n_workers),
                       make_tab<PtrTab>(grad, n_workers), make_tab<MutPtrTab>(delta, n_workers), ctx->n, eta,
                       (int)((flags & SLIMDP_LOCAL_FIRST) != 0), vec_ok);
    SLIMDP_LAUNCHED(ctx, "k_local_step");
    return SLIMDP_OK;
}

int slimdp_local_step_pack(slimdp_ctx* ctx, uint32_t n_workers, float* const* w_local, const float* const* grad,
                           float* const* delta, float eta, uint32_t flags, const uint32_t* core_idx, const uint32_t* core_off,
                           uint64_t k, const uint32_t* const* expl_idx, const uint32_t* const* expl_off, const uint64_t* m_w,
                           float* const* core_val, float* const* expl_val, uint64_t core_epoch)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    if (flags & ~SLIMDP_LOCAL_FIRST) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_local_step_pack: unknown flag bits 0x%x", flags);
    int rc = check_lists(ctx, "slimdp_local_step_pack", n_workers, core_idx, core_off, k, expl_idx, expl_off, m_w);
    if (rc) return rc;
    if (!table_ok(w_local, n_workers) || !table_ok(grad, n_workers) || !table_ok(delta, n_workers))
        return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_local_step_pack: NULL array");
    if (!std::isfinite(eta)) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_local_step_pack: eta must be finite");
    int vec_ok = 1;
    for (uint32_t q = 0; q < n_workers; ++q) {
        vec_ok = vec_ok && aligned16(w_local[q]) && aligned16(grad[q]) && aligned16(delta[q]);
        if (static_cast<const void*>(w_local[q]) == static_cast<const void*>(delta[q]) ||
            static_cast<const void*>(grad[q]) == static_cast<const void*>(delta[q]) ||
            static_cast<const void*>(grad[q]) == static_cast<const void*>(w_local[q]))
            return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_local_step_pack: arrays of worker %u alias", q);
        if (k && (!core_val || !core_val[q])) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_local_step_pack: NULL core_val entry");
        if (m_w[q] && (!expl_val || !expl_val[q])) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_local_step_pack: NULL expl_val entry");
    }
    rc = check_epoch(ctx, core_epoch);
    if (rc) return rc;
    rc = wait_for_lists(ctx, n_workers, expl_idx, expl_off, m_w);
    if (rc) return rc;
    const int first = (flags & SLIMDP_LOCAL_FIRST) != 0;
    if (ctx->opt_pack_nbuf == 2)
        hipLaunchKernelGGL(k_local_step_pack<2>, dim3(ctx->T), dim3(BLOCK), 0, ctx->stream, make_tab<MutPtrTab>(w_local, n_workers),
                           make_tab<PtrTab>(grad, n_workers), make_tab<MutPtrTab>(delta, n_workers), eta, first, n_workers,
                           ctx->d_tile_start, core_idx, core_off, make_tab<PtrTab>(expl_idx, n_workers),
                           make_tab<PtrTab>(expl_off, n_workers), make_tab<MutPtrTab>(core_val, n_workers),
                           make_tab<MutPtrTab>(expl_val, n_workers), vec_ok);
    else
        hipLaunchKernelGGL(k_local_step_pack<1>, dim3(ctx->T), dim3(BLOCK), 0, ctx->stream, make_tab<MutPtrTab>(w_local, n_workers),
                           make_tab<PtrTab>(grad, n_workers), make_tab<MutPtrTab>(delta, n_workers), eta, first, n_workers,
                           ctx->d_tile_start, core_idx, core_off, make_tab<PtrTab>(expl_idx, n_workers),
                           make_tab<PtrTab>(expl_off, n_workers), make_tab<MutPtrTab>(core_val, n_workers),
                           make_tab<MutPtrTab>(expl_val, n_workers), vec_ok);
    SLIMDP_LAUNCHED(ctx, "k_local_step_pack");
    return SLIMDP_OK;
}

int slimdp_pull_local_step(slimdp_ctx* ctx, const float* w, uint64_t core_epoch, uint32_t n_workers, const uint32_t* core_idx,
                           const uint32_t* core_off, uint64_t k, const uint32_t* const* expl_idx,
                           const uint32_t* const* expl_off, const uint64_t* m_w, float* const* w_local,
                           const float* const* grad, float* const* delta, float eta, uint32_t flags)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    if (!w) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_pull_local_step: w is NULL");
    if (flags & ~SLIMDP_LOCAL_FIRST) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_pull_local_step: unknown flag bits 0x%x", flags);
    int rc = check_lists(ctx, "slimdp_pull_local_step", n_workers, core_idx, core_off, k, expl_idx, expl_off, m_w);
    if (rc) return rc;
    if (!table_ok(w_local, n_workers) || !table_ok(grad, n_workers) || !table_ok(delta, n_workers))
        return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_pull_local_step: NULL array");
    if (!std::isfinite(eta)) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_pull_local_step: eta must be finite");
    int vec_ok = aligned16(w);
    for (uint32_t q = 0; q < n_workers; ++q) {
        vec_ok = vec_ok && aligned16(w_local[q]) && aligned16(grad[q]) && aligned16(delta[q]);
        const void *a = w_local[q], *b = grad[q], *c = delta[q];
        if (a == b || a == c || b == c || a == static_cast<const void*>(w) || c == static_cast<const void*>(w))
            return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_pull_local_step: arrays of worker %u alias", q);
    }
    rc = check_epoch(ctx, core_epoch);
    if (rc) return rc;
    rc = wait_for_lists(ctx, n_workers, expl_idx, expl_off, m_w);
    if (rc) return rc;
    hipLaunchKernelGGL(k_pull_local_step<1>, dim3(ctx->T), dim3(BLOCK), 0, ctx->stream, w, make_tab<MutPtrTab>(w_local, n_workers),
                       make_tab<PtrTab>(grad, n_workers), make_tab<MutPtrTab>(delta, n_workers), eta,
                       (int)((flags & SLIMDP_LOCAL_FIRST) != 0), n_workers, ctx->d_tile_start, core_idx, core_off,
                       make_tab<PtrTab>(expl_idx, n_workers), make_tab<PtrTab>(expl_off, n_workers), vec_ok);
    SLIMDP_LAUNCHED(ctx, "k_pull_local_step");
    return SLIMDP_OK;
}

static int quant_args(slimdp_ctx* ctx, const char* who, uint32_t n_workers, const void* const* a, const void* const* b,
                      const void* const* c, const uint64_t* count, Count64Tab* ct, uint64_t* cmax)
{
    if (n_workers == 0 || n_workers > ctx->maxW)
        return fail(ctx, SLIMDP_ERR_INVALID_ARG, "%s: n_workers=%u outside [1, %u]", who, n_workers, ctx->maxW);
    if (!count || !a || !b || !c) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "%s: NULL argument", who);
    *cmax = 0;
    for (uint32_t q = 0; q < n_workers; ++q) {
        if (count[q] > ctx->n) return fail(ctx, SLIMDP_ERR_OUT_OF_RANGE, "%s: count[%u] exceeds n", who, q);
        if (count[q] && (!a[q] || !b[q] || !c[q])) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "%s: NULL array of worker %u", who, q);
        ct->c[q] = count[q];
        if (count[q] > *cmax) *cmax = count[q];
    }
    return SLIMDP_OK;
}

int slimdp_quantize(slimdp_ctx* ctx, uint32_t n_workers, uint32_t worker0, const float* const* val, const uint64_t* count,
                    uint32_t kind, uint64_t iteration, uint8_t* const* code, float* const* scale)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    if (kind > 1) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_quantize: kind must be 0 (core values) or 1 (explorer values)");
    Count64Tab ct{};
    uint64_t cmax = 0;
    int rc = quant_args(ctx, "slimdp_quantize", n_workers, reinterpret_cast<const void* const*>(val),
                        reinterpret_cast<const void* const*>(code), reinterpret_cast<const void* const*>(scale), count, &ct, &cmax);
    if (rc) return rc;
    if (cmax == 0) return SLIMDP_OK;
    int vec_ok = 1;
    for (uint32_t q = 0; q < n_workers; ++q)
        vec_ok = vec_ok && aligned16(val[q]) && (reinterpret_cast<uintptr_t>(code[q]) & 3u) == 0;
    const uint64_t buckets = (cmax + QB - 1) / QB;
    const PhiloxKey pk{(uint32_t)ctx->seed, (uint32_t)(ctx->seed >> 32), (uint32_t)iteration, (uint32_t)(iteration >> 32)};
    hipLaunchKernelGGL(k_quantize, dim3((uint32_t)((buckets + 3) / 4), n_workers), dim3(BLOCK), 0, ctx->stream,
                       make_tab<PtrTab>(val, n_workers), ct, kind, worker0, pk, make_tab<MutPtrTab>(code, n_workers),
                       make_tab<MutPtrTab>(scale, n_workers), vec_ok);
    SLIMDP_LAUNCHED(ctx, "k_quantize");
    return SLIMDP_OK;
}

int slimdp_dequantize(slimdp_ctx* ctx, uint32_t n_workers, const uint8_t* const* code, const float* const* scale,
                      const uint64_t* count, float* const* val)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    Count64Tab ct{};
    uint64_t cmax = 0;
    int rc = quant_args(ctx, "slimdp_dequantize", n_workers, reinterpret_cast<const void* const*>(code),
                        reinterpret_cast<const void* const*>(scale), reinterpret_cast<const void* const*>(val), count, &ct, &cmax);
    if (rc) return rc;
    if (cmax == 0) return SLIMDP_OK;
    int vec_ok = 1;
    for (uint32_t q = 0; q < n_workers; ++q)
        vec_ok = vec_ok && aligned16(val[q]) && (reinterpret_cast<uintptr_t>(code[q]) & 3u) == 0;
    uint64_t blocks = (cmax / 4 + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(k_dequantize, dim3((uint32_t)blocks, n_workers), dim3(256), 0, ctx->stream, make_tab<PtrTab>(code, n_workers),
                       make_tab<PtrTab>(scale, n_workers), ct, make_tab<MutPtrTab>(val, n_workers), vec_ok);
    SLIMDP_LAUNCHED(ctx, "k_dequantize");
    return SLIMDP_OK;
}

int slimdp_core_signature(slimdp_ctx* ctx, const uint32_t* core_idx, uint64_t k, uint64_t* sig)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    if (!sig || (k && !core_idx)) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_core_signature: NULL argument");
    if (k > ctx->n) return fail(ctx, SLIMDP_ERR_OUT_OF_RANGE, "slimdp_core_signature: k exceeds n");
    int rc = fill(ctx, reinterpret_cast<uint32_t*>(sig), 2, 0u);
    if (rc) return rc;
    if (k) {
        hipLaunchKernelGGL(k_signature, dim3(fill_grid(k)), dim3(256), 0, ctx->stream, core_idx, k,
                           reinterpret_cast<unsigned long long*>(sig));
        SLIMDP_LAUNCHED(ctx, "k_signature");
    }
    return SLIMDP_OK;
}

int slimdp_debug_philox(slimdp_ctx* ctx, uint64_t iteration, uint32_t worker, uint32_t i0, uint64_t count, uint32_t* out)
{
    if (!ctx) return SLIMDP_ERR_INVALID_ARG;
    if (count && !out) return fail(ctx, SLIMDP_ERR_INVALID_ARG, "slimdp_debug_philox: out is NULL");
    if (count == 0) return SLIMDP_OK;
    hipLaunchKernelGGL(k_debug_philox, dim3(fill_grid(count)), dim3(256), 0, ctx->stream, (uint32_t)ctx->seed,
                       (uint32_t)(ctx->seed >> 32), (uint32_t)iteration, (uint32_t)(iteration >> 32), worker, i0, count, out);
    SLIMDP_LAUNCHED(ctx, "k_debug_philox");
    return SLIMDP_OK;
}

}  // extern "C"
