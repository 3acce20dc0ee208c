// Host side of libcusa: argument checks, workspace layout, launch geometry and
// the per-layer walk of Alg. 1.  Everything here only enqueues kernels on the
// caller's stream; nothing allocates device memory or synchronises.
#include "../../include/cusa.h"

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <atomic>
#include <mutex>
#include <utility>
#include <vector>

#include "cusa_kernels.hpp"

using namespace cusa;

namespace {

// ------------------------------------------------------------------ profiling

enum KernelId { KID_SCORE = 0, KID_TOPK, KID_UNION, KID_ATTN_FULL, KID_ATTN_SPARSE, KID_REDUCE, KID_ATTN_SELECT, KID_ATTN_PER_HEAD, KID_RHO_PER_HEAD, KID_RANK_AGG, KID_RECALL, KID_PROBE, KID_TOPK_SLICE, KID_TOPK_MERGE, KID_PROBE_GATHER, KID_PROBE_RW_SCATTER, KID_PROBE_RW_BURST, KID_SAMPLE_THRESHOLD, KID_TOPK_FILTERED, KID_PROBE_TILES, KID_COUNT };
const char* const kKernelNames[KID_COUNT] = {"attn_kernel<scores only>", "topk_kernel", "union_kernel",
                                             "attn_kernel<full>", "attn_kernel<sparse>", "attn_reduce_kernel",
                                             "attn_kernel<full+score>", "attn_kernel<per-head>", "per_head_rho_kernel",
                                             "rank_aggregate_kernel", "recall_kernel", "probe_stream_read_kernel", "topk_kernel<slice>",
                                             "topk_kernel<merge>", "probe_traffic_kernel<gather>", "probe_traffic_kernel<scattered writes>",
                                             "probe_traffic_kernel<burst writes>", "sample_threshold_kernel", "topk_kernel<filtered>", "probe_traffic_kernel<stream>"};

// With the profiler on, every launch carries a start and a stop event that the runtime fills
// from the dispatch's own begin and end timestamps (hipExtLaunchKernelGGL), which is what a
// kernel trace reports: the figures exclude the gaps between kernels and the events' own cost.
struct ProfRec {
    int id;
    hipEvent_t start, stop;
};
struct Profiler {
    std::mutex mu;
    std::atomic<bool> on{false};
    std::vector<ProfRec> recs;
    std::vector<hipEvent_t> pool;
    int64_t calls[KID_COUNT] = {0};
    double ms[KID_COUNT] = {0};
} g_prof;

hipEvent_t prof_event() {
    if (!g_prof.pool.empty()) {
        hipEvent_t e = g_prof.pool.back();
        g_prof.pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    return e;
}

template <typename T>
struct same_as { using type = T; };

// Every kernel of the library is launched through here; the arguments are converted to the
// kernel's parameter types before they are packed.
template <typename... KArgs>
void launch(int kid, void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t shmem, hipStream_t s,
            typename same_as<KArgs>::type... args) {
    if (!g_prof.on.load(std::memory_order_acquire)) {
        kernel<<<grid, block, shmem, s>>>(args...);
        return;
    }
    ProfRec rec;
    rec.id = kid;
    {
        std::lock_guard<std::mutex> lk(g_prof.mu);
        rec.start = prof_event();
        rec.stop = prof_event();
        if (!rec.start || !rec.stop) {                // no events to be had: launch untimed
            if (rec.start) g_prof.pool.push_back(rec.start);
            if (rec.stop) g_prof.pool.push_back(rec.stop);
            rec.start = rec.stop = nullptr;
        }
    }
    if (!rec.start) {
        kernel<<<grid, block, shmem, s>>>(args...);
        return;
    }
    hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)shmem, s, rec.start, rec.stop, 0, args...);
    std::lock_guard<std::mutex> lk(g_prof.mu);
    g_prof.recs.push_back(rec);
}

// ------------------------------------------------------------------ validation

bool valid_group(int g) { return g == 1 || g == 2 || g == 4 || g == 8; }

int resolved_k(const cusa_params* p) { return p->topk_per_head > 0 ? p->topk_per_head : p->budget - p->window; }

cusa_status check_params(const cusa_params* p, bool need_budget) {
    if (!p) return CUSA_ERR_INVALID_ARG;
    if (p->batch < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1) return CUSA_ERR_INVALID_ARG;
    if (p->n_q_heads % p->n_kv_heads != 0) return CUSA_ERR_INVALID_ARG;
    if (p->head_dim != D) return CUSA_ERR_UNSUPPORTED;
    if (!valid_group(p->n_q_heads / p->n_kv_heads)) return CUSA_ERR_UNSUPPORTED;
    if (p->batch > 65535 || p->n_q_heads > 65535) return CUSA_ERR_UNSUPPORTED;
    if (!(p->sm_scale > 0.0f) || !(p->sm_scale < 1e30f)) return CUSA_ERR_INVALID_ARG;
    if (need_budget) {
        if (p->budget < 1 || p->window < 0 || p->window > p->budget) return CUSA_ERR_INVALID_ARG;
        if (p->topk_per_head < 0) return CUSA_ERR_INVALID_ARG;
        if (p->n_sink < 0 || p->n_sink > p->budget - p->window) return CUSA_ERR_INVALID_ARG;
        if (p->rank_mode != CUSA_RANK_FIRST_OCCURRENCE && p->rank_mode != CUSA_RANK_VOTES &&
            p->rank_mode != CUSA_RANK_MAX_SCORE)
            return CUSA_ERR_INVALID_ARG;
        const int k = resolved_k(p);
        if (k < p->budget - p->window - p->n_sink) return CUSA_ERR_INVALID_ARG;
        if (k > 8192) return CUSA_ERR_UNSUPPORTED;
    }
    return CUSA_OK;
}

cusa_status check_kv(const cusa_params* p, const cusa_kv* kv) {
    if (!kv || !kv->k || !kv->v || !kv->seq_lens) return CUSA_ERR_INVALID_ARG;
    if (kv->max_seq_len < 1) return CUSA_ERR_INVALID_ARG;
    if (((uintptr_t)kv->k | (uintptr_t)kv->v) & 15) return CUSA_ERR_INVALID_ARG;
    if (kv->layout == CUSA_KV_CONTIGUOUS) {
        if (kv->stride_token < D || (kv->stride_token & 7) || (kv->stride_head & 7) || (kv->stride_batch & 7))
            return CUSA_ERR_INVALID_ARG;
        if (kv->stride_head < 0 || kv->stride_batch < 0) return CUSA_ERR_INVALID_ARG;
    } else if (kv->layout == CUSA_KV_PAGED) {
        if (kv->page_size != PAGE) return CUSA_ERR_UNSUPPORTED;
        if (!kv->block_table || kv->n_pages < 1) return CUSA_ERR_INVALID_ARG;
        if ((int64_t)kv->max_pages * PAGE < kv->max_seq_len) return CUSA_ERR_INVALID_ARG;
    } else {
        return CUSA_ERR_INVALID_ARG;
    }
    (void)p;
    return CUSA_OK;
}

KvView make_view(const cusa_params* p, const cusa_kv* kv) {
    KvView v;
    v.k = static_cast<const uint16_t*>(kv->k);
    v.v = static_cast<const uint16_t*>(kv->v);
    v.sb = kv->stride_batch;
    v.sh = kv->stride_head;
    v.st = kv->stride_token;
    v.bt = kv->block_table;
    v.max_pages = kv->max_pages;
    v.G = p->n_kv_heads;
    v.seq_lens = kv->seq_lens;
    return v;
}

// ------------------------------------------------------------------ workspace

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

constexpr int MAX_SPLITS = 256;
constexpr int TARGET_WGS = 512;     // two resident workgroups per CU
constexpr int CHUNK_CAP = 2048;
static_assert(ATTN_SCORE_CHUNK_CAP <= CHUNK_CAP && ATTN_SCORE_CHUNK_CAP_G8 <= CHUNK_CAP, "the split bound assumes it");

struct AttnPlan {
    int ti;        // row-load instructions per wave iteration (4 or 8)
    int chunk;     // tokens per workgroup, a multiple of the workgroup tile
    int n_splits;  // grid.x = ceil(n_max / chunk)
};

// Workgroup granularity for n_max tokens per (sequence, KV head): about TARGET_WGS workgroups
// when every sequence has n_max tokens, but never more than CHUNK_CAP tokens per workgroup, so
// that a large ragged batch is cut into equal pieces instead of one piece per sequence.
// Workgroups with long runs (1024 tokens or more) load 8 rows per lane and iteration, which keeps
// more bytes in flight; short runs are faster with 4 (measured on all five workloads).
AttnPlan plan_attn(int n_max, int BG, int g, bool wide = false) {
    AttnPlan pl;
    int64_t chunk = ((int64_t)n_max * BG + TARGET_WGS - 1) / TARGET_WGS;
    // the scoring variant keeps the scores of a workgroup's whole run in LDS
    const int cap = !wide ? CHUNK_CAP : g >= 8 ? ATTN_SCORE_CHUNK_CAP_G8 : ATTN_SCORE_CHUNK_CAP;
    if (chunk > cap) chunk = cap;
    pl.ti = wide ? (chunk >= 512 ? 16 : 8) : chunk >= 1024 ? 8 : 4;
    const int wg_tile = pl.ti * 4 * ATTN_WAVES;
    chunk = (chunk + wg_tile - 1) / wg_tile * wg_tile;
    if ((n_max + chunk - 1) / chunk > MAX_SPLITS) {
        chunk = ((int64_t)n_max + MAX_SPLITS - 1) / MAX_SPLITS;
        chunk = (chunk + wg_tile - 1) / wg_tile * wg_tile;
    }
    pl.chunk = (int)chunk;
    pl.n_splits = (int)((n_max + chunk - 1) / chunk);
    if (pl.n_splits < 1) pl.n_splits = 1;
    return pl;
}

// Upper bound of plan_attn(m, BG', g).n_splits over every m <= n_max and BG' >= BG: with the chunk
// below its cap a token list is cut into at most ceil(TARGET_WGS / BG) pieces, at the cap into
// ceil(m / cap).  Monotone in n_max, so a workspace sized for a capacity serves every
// shorter bound.
int max_splits_bound(int n_max, int BG, int g) {
    const int cap = g >= 8 ? ATTN_SCORE_CHUNK_CAP_G8 : CHUNK_CAP;   // the smallest cap any variant of this group size has
    const int by_wgs = (TARGET_WGS + BG - 1) / BG;
    const int by_cap = (n_max + cap - 1) / cap;
    const int m = by_wgs > by_cap ? by_wgs : by_cap;
    return m < MAX_SPLITS ? m : MAX_SPLITS;
}

// Slices a row of up to lc_max candidates is cut into: only few long rows are cut (more rows than
// CUs keep every CU busy anyway), into pieces of about 32768 candidates that a workgroup holds in
// registers, and only as far as the merge can hold the slices' picks in registers (16384 composites).
int plan_topk_slices(int64_t rows, int lc_max, int k) {
    if (lc_max <= 32768 || k < 1) return 1;
    int64_t s = ((int64_t)lc_max + 32767) / 32768;
    if (s > 8) s = 8;
    if (s > 16384 / k) s = 16384 / k;
    if (s > 512 / rows) s = 512 / rows;
    return s < 1 ? 1 : (int)s;
}

// Sampling plan of the filtered fast path for sequences of up to lc candidate positions: the kernel
// samples every SAMPLE_STEP-th tile of 64 tokens of a sequence, or as many tiles as it has LDS for
// (n_slots sample slots per head); tile_step is the step of a sequence as long as the bound.
struct SamplePlan {
    int tile_step, n_slots;
};
SamplePlan plan_sample(int64_t lc) {
    const int64_t tiles_all = (lc + SCORE_ROWS - 1) / SCORE_ROWS;
    int64_t tiles = (tiles_all + SAMPLE_STEP - 1) / SAMPLE_STEP;
    if (tiles > SAMPLE_MAX_TILES) tiles = SAMPLE_MAX_TILES;
    int64_t step = (tiles_all + tiles - 1) / tiles;
    if (step < SAMPLE_STEP) step = SAMPLE_STEP;
    return {(int)step, (int)tiles * SCORE_ROWS};
}
int filter_cap_for(int k) { return k <= 2048 ? 4096 : 8192; }
size_t sample_lds_bytes(int g, int n_slots) { return (size_t)g * ((size_t)n_slots + THR_BINS) * 4; }

// Whether a selection layer takes the filtered fast path (sample_threshold_kernel): it pays where the
// scores of the layer are many (tens of MB of them) and a head keeps a small share of its candidates;
// it needs the default ranking (the max-score reading looks picks' scores up in P, which the fast path
// does not write), a k the merge form of the top-k holds in registers, query groups of at most 4 heads
// (the filtered pass of a group of 8 does not fit the register file), and a sample dense enough that
// what a head of the longest sequence is expected to keep fits its buffer with room to spare.
constexpr int64_t FILTER_MIN_SCORES = (int64_t)8 << 20;
// Everything but the sample's density: once true it stays true for longer bounds, so the workspace laid
// out for a capacity serves every shorter bound.
bool filter_buffers_needed(const cusa_params* p, int max_seq_len) {
    const int64_t lc = (int64_t)max_seq_len - p->window;
    const int k = resolved_k(p);
    return p->rank_mode == CUSA_RANK_FIRST_OCCURRENCE && p->n_q_heads / p->n_kv_heads <= 4 && k >= 1 && k <= 4096 &&
           lc >= 4 * (int64_t)k && (int64_t)p->batch * p->n_q_heads * lc >= FILTER_MIN_SCORES;
}
bool filtered_select(const cusa_params* p, int max_seq_len) {
    if (!filter_buffers_needed(p, max_seq_len)) return false;
    const int64_t lc = (int64_t)max_seq_len - p->window;
    const int k = resolved_k(p);
    const float n = (float)(lc - p->n_sink), n_s = n / (float)plan_sample(lc).tile_step;
    const int j = filter_sample_rank((float)k, n, n_s);
    return filter_kept_bound(n, n_s, (float)j + 2.0f) <= 0.9f * (float)filter_cap_for(k);
}

struct WsLayout {
    size_t scores, rho_head, part_acc, part_ml, agg, rho_rank, lse, out_tmp, topk_parts, total;
    size_t f_thr, f_cnt, f_fail, f_nfailed, f_cand;           // the selection's filtered fast path
    int filter_cap;                                           // 0: not laid out
    int64_t ldp;
    int k;
    int max_splits;
};

WsLayout make_layout(const cusa_params* p, int max_seq_len) {
    WsLayout w;
    const int64_t B = p->batch, H = p->n_q_heads;
    const int BG = p->batch * p->n_kv_heads, g = p->n_q_heads / p->n_kv_heads;
    int64_t lc = (int64_t)max_seq_len - p->window;
    if (lc < 1) lc = 1;
    w.ldp = (lc + 63) / 64 * 64;
    w.k = resolved_k(p);
    if (w.k < 1) w.k = 1;
    w.max_splits = max_splits_bound(max_seq_len > p->budget ? max_seq_len : p->budget, BG, g);
    size_t off = 0;
    w.scores = off;    off += align256((size_t)(B * H * w.ldp) * 4);
    w.rho_head = off;  off += align256((size_t)(B * w.k * H) * 4);
    w.part_acc = off;  off += align256((size_t)(B * H * w.max_splits * D) * 4);
    w.part_ml = off;   off += align256((size_t)(B * H * w.max_splits * 2) * 4);
    w.agg = w.rho_rank = off;
    if (p->rank_mode != CUSA_RANK_FIRST_OCCURRENCE) {   // per-position ranking keys and the unified ranked list
        w.agg = off;       off += align256((size_t)(B * 2 * w.ldp) * 4);
        w.rho_rank = off;  off += align256((size_t)(B * (p->budget - p->window + 1)) * 4);
    }
    {   // per-head top-k of few long rows: room for the slices' picks (none when rows are not cut)
        const int lc_i = (int)(lc > 0x7fffffff ? 0x7fffffff : lc);
        const int s1 = plan_topk_slices(B * H, lc_i, w.k);
        size_t n = s1 > 1 ? (size_t)s1 * B * H * w.k : 0;
        const int n_hist = p->budget - p->window - p->n_sink;
        if (p->rank_mode != CUSA_RANK_FIRST_OCCURRENCE && n_hist > 0) {   // one key row per sequence is ranked too
            const int s2 = plan_topk_slices(B, lc_i, n_hist);
            if (s2 > 1 && (size_t)s2 * B * n_hist > n) n = (size_t)s2 * B * n_hist;
        }
        w.topk_parts = off;
        off += align256(n * 8);
    }
    w.filter_cap = 0;
    w.f_thr = w.f_cnt = w.f_fail = w.f_nfailed = w.f_cand = off;
    if (filter_buffers_needed(p, max_seq_len)) {
        w.filter_cap = filter_cap_for(w.k);
        w.f_thr = off;      off += align256((size_t)(B * H) * 4);
        w.f_cnt = off;      off += align256((size_t)(B * H) * 4);
        w.f_fail = off;     off += align256((size_t)(B * H) * 4);
        w.f_nfailed = off;  off += 256;
        w.f_cand = off;     off += align256((size_t)(B * H) * w.filter_cap * 8);
    }
    w.lse = off;      off += align256((size_t)(B * H * 2) * 4);        // recall: denominators over the set and over all tokens
    w.out_tmp = off;  off += align256((size_t)(B * H * D) * 2);        // recall: the attention outputs nobody reads
    w.total = off;
    return w;
}

bool device_ready();

cusa_status check_ws(const WsLayout& w, void* ws, size_t ws_bytes) {
    if (!ws || ((uintptr_t)ws & 255)) return CUSA_ERR_INVALID_ARG;
    if (ws_bytes < w.total) return CUSA_ERR_WORKSPACE_TOO_SMALL;
    return device_ready() ? CUSA_OK : CUSA_ERR_LAUNCH;
}

// The union kernel's bitmap over candidate positions has to fit LDS.
cusa_status check_select_length(const cusa_params* p, const cusa_kv* kv) {
    return (int64_t)kv->max_seq_len - p->window > UNION_MAX_POSITIONS ? CUSA_ERR_UNSUPPORTED : CUSA_OK;
}

template <typename T>
T* ws_ptr(void* ws, size_t off) {
    return reinterpret_cast<T*>(static_cast<char*>(ws) + off);
}

cusa_status launch_status() { return hipGetLastError() == hipSuccess ? CUSA_OK : CUSA_ERR_LAUNCH; }

// ------------------------------------------------------------------ launches

// What a pass over all tokens of a selection layer also emits (scores of the candidate range).
struct ScoreOut {
    float* P = nullptr;     // nullptr: plain attention
    int64_t ldp = 0;
    int window = 0;
    FilterState filter = {};   // thr set: the pass keeps the candidates at or above the heads' thresholds instead of writing P
};

struct AttnArgs {
    bool paged;
    dim3 grid;
    hipStream_t s;
    KvView view;
    const uint16_t* q;
    const int32_t* idx;
    const int32_t* cnt;
    int budget;
    float scale;
    float* pa;
    float* pm;
    uint16_t* out;
    float* lse = nullptr;   // optional: log2 of the softmax denominators, [B][H]
    int n_splits, chunk;
    ScoreOut score;
};

template <int GQ, int TI, bool SPARSE, bool SCORE, bool FILTER = false>
void launch_attn_partial(const AttnArgs& a) {
    const int kid = SPARSE ? KID_ATTN_SPARSE : SCORE ? KID_ATTN_SELECT : KID_ATTN_FULL;
    if (a.paged)
        launch(kid, attn_kernel<GQ, TI, SPARSE, true, SCORE, false, FILTER>, a.grid, ATTN_THREADS, 0, a.s, a.idx, a.cnt, a.view.seq_lens, a.q,
               a.budget, a.n_splits, a.chunk, a.view.G, a.scale, a.pa, a.pm, a.out, a.lse, a.score.P, a.score.ldp, a.score.window, 0, a.score.filter, a.view);
    else
        launch(kid, attn_kernel<GQ, TI, SPARSE, false, SCORE, false, FILTER>, a.grid, ATTN_THREADS, 0, a.s, a.idx, a.cnt, a.view.seq_lens, a.q,
               a.budget, a.n_splits, a.chunk, a.view.G, a.scale, a.pa, a.pm, a.out, a.lse, a.score.P, a.score.ldp, a.score.window, 0, a.score.filter, a.view);
}

// Sparse attention with one token list per query head: grid.y counts query heads.
template <int TI>
void launch_attn_per_head(const AttnArgs& a, int H, int hshift) {
    if (a.paged)
        launch(KID_ATTN_PER_HEAD, attn_kernel<1, TI, true, true, false, true>, a.grid, ATTN_THREADS, 0, a.s, a.idx, a.cnt,
               a.view.seq_lens, a.q, a.budget, a.n_splits, a.chunk, H, a.scale, a.pa, a.pm, a.out, a.lse, nullptr, 0, 0, hshift, FilterState{}, a.view);
    else
        launch(KID_ATTN_PER_HEAD, attn_kernel<1, TI, true, false, false, true>, a.grid, ATTN_THREADS, 0, a.s, a.idx, a.cnt,
               a.view.seq_lens, a.q, a.budget, a.n_splits, a.chunk, H, a.scale, a.pa, a.pm, a.out, a.lse, nullptr, 0, 0, hshift, FilterState{}, a.view);
}

template <int GQ, bool SPARSE>
void launch_attn_ti(int ti, const AttnArgs& a) {
    if constexpr (!SPARSE) {
        if (a.score.P) {                              // the scoring chain repeats work for tiles under 64 tokens: always the wider tile
            if (a.score.filter.thr) {                 // groups of up to 4 only (filtered_select)
                if constexpr (GQ <= 4) {
                    if (ti == 16) launch_attn_partial<GQ, 16, false, true, true>(a);
                    else launch_attn_partial<GQ, 8, false, true, true>(a);
                }
            } else {
                if (ti == 16) launch_attn_partial<GQ, 16, false, true>(a);
                else launch_attn_partial<GQ, 8, false, true>(a);
            }
            return;
        }
    }
    if (ti == 8) {
        launch_attn_partial<GQ, 8, SPARSE, false>(a);
        return;
    }
    launch_attn_partial<GQ, 4, SPARSE, false>(a);
}

// Attention over all tokens (idx == nullptr) or over idx/cnt; n_max bounds the token count.
// With score.P set (all tokens only) the pass also writes the selection scores.
template <bool SPARSE>
cusa_status run_attention(const cusa_params* p, const void* q, const cusa_kv* kv, const int32_t* idx,
                          const int32_t* cnt, int n_max, void* out, void* ws, const WsLayout& w, hipStream_t s,
                          ScoreOut score = ScoreOut(), float* lse = nullptr) {
    const int g = p->n_q_heads / p->n_kv_heads, BG = p->batch * p->n_kv_heads, H = p->n_q_heads;
    const AttnPlan pl = plan_attn(n_max, BG, g, score.P != nullptr);
    if (pl.n_splits > w.max_splits) return CUSA_ERR_WORKSPACE_TOO_SMALL;
    AttnArgs a;
    a.paged = kv->layout == CUSA_KV_PAGED;
    a.grid = dim3(pl.n_splits, p->n_kv_heads, p->batch);
    a.s = s;
    a.view = make_view(p, kv);
    a.q = static_cast<const uint16_t*>(q);
    a.idx = idx;
    a.cnt = cnt;
    a.budget = p->budget;
    a.scale = p->sm_scale * 1.4426950408889634f;
    a.pa = ws_ptr<float>(ws, w.part_acc);
    a.pm = ws_ptr<float>(ws, w.part_ml);
    a.out = static_cast<uint16_t*>(out);
    a.lse = lse;
    a.n_splits = pl.n_splits;
    a.chunk = pl.chunk;
    a.score = score;
    switch (g) {
        case 1: launch_attn_ti<1, SPARSE>(pl.ti, a); break;
        case 2: launch_attn_ti<2, SPARSE>(pl.ti, a); break;
        case 4: launch_attn_ti<4, SPARSE>(pl.ti, a); break;
        default: launch_attn_ti<8, SPARSE>(pl.ti, a); break;
    }
    if (launch_status() != CUSA_OK) return CUSA_ERR_LAUNCH;
    if (pl.n_splits > 1) {
        launch(KID_REDUCE, attn_reduce_kernel, dim3(H, p->batch), 256, 0, s, a.pa, a.pm, a.out, SPARSE ? cnt : kv->seq_lens,
               SPARSE ? p->budget : 0x7fffffff, pl.n_splits, pl.chunk, H, lse);
    }
    return launch_status();
}

// Sparse attention over idx_head [B][H][budget]: every query head is its own "group".
cusa_status run_attention_per_head(const cusa_params* p, const void* q, const cusa_kv* kv, const int32_t* idx_head,
                                   const int32_t* cnt, void* out, void* ws, const WsLayout& w, hipStream_t s,
                                   float* lse = nullptr) {
    const int H = p->n_q_heads, g = H / p->n_kv_heads;
    const int n_max = p->budget < kv->max_seq_len ? p->budget : kv->max_seq_len;
    const AttnPlan pl = plan_attn(n_max, p->batch * H, 1);
    if (pl.n_splits > w.max_splits) return CUSA_ERR_WORKSPACE_TOO_SMALL;
    AttnArgs a;
    a.paged = kv->layout == CUSA_KV_PAGED;
    a.grid = dim3(pl.n_splits, H, p->batch);
    a.s = s;
    a.view = make_view(p, kv);
    a.q = static_cast<const uint16_t*>(q);
    a.idx = idx_head;
    a.cnt = cnt;
    a.budget = p->budget;
    a.scale = p->sm_scale * 1.4426950408889634f;
    a.pa = ws_ptr<float>(ws, w.part_acc);
    a.pm = ws_ptr<float>(ws, w.part_ml);
    a.out = static_cast<uint16_t*>(out);
    a.lse = lse;
    a.n_splits = pl.n_splits;
    a.chunk = pl.chunk;
    const int hshift = g == 1 ? 0 : g == 2 ? 1 : g == 4 ? 2 : 3;
    if (pl.ti == 8) launch_attn_per_head<8>(a, H, hshift);
    else launch_attn_per_head<4>(a, H, hshift);
    if (launch_status() != CUSA_OK) return CUSA_ERR_LAUNCH;
    if (pl.n_splits > 1)
        launch(KID_REDUCE, attn_reduce_kernel, dim3(H, p->batch), 256, 0, s, a.pa, a.pm, a.out, cnt, p->budget, pl.n_splits,
               pl.chunk, H, lse);
    return launch_status();
}

// LDS beyond 48 KB per workgroup has to be granted per kernel and per device.  All kernels that
// can ask for more are granted their maximum once per device, outside any enqueueing work: on the
// first library call made with that device current (cusa_workspace_bytes included), so that later
// calls only enqueue kernels.
constexpr size_t SEL_LDS_MAX = (size_t)UNION_MAX_POSITIONS / 8;   // the selection bitmaps

template <int ITEMS, int MTOP, bool MERGE = false>
constexpr size_t topk_lds_bytes() {
    return ((size_t)MTOP * SEL_THREADS + topk_area_entries(ITEMS, MTOP, MERGE)) * sizeof(uint64_t);
}

bool grant_lds(const void* fn, size_t bytes) {
    if (bytes <= 48 * 1024) return true;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return true;
}

template <int ITEMS, bool MERGE = false>
bool grant_topk_items() {
    return grant_lds(reinterpret_cast<const void*>(topk_kernel<ITEMS, 1, MERGE>), topk_lds_bytes<ITEMS, 1, MERGE>()) &&
           grant_lds(reinterpret_cast<const void*>(topk_kernel<ITEMS, 2, MERGE>), topk_lds_bytes<ITEMS, 2, MERGE>()) &&
           grant_lds(reinterpret_cast<const void*>(topk_kernel<ITEMS, 4, MERGE>), topk_lds_bytes<ITEMS, 4, MERGE>()) &&
           grant_lds(reinterpret_cast<const void*>(topk_kernel<ITEMS, 8, MERGE>), topk_lds_bytes<ITEMS, 8, MERGE>());
}

// Split-K partials of cusa_sparse_attn_noalloc: device memory that belongs to the library image,
// one copy per GPU, held until the process ends.  Host code never uses the array's name as an
// address: the per-device address is asked for once (device_ready) and passed to the kernels.
constexpr size_t NOALLOC_SCRATCH_BYTES = (size_t)8 << 20;
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES] = {nullptr};

// True once the current device's kernels hold their LDS grants.  Without a device (a host that
// only sizes workspaces) nothing is done and false is returned.
template <int GQ>
bool grant_sample() {
    const size_t bytes = sample_lds_bytes(GQ, SAMPLE_MAX_TILES * SCORE_ROWS);
    return grant_lds(reinterpret_cast<const void*>(sample_threshold_kernel<GQ, false>), bytes) &&
           grant_lds(reinterpret_cast<const void*>(sample_threshold_kernel<GQ, true>), bytes);
}

bool device_ready() {
    static std::mutex mu;
    static bool ready[MAX_DEVICES] = {false};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) {
        (void)hipGetLastError();
        return false;
    }
    std::lock_guard<std::mutex> lk(mu);
    if (ready[dev]) return true;
    const bool ok = grant_topk_items<4>() && grant_topk_items<8>() && grant_topk_items<16>() && grant_topk_items<32>() &&
                    grant_topk_items<0>() && grant_topk_items<-1>() && grant_topk_items<4, true>() &&
                    grant_topk_items<8, true>() && grant_topk_items<16, true>() && grant_lds(reinterpret_cast<const void*>(union_kernel), SEL_LDS_MAX) &&
                    grant_lds(reinterpret_cast<const void*>(per_head_rho_kernel), SEL_LDS_MAX) && grant_sample<1>() &&
                    grant_sample<2>() && grant_sample<4>();
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
        (void)hipGetLastError();
        return false;
    }
    g_scratch_ptr[dev] = ptr;
    ready[dev] = ok;
    return ok;
}

// Arguments of one per-head top-k pass.  parts == nullptr: whole rows, ranked output.  Otherwise the
// rows are cut into n_slices slices of slice_len positions (grid.z) that leave their k best in parts,
// and a merge launch ranks among those.
struct TopkArgs {
    dim3 grid;
    hipStream_t s;
    const float* P;
    int64_t ldp;
    const int32_t* seq_lens;
    int32_t* rho_head;
    int H, k, budget, window, raw, n_sink;
    uint64_t* parts;
    int slice_len, n_slices;
    const int32_t* only_rows = nullptr;   // rank only the rows whose flag is set
    FilterState filter = {};              // merge form: rank the candidates the filtered pass kept
};

template <int ITEMS, int MTOP, bool MERGE>
cusa_status launch_topk_m(const TopkArgs& a) {
    const size_t shmem = topk_lds_bytes<ITEMS, MTOP, MERGE>();
    launch(MERGE ? (a.filter.thr ? KID_TOPK_FILTERED : KID_TOPK_MERGE) : a.parts ? KID_TOPK_SLICE : KID_TOPK, topk_kernel<ITEMS, MTOP, MERGE>, a.grid, SEL_THREADS, shmem, a.s, a.P, a.ldp, a.seq_lens, a.rho_head, a.H, a.k,
           a.budget, a.window, a.raw, a.n_sink, a.parts, a.slice_len, a.n_slices, a.only_rows, a.filter);
    return launch_status();
}

// MTOP: composites sorted per thread (MTOP * 1024 >= k), also the number of per-thread
// candidates kept for the lower bound.
template <int ITEMS, bool MERGE = false>
cusa_status launch_topk(const TopkArgs& a) {
    if (a.k <= 1024) return launch_topk_m<ITEMS, 1, MERGE>(a);
    if (a.k <= 2048) return launch_topk_m<ITEMS, 2, MERGE>(a);
    if (a.k <= 4096) return launch_topk_m<ITEMS, 4, MERGE>(a);
    return launch_topk_m<ITEMS, 8, MERGE>(a);
}

// Ranked top-k of every row of P: rows (b, h) of length L_b - W, output rank-major out[b][j][h].
// raw: the rows hold uint32 keys instead of scores.  parts: room for rows * slices * k composites.
cusa_status run_topk(int lc_max, int B, int H, hipStream_t s, const float* P, int64_t ldp, const int32_t* seq_lens,
                     int32_t* out, int k, int budget, int window, int raw, int n_sink, uint64_t* parts,
                     const int32_t* only_rows = nullptr) {
    TopkArgs a = {dim3(H, B), s, P, ldp, seq_lens, out, H, k, budget, window, raw, n_sink, nullptr, 0, 1};
    a.only_rows = only_rows;
    const int n_slices = plan_topk_slices((int64_t)B * H, lc_max, k);
    int n_cand = lc_max;                                  // candidates a workgroup walks
    if (n_slices > 1) {
        a.parts = parts;
        a.n_slices = n_slices;
        a.slice_len = ((lc_max + n_slices - 1) / n_slices + 4095) / 4096 * 4096;
        a.grid = dim3(H, B, n_slices);
        n_cand = a.slice_len;
    }
    const int items = (n_cand + SEL_THREADS - 1) / SEL_THREADS;
    cusa_status st;
    // many more rows than CUs: the lean streamed kernel, two rows at a time per CU
    if ((int64_t)B * H >= 512 && items > 8) st = launch_topk<-1>(a);
    else if (items <= 4) st = launch_topk<4>(a);
    else if (items <= 8) st = launch_topk<8>(a);
    else if (items <= 16) st = launch_topk<16>(a);
    else if (items <= 32) st = launch_topk<32>(a);
    else st = launch_topk<0>(a);
    if (st != CUSA_OK || n_slices == 1) return st;
    a.grid = dim3(H, B);
    const int m_items = (n_slices * k + SEL_THREADS - 1) / SEL_THREADS;   // <= 16 by the plan
    if (m_items <= 4) return launch_topk<4, true>(a);
    if (m_items <= 8) return launch_topk<8, true>(a);
    return launch_topk<16, true>(a);
}

// P = q.K^T over the candidate range: the selection pass in its scores-only form (no V rows, no output).
// only_failed / n_failed: the second chance of the filtered selection scores the flagged heads' groups only.
template <int GQ, int TI>
void launch_scores_only(const AttnArgs& a) {
    if (a.paged)
        launch(KID_SCORE, attn_kernel<GQ, TI, false, true, true, false, false, true>, a.grid, ATTN_THREADS, 0, a.s, a.idx, a.cnt, a.view.seq_lens,
               a.q, a.budget, a.n_splits, a.chunk, a.view.G, a.scale, a.pa, a.pm, a.out, a.lse, a.score.P, a.score.ldp, a.score.window, 0,
               a.score.filter, a.view);
    else
        launch(KID_SCORE, attn_kernel<GQ, TI, false, false, true, false, false, true>, a.grid, ATTN_THREADS, 0, a.s, a.idx, a.cnt, a.view.seq_lens,
               a.q, a.budget, a.n_splits, a.chunk, a.view.G, a.scale, a.pa, a.pm, a.out, a.lse, a.score.P, a.score.ldp, a.score.window, 0,
               a.score.filter, a.view);
}
template <int GQ>
void launch_scores_only_ti(int ti, const AttnArgs& a) {
    if (ti == 16) launch_scores_only<GQ, 16>(a);
    else launch_scores_only<GQ, 8>(a);
}

cusa_status run_score(const cusa_params* p, const void* q, const cusa_kv* kv, float* P, int64_t ldp, hipStream_t s,
                      int32_t* only_failed, int32_t* n_failed) {
    const int g = p->n_q_heads / p->n_kv_heads, BG = p->batch * p->n_kv_heads;
    const int lc_max = kv->max_seq_len - p->window;
    if (lc_max < 1) return CUSA_OK;
    const AttnPlan pl = plan_attn(lc_max, BG, g, true);
    AttnArgs a;
    a.paged = kv->layout == CUSA_KV_PAGED;
    a.grid = dim3(pl.n_splits, p->n_kv_heads, p->batch);
    a.s = s;
    a.view = make_view(p, kv);
    a.q = static_cast<const uint16_t*>(q);
    a.idx = nullptr;
    a.cnt = nullptr;
    a.budget = p->budget;
    a.scale = 0.0f;
    a.pa = a.pm = nullptr;
    a.out = nullptr;
    a.n_splits = pl.n_splits;
    a.chunk = pl.chunk;
    a.score.P = P;
    a.score.ldp = ldp;
    a.score.window = p->window;
    a.score.filter.fail = only_failed;                   // nullptr: every group
    a.score.filter.n_failed = n_failed;
    switch (g) {
        case 1: launch_scores_only_ti<1>(pl.ti, a); break;
        case 2: launch_scores_only_ti<2>(pl.ti, a); break;
        case 4: launch_scores_only_ti<4>(pl.ti, a); break;
        default: launch_scores_only_ti<8>(pl.ti, a); break;
    }
    return launch_status();
}

// scores_ready: P was already written by the layer's attention pass (cusa_decode_step).
// per_head: idx is [B][H][budget], every head keeps its own first K-W picks (head-to-head selection).
cusa_status run_select(const cusa_params* p, const void* q, const cusa_kv* kv, int32_t* idx, int32_t* cnt, void* ws,
                       const WsLayout& w, hipStream_t s, bool scores_ready = false, bool per_head = false,
                       const FilterState* redo = nullptr) {
    const int H = p->n_q_heads, B = p->batch;
    // redo: the filtered fast path has ranked most heads already; only the flagged ones are scored and ranked here
    int32_t* only_failed = redo ? redo->fail : nullptr;
    int32_t* n_failed = redo ? redo->n_failed : nullptr;
    float* P = ws_ptr<float>(ws, w.scores);
    int32_t* rho_head = ws_ptr<int32_t>(ws, w.rho_head);

    if (kv->max_seq_len > p->budget) {            // otherwise no sequence can need scoring
        const int lc_max = kv->max_seq_len - p->window;
        if (!scores_ready) {
            const cusa_status st = run_score(p, q, kv, P, w.ldp, s, only_failed, n_failed);
            if (st != CUSA_OK) return st;
        }
        cusa_status st = run_topk(lc_max, B, H, s, P, w.ldp, kv->seq_lens, rho_head, w.k, p->budget, p->window, 0, p->n_sink,
                                  ws_ptr<uint64_t>(ws, w.topk_parts), only_failed);
        if (st != CUSA_OK) return st;
    }
    {
        // the union's bitmap over candidate positions lives in LDS
        const int lc_max = kv->max_seq_len > p->window ? kv->max_seq_len - p->window : 0;
        const size_t bitmap = ((((size_t)lc_max + 31) / 32) * 4 + 255) & ~(size_t)255;
        const int n_hist = p->budget - p->window - p->n_sink;
        if (!per_head && p->rank_mode != CUSA_RANK_FIRST_OCCURRENCE) {
            // votes / max-score readings: one key per candidate position, the K-W best positions by key
            // (the same ranked top-k kernel, one row per sequence), then the ascending emission
            int32_t* rho_rank = ws_ptr<int32_t>(ws, w.rho_rank);
            if (n_hist > 0 && kv->max_seq_len > p->budget) {
                uint32_t* agg = ws_ptr<uint32_t>(ws, w.agg);
                launch(KID_RANK_AGG, rank_aggregate_kernel, B, SEL_THREADS, 0, s, rho_head, P, w.ldp, kv->seq_lens, agg, w.ldp,
                       H, w.k, p->budget, p->window, p->rank_mode == CUSA_RANK_MAX_SCORE ? 1 : 0, p->n_sink);
                if (launch_status() != CUSA_OK) return CUSA_ERR_LAUNCH;
                const cusa_status st = run_topk(lc_max, B, 1, s, reinterpret_cast<const float*>(agg), 2 * w.ldp, kv->seq_lens,
                                                rho_rank, n_hist, p->budget, p->window, 1, p->n_sink, ws_ptr<uint64_t>(ws, w.topk_parts));
                if (st != CUSA_OK) return st;
            }
            launch(KID_RHO_PER_HEAD, per_head_rho_kernel, dim3(1, B), SEL_THREADS, bitmap, s, rho_rank, kv->seq_lens, idx, cnt, 1,
                   n_hist, p->budget, p->window, p->n_sink);
            return launch_status();
        }
        if (per_head) {
            launch(KID_RHO_PER_HEAD, per_head_rho_kernel, dim3(H, B), SEL_THREADS, bitmap, s, rho_head, kv->seq_lens, idx, cnt, H,
                   w.k, p->budget, p->window, p->n_sink);
            return launch_status();
        }
        launch(KID_UNION, union_kernel, B, SEL_THREADS, bitmap, s, rho_head, kv->seq_lens, idx, cnt, H, w.k, p->budget,
               p->window, p->n_sink);
    }
    return launch_status();
}

template <int GQ>
void launch_sample_threshold_g(const cusa_params* p, const void* q, const cusa_kv* kv, const SamplePlan& sp,
                               const FilterState& f, int k, hipStream_t s) {
    const KvView view = make_view(p, kv);
    const dim3 grid(p->n_kv_heads, p->batch);
    const size_t shmem = sample_lds_bytes(GQ, sp.n_slots);
    const uint16_t* qf = static_cast<const uint16_t*>(q);
    if (kv->layout == CUSA_KV_PAGED)
        launch(KID_SAMPLE_THRESHOLD, sample_threshold_kernel<GQ, true>, grid, SEL_THREADS, shmem, s, qf, p->n_q_heads, k, p->budget,
               p->window, sp.n_slots, f, view);
    else
        launch(KID_SAMPLE_THRESHOLD, sample_threshold_kernel<GQ, false>, grid, SEL_THREADS, shmem, s, qf, p->n_q_heads, k, p->budget,
               p->window, sp.n_slots, f, view);
}
void launch_sample_threshold(const cusa_params* p, const void* q, const cusa_kv* kv, const SamplePlan& sp,
                             const FilterState& f, int k, hipStream_t s) {
    switch (p->n_q_heads / p->n_kv_heads) {           // groups of up to 4 only (filtered_select)
        case 1: launch_sample_threshold_g<1>(p, q, kv, sp, f, k, s); break;
        case 2: launch_sample_threshold_g<2>(p, q, kv, sp, f, k, s); break;
        default: launch_sample_threshold_g<4>(p, q, kv, sp, f, k, s); break;
    }
}

// A selection layer (Alg. 1): full attention for the layer's output and rho from the same q and K.
// The pass over all tokens also writes the scores, so K is read once.
cusa_status run_select_layer(const cusa_params* p, const void* q, const cusa_kv* kv, void* out, int32_t* idx,
                             int32_t* cnt, void* ws, const WsLayout& w, hipStream_t s) {
    ScoreOut score;
    if (kv->max_seq_len > p->budget) {
        score.P = ws_ptr<float>(ws, w.scores);
        score.ldp = w.ldp;
        score.window = p->window;
    }
    if (score.P && w.filter_cap > 0 && filtered_select(p, kv->max_seq_len)) {
        // The filtered fast path: thresholds from a sample, the pass keeps the candidates above them, the
        // top-k ranks among those, and whatever the guess failed for is scored and ranked the ordinary way.
        const int H = p->n_q_heads, B = p->batch;
        FilterState f;
        f.thr = ws_ptr<uint32_t>(ws, w.f_thr);
        f.cand_cnt = ws_ptr<int32_t>(ws, w.f_cnt);
        f.fail = ws_ptr<int32_t>(ws, w.f_fail);
        f.n_failed = ws_ptr<int32_t>(ws, w.f_nfailed);
        f.cand = ws_ptr<uint64_t>(ws, w.f_cand);
        f.cap = w.filter_cap;
        f.n_sink = p->n_sink;
        const SamplePlan sp = plan_sample((int64_t)kv->max_seq_len - p->window);
        launch_sample_threshold(p, q, kv, sp, f, w.k, s);
        if (launch_status() != CUSA_OK) return CUSA_ERR_LAUNCH;
        score.filter = f;
        cusa_status st = run_attention<false>(p, q, kv, nullptr, nullptr, kv->max_seq_len, out, ws, w, s, score);
        if (st != CUSA_OK) return st;
        TopkArgs a = {dim3(H, B), s, nullptr, 0, kv->seq_lens, ws_ptr<int32_t>(ws, w.rho_head), H, w.k, p->budget, p->window, 0,
                      p->n_sink, nullptr, 0, 1};
        a.filter = f;
        const int items = (f.cap + SEL_THREADS - 1) / SEL_THREADS;
        st = items <= 4 ? launch_topk<4, true>(a) : items <= 8 ? launch_topk<8, true>(a) : launch_topk<16, true>(a);
        if (st != CUSA_OK) return st;
        return run_select(p, q, kv, idx, cnt, ws, w, s, false, false, &f);
    }
    cusa_status st = run_attention<false>(p, q, kv, nullptr, nullptr, kv->max_seq_len, out, ws, w, s, score);
    if (st != CUSA_OK) return st;
    return run_select(p, q, kv, idx, cnt, ws, w, s, score.P != nullptr);
}

}  // namespace

// ------------------------------------------------------------------ C ABI

extern "C" {

cusa_status cusa_workspace_bytes(const cusa_params* params, int32_t max_seq_len, size_t* bytes) {
    cusa_status st = check_params(params, true);
    if (st != CUSA_OK) return st;
    if (!bytes || max_seq_len < 1) return CUSA_ERR_INVALID_ARG;
    (void)device_ready();
    *bytes = make_layout(params, max_seq_len).total;
    return CUSA_OK;
}

cusa_status cusa_workspace_layout(const cusa_params* params, int32_t max_seq_len, cusa_ws_layout* layout) {
    cusa_status st = check_params(params, true);
    if (st != CUSA_OK) return st;
    if (!layout || max_seq_len < 1) return CUSA_ERR_INVALID_ARG;
    (void)device_ready();
    const WsLayout w = make_layout(params, max_seq_len);
    layout->scores_offset = w.scores;
    layout->ld_scores = w.ldp;
    layout->rho_head_offset = w.rho_head;
    layout->k = w.k;
    layout->total_bytes = w.total;
    layout->filtered_select = filtered_select(params, max_seq_len) ? 1 : 0;
    layout->second_chance_offset = w.f_nfailed;
    return CUSA_OK;
}

cusa_status cusa_select(const cusa_params* params, const void* q, const cusa_kv* kv, int32_t* idx, int32_t* cnt,
                        void* ws, size_t ws_bytes, void* stream) {
    cusa_status st = check_params(params, true);
    if (st != CUSA_OK) return st;
    if ((st = check_kv(params, kv)) != CUSA_OK) return st;
    if (!q || !idx || !cnt || ((uintptr_t)q & 15)) return CUSA_ERR_INVALID_ARG;
    if ((st = check_select_length(params, kv)) != CUSA_OK) return st;
    const WsLayout w = make_layout(params, kv->max_seq_len);
    if ((st = check_ws(w, ws, ws_bytes)) != CUSA_OK) return st;
    return run_select(params, q, kv, idx, cnt, ws, w, static_cast<hipStream_t>(stream));
}

cusa_status cusa_sparse_attn(const cusa_params* params, const void* q, const cusa_kv* kv, const int32_t* idx,
                             const int32_t* cnt, void* out, void* ws, size_t ws_bytes, void* stream) {
    cusa_status st = check_params(params, true);
    if (st != CUSA_OK) return st;
    if ((st = check_kv(params, kv)) != CUSA_OK) return st;
    if (!q || !idx || !cnt || !out || ((uintptr_t)q & 15)) return CUSA_ERR_INVALID_ARG;
    const WsLayout w = make_layout(params, kv->max_seq_len);
    if ((st = check_ws(w, ws, ws_bytes)) != CUSA_OK) return st;
    const int n_max = params->budget < kv->max_seq_len ? params->budget : kv->max_seq_len;
    return run_attention<true>(params, q, kv, idx, cnt, n_max, out, ws, w, static_cast<hipStream_t>(stream));
}

size_t cusa_noalloc_max_scratch_bytes(void) { return NOALLOC_SCRATCH_BYTES; }

cusa_status cusa_sparse_attn_noalloc(const cusa_params* params, const void* q, const cusa_kv* kv, const int32_t* idx,
                                     const int32_t* cnt, void* out, void* stream) {
    cusa_status st = check_params(params, true);
    if (st != CUSA_OK) return st;
    if ((st = check_kv(params, kv)) != CUSA_OK) return st;
    if (!q || !idx || !cnt || !out || ((uintptr_t)q & 15)) return CUSA_ERR_INVALID_ARG;
    const int n_max = params->budget < kv->max_seq_len ? params->budget : kv->max_seq_len;
    const int g = params->n_q_heads / params->n_kv_heads, BG = params->batch * params->n_kv_heads;
    // only the two partial arrays are laid out, for exactly the splits this launch makes
    WsLayout w = {};
    w.max_splits = plan_attn(n_max, BG, g).n_splits;
    const size_t rows = (size_t)params->batch * params->n_q_heads * w.max_splits;
    w.part_acc = 0;
    w.part_ml = align256(rows * D * 4);
    w.total = w.part_ml + align256(rows * 2 * 4);
    if (w.total > NOALLOC_SCRATCH_BYTES) return CUSA_ERR_UNSUPPORTED;   // beyond the static scratch
    if (!device_ready()) return CUSA_ERR_LAUNCH;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES || !g_scratch_ptr[dev]) return CUSA_ERR_LAUNCH;
    return run_attention<true>(params, q, kv, idx, cnt, n_max, out, g_scratch_ptr[dev], w, static_cast<hipStream_t>(stream));
}

cusa_status cusa_probe_stream_read(const void* src, size_t bytes, void* sink, void* stream) {
    if (!src || !sink || bytes < 16 || ((uintptr_t)src & 15) || ((uintptr_t)sink & 3)) return CUSA_ERR_INVALID_ARG;
    const int64_t n_vec = (int64_t)(bytes / 16);
    int64_t wgs = (n_vec + PROBE_THREADS - 1) / PROBE_THREADS;
    if (wgs > 2048) wgs = 2048;                       // 8 resident workgroups per CU
    launch(KID_PROBE, probe_stream_read_kernel, dim3((unsigned)wgs), PROBE_THREADS, 0, static_cast<hipStream_t>(stream),
           static_cast<const u32x4*>(src), n_vec, static_cast<uint32_t*>(sink));
    return launch_status();
}

cusa_status cusa_probe_traffic(int32_t pattern, const void* src, size_t bytes, void* dst, size_t dst_bytes, void* stream) {
    if (pattern < 0 || pattern > 3 || !src || !dst || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return CUSA_ERR_INVALID_ARG;
    const size_t chunk_bytes = (size_t)PROBE_CHUNK_TILES * 32768;             // 1 MiB read per chunk
    // the gathered tiles come from a region four times their size
    const int64_t n_chunks = (int64_t)(bytes / (pattern == 1 ? 4 * chunk_bytes : chunk_bytes));
    if (n_chunks < 1) return CUSA_ERR_INVALID_ARG;
    // results: 1 KiB per tile, in groups of 512 tiles (four rows of 32768 floats) resp. 16 chunks
    const size_t need = pattern <= 1 ? 16 : (size_t)((n_chunks + 15) / 16) * 16 * PROBE_CHUNK_TILES * 1024;
    if (dst_bytes < need) return CUSA_ERR_INVALID_ARG;
    const dim3 grid((unsigned)(n_chunks < 512 ? n_chunks : 512));              // two workgroups per CU
    hipStream_t s = static_cast<hipStream_t>(stream);
    const u32x4* sp = static_cast<const u32x4*>(src);
    float* dp = static_cast<float*>(dst);
    if (pattern == 0) launch(KID_PROBE_TILES, probe_traffic_kernel<0>, grid, 256, 0, s, sp, dp, n_chunks);
    else if (pattern == 1) launch(KID_PROBE_GATHER, probe_traffic_kernel<1>, grid, 256, 0, s, sp, dp, n_chunks);
    else if (pattern == 2) launch(KID_PROBE_RW_SCATTER, probe_traffic_kernel<2>, grid, 256, 0, s, sp, dp, n_chunks);
    else launch(KID_PROBE_RW_BURST, probe_traffic_kernel<3>, grid, 256, 0, s, sp, dp, n_chunks);
    return launch_status();
}

cusa_status cusa_select_per_head(const cusa_params* params, const void* q, const cusa_kv* kv, int32_t* idx_head,
                                 int32_t* cnt, void* ws, size_t ws_bytes, void* stream) {
    cusa_status st = check_params(params, true);
    if (st != CUSA_OK) return st;
    if ((st = check_kv(params, kv)) != CUSA_OK) return st;
    if (!q || !idx_head || !cnt || ((uintptr_t)q & 15)) return CUSA_ERR_INVALID_ARG;
    if ((st = check_select_length(params, kv)) != CUSA_OK) return st;
    const WsLayout w = make_layout(params, kv->max_seq_len);
    if ((st = check_ws(w, ws, ws_bytes)) != CUSA_OK) return st;
    return run_select(params, q, kv, idx_head, cnt, ws, w, static_cast<hipStream_t>(stream), false, true);
}

cusa_status cusa_sparse_attn_per_head(const cusa_params* params, const void* q, const cusa_kv* kv,
                                      const int32_t* idx_head, const int32_t* cnt, void* out, void* ws,
                                      size_t ws_bytes, void* stream) {
    cusa_status st = check_params(params, true);
    if (st != CUSA_OK) return st;
    if ((st = check_kv(params, kv)) != CUSA_OK) return st;
    if (!q || !idx_head || !cnt || !out || ((uintptr_t)q & 15)) return CUSA_ERR_INVALID_ARG;
    const WsLayout w = make_layout(params, kv->max_seq_len);
    if ((st = check_ws(w, ws, ws_bytes)) != CUSA_OK) return st;
    return run_attention_per_head(params, q, kv, idx_head, cnt, out, ws, w, static_cast<hipStream_t>(stream));
}

cusa_status cusa_attention_recall(const cusa_params* params, const void* q, const cusa_kv* kv, const int32_t* idx,
                                  const int32_t* cnt, int32_t idx_per_head, float* recall, void* ws, size_t ws_bytes,
                                  void* stream) {
    cusa_status st = check_params(params, true);
    if (st != CUSA_OK) return st;
    if ((st = check_kv(params, kv)) != CUSA_OK) return st;
    if (!q || !idx || !cnt || !recall || ((uintptr_t)q & 15)) return CUSA_ERR_INVALID_ARG;
    const WsLayout w = make_layout(params, kv->max_seq_len);
    if ((st = check_ws(w, ws, ws_bytes)) != CUSA_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int n = params->batch * params->n_q_heads;
    float* lse_set = ws_ptr<float>(ws, w.lse);
    float* lse_all = lse_set + n;
    void* out_tmp = ws_ptr<uint16_t>(ws, w.out_tmp);
    const int n_max = params->budget < kv->max_seq_len ? params->budget : kv->max_seq_len;
    if (idx_per_head) st = run_attention_per_head(params, q, kv, idx, cnt, out_tmp, ws, w, s, lse_set);
    else st = run_attention<true>(params, q, kv, idx, cnt, n_max, out_tmp, ws, w, s, ScoreOut(), lse_set);
    if (st != CUSA_OK) return st;
    st = run_attention<false>(params, q, kv, nullptr, nullptr, kv->max_seq_len, out_tmp, ws, w, s, ScoreOut(), lse_all);
    if (st != CUSA_OK) return st;
    launch(KID_RECALL, recall_kernel, (n + 255) / 256, 256, 0, s, lse_set, lse_all, recall, n);
    return launch_status();
}

cusa_status cusa_full_attn(const cusa_params* params, const void* q, const cusa_kv* kv, void* out, void* ws,
                           size_t ws_bytes, void* stream) {
    cusa_status st = check_params(params, true);
    if (st != CUSA_OK) return st;
    if ((st = check_kv(params, kv)) != CUSA_OK) return st;
    if (!q || !out || ((uintptr_t)q & 15)) return CUSA_ERR_INVALID_ARG;
    const WsLayout w = make_layout(params, kv->max_seq_len);
    if ((st = check_ws(w, ws, ws_bytes)) != CUSA_OK) return st;
    return run_attention<false>(params, q, kv, nullptr, nullptr, kv->max_seq_len, out, ws, w,
                                static_cast<hipStream_t>(stream));
}

cusa_status cusa_select_layer(const cusa_params* params, const void* q, const cusa_kv* kv, void* out, int32_t* idx,
                              int32_t* cnt, void* ws, size_t ws_bytes, void* stream) {
    cusa_status st = check_params(params, true);
    if (st != CUSA_OK) return st;
    if ((st = check_kv(params, kv)) != CUSA_OK) return st;
    if (!q || !out || !idx || !cnt || ((uintptr_t)q & 15)) return CUSA_ERR_INVALID_ARG;
    if ((st = check_select_length(params, kv)) != CUSA_OK) return st;
    const WsLayout w = make_layout(params, kv->max_seq_len);
    if ((st = check_ws(w, ws, ws_bytes)) != CUSA_OK) return st;
    return run_select_layer(params, q, kv, out, idx, cnt, ws, w, static_cast<hipStream_t>(stream));
}

cusa_status cusa_decode_step(const cusa_params* params, int32_t n_layers, const int32_t* layer_kind,
                             const void* const* q_layers, const cusa_kv* kv_layers, void* const* out_layers,
                             int32_t* idx, int32_t* cnt, void* ws, size_t ws_bytes, void* stream) {
    cusa_status st = check_params(params, true);
    if (st != CUSA_OK) return st;
    if (n_layers < 1 || !layer_kind || !q_layers || !kv_layers || !out_layers || !idx || !cnt)
        return CUSA_ERR_INVALID_ARG;
    int max_len = 0;
    bool have_rho = false;
    for (int i = 0; i < n_layers; ++i) {
        if ((st = check_kv(params, &kv_layers[i])) != CUSA_OK) return st;
        if (!q_layers[i] || !out_layers[i] || ((uintptr_t)q_layers[i] & 15)) return CUSA_ERR_INVALID_ARG;
        if (kv_layers[i].max_seq_len > max_len) max_len = kv_layers[i].max_seq_len;
        switch (layer_kind[i]) {
            case CUSA_LAYER_FULL: break;
            case CUSA_LAYER_SELECT:
                if ((st = check_select_length(params, &kv_layers[i])) != CUSA_OK) return st;
                have_rho = true;
                break;
            case CUSA_LAYER_SPARSE:
                if (!have_rho) return CUSA_ERR_INVALID_ARG;
                break;
            default: return CUSA_ERR_INVALID_ARG;
        }
    }
    const WsLayout w = make_layout(params, max_len);
    if ((st = check_ws(w, ws, ws_bytes)) != CUSA_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (int i = 0; i < n_layers; ++i) {
        const cusa_kv* kv = &kv_layers[i];
        if (layer_kind[i] == CUSA_LAYER_SPARSE) {
            const int n_max = params->budget < kv->max_seq_len ? params->budget : kv->max_seq_len;
            st = run_attention<true>(params, q_layers[i], kv, idx, cnt, n_max, out_layers[i], ws, w, s);
        } else if (layer_kind[i] == CUSA_LAYER_SELECT) {
            st = run_select_layer(params, q_layers[i], kv, out_layers[i], idx, cnt, ws, w, s);
        } else {
            st = run_attention<false>(params, q_layers[i], kv, nullptr, nullptr, kv->max_seq_len, out_layers[i], ws, w, s);
        }
        if (st != CUSA_OK) return st;
    }
    return CUSA_OK;
}

#ifndef CUSA_BUILD_ID
#define CUSA_BUILD_ID "unknown"
#endif
// The marker also lets a loader read the id from the file without mapping the library.
static const char kBuildId[] = "CUSA_BUILD_ID=" CUSA_BUILD_ID;
const char* cusa_build_id(void) { return kBuildId + 14; }

const char* cusa_strerror(cusa_status status) {
    switch (status) {
        case CUSA_OK: return "ok";
        case CUSA_ERR_INVALID_ARG: return "invalid argument";
        case CUSA_ERR_UNSUPPORTED: return "unsupported configuration";
        case CUSA_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case CUSA_ERR_LAUNCH: return "kernel launch failed";
    }
    return "unknown status";
}

int32_t cusa_profile_num_kernels(void) { return KID_COUNT; }

const char* cusa_profile_kernel_name(int32_t id) { return (id >= 0 && id < KID_COUNT) ? kKernelNames[id] : ""; }

void cusa_profile_enable(int32_t on) {
    std::lock_guard<std::mutex> lk(g_prof.mu);
    g_prof.on.store(on != 0, std::memory_order_release);
}

static void prof_drain_locked() {
    for (const ProfRec& r : g_prof.recs) {
        float ms = 0.0f;
        if (hipEventSynchronize(r.stop) == hipSuccess && hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
            g_prof.calls[r.id] += 1;
            g_prof.ms[r.id] += ms;
        }
        g_prof.pool.push_back(r.start);
        g_prof.pool.push_back(r.stop);
    }
    g_prof.recs.clear();
}

void cusa_profile_reset(void) {
    std::lock_guard<std::mutex> lk(g_prof.mu);
    prof_drain_locked();
    for (int i = 0; i < KID_COUNT; ++i) {
        g_prof.calls[i] = 0;
        g_prof.ms[i] = 0.0;
    }
}

cusa_status cusa_profile_read(int32_t n, int64_t* calls, double* total_ms) {
    if (n < 0 || !calls || !total_ms) return CUSA_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(g_prof.mu);
    prof_drain_locked();
    for (int i = 0; i < n && i < KID_COUNT; ++i) {
        calls[i] = g_prof.calls[i];
        total_ms[i] = g_prof.ms[i];
    }
    return CUSA_OK;
}

}  // extern "C"
