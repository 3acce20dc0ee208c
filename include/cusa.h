/*
 * libcusa -- decode-time hot path of Cross-Head Unified Sparse Attention (CUSA,
 * "LessIsMore", arXiv 2508.07101) for AMD MI355X (gfx950).
 *
 * One decode step of the attention part of the paper's Alg. 1: full attention
 * layers, a token-selection layer that turns per-head top-k picks into ONE
 * token set rho shared by all heads (Sec. 3.2) plus a recency window (Sec. 3.3),
 * and sparse-attention layers that reuse rho (Sec. 3.1, 3.4).
 *
 * Conventions for every entry point
 *  - "host" pointers are read during the call and may be freed afterwards;
 *    "device" pointers are GPU memory owned by the caller and must stay valid
 *    until the work enqueued on `stream` has finished.
 *  - Calls only ENQUEUE kernels on `stream` (a hipStream_t passed as void*,
 *    NULL = the default stream).  They never allocate, free or synchronise, so
 *    a caller may capture them into a HIP graph.  One exception, once per
 *    device: the first library call made with a device current sets that
 *    device's kernel attributes (LDS limits) and looks up the library's own
 *    device symbols -- host-side calls that enqueue nothing.  Every caller
 *    sizes its workspace with cusa_workspace_bytes before anything else, and
 *    that call does this set-up; a capture therefore never sees it, provided
 *    cusa_workspace_bytes has run on that device beforehand.
 *  - The per-kernel timing facility at the end of this header is the other
 *    exception: while it is enabled the library creates HIP events and keeps
 *    host-side records, so it must be off under graph capture.
 *  - Argument errors are detected on the host before anything is enqueued and
 *    returned as a cusa_status; no C++ exception crosses this boundary.  A
 *    failed kernel launch returns CUSA_ERR_LAUNCH.
 *  - q, K, V and outputs are bf16 (IEEE-like, 8-bit exponent, 8-bit
 *    significand); scores and softmax run in binary32; indices are int32.
 *  - head_dim must be 128; n_q_heads / n_kv_heads (the GQA group g) must be
 *    1, 2, 4 or 8; a paged cache must use 16-token pages.
 */
#ifndef CUSA_H
#define CUSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CUSA_OK = 0,
    CUSA_ERR_INVALID_ARG = 1,        /* NULL pointer, bad shape, inconsistent sizes        */
    CUSA_ERR_UNSUPPORTED = 2,        /* valid request this build has no kernel for         */
    CUSA_ERR_WORKSPACE_TOO_SMALL = 3,
    CUSA_ERR_LAUNCH = 4              /* the HIP runtime refused a launch                   */
} cusa_status;

/* Layer kinds of Alg. 1's per-layer branch. */
typedef enum { CUSA_LAYER_FULL = 0, CUSA_LAYER_SELECT = 1, CUSA_LAYER_SPARSE = 2 } cusa_layer_kind;

typedef enum { CUSA_KV_CONTIGUOUS = 0, CUSA_KV_PAGED = 1 } cusa_kv_layout;

/* Reading of "globally ranked" in Sec. 3.2 (the paper names no ranking key).
 * FIRST_OCCURRENCE (the default reading): flatten the per-head ranked lists
 * rank-major (all rank-0 picks in head order, then all rank-1 picks, ...), drop
 * repeats, keep the first K-W tokens.
 * VOTES: rank the distinct picks by the number of heads proposing them
 * (descending), then by the best rank any head gave them, then by position.
 * MAX_SCORE: rank them by the largest score among the proposing heads
 * (descending), then by position.  Both keep the first K-W of that order. */
typedef enum { CUSA_RANK_FIRST_OCCURRENCE = 0, CUSA_RANK_VOTES = 1, CUSA_RANK_MAX_SCORE = 2 } cusa_rank_mode;

/* Problem statement of Alg. 1 (its inputs: the token budget and the recency ratio), host memory. */
typedef struct {
    int32_t batch;          /* B sequences, each with its own rho                              */
    int32_t n_q_heads;      /* H                                                               */
    int32_t n_kv_heads;     /* G, divides H                                                    */
    int32_t head_dim;       /* d = 128                                                         */
    int32_t budget;         /* K: tokens attended by a sparse layer, window included           */
    int32_t window;         /* W = K*r most recent tokens always kept, 0 <= W <= K             */
    int32_t topk_per_head;  /* k picks proposed per head; 0 means K-W; K-W-n_sink <= k <= 8192 */
    int32_t n_sink;         /* attention sinks (Sec. 4.1 reserves four): the first n_sink       */
                            /* positions are always in rho, inside the budget; 0 <= n_sink <= K-W */
    int32_t rank_mode;      /* cusa_rank_mode                                                  */
    float   sm_scale;       /* softmax scale of Eq. 1, normally 1/sqrt(d)                      */
} cusa_params;

/* One layer's KV cache view, host memory; the pointers inside are device memory.
 * contiguous: element (b, kv, t, i) of K is k[b*stride_batch + kv*stride_head +
 *             t*stride_token + i] (strides in elements, stride_token >= 128 and a
 *             multiple of 8 so rows are 16-byte aligned); V uses the same strides.
 * paged:      pools are [n_pages][n_kv_heads][page_size][128]; logical token t of
 *             sequence b lives in pool page block_table[b*max_pages + t/page_size],
 *             slot t % page_size.
 * seq_lens[b] = L_b >= 1 counts the token appended in this step (Alg. 1 appends
 * before attending); max_seq_len is a host-side bound L_b <= max_seq_len used
 * to size grids and workspace. */
typedef struct {
    const void*    k;
    const void*    v;
    int32_t        layout;          /* cusa_kv_layout */
    int64_t        stride_batch, stride_head, stride_token;
    const int32_t* block_table;     /* device, [batch][max_pages]; paged only */
    int32_t        max_pages;
    int32_t        page_size;       /* 16 */
    int64_t        n_pages;
    const int32_t* seq_lens;        /* device, [batch] */
    int32_t        max_seq_len;
} cusa_kv;

/* Where the selection intermediates live inside the workspace after cusa_select
 * (byte offsets from the workspace base), so that a test can read them back:
 *   scores    float  [batch][n_q_heads][ld_scores]   P = q.K^T over [0, L_b-W)
 *   rho_head  int32  [batch][k][n_q_heads]           ranked picks, RANK-MAJOR:
 *             entry (b, j, h) is head h's rank-j pick; valid for j < min(k, L_b-W)
 * Both are defined only for sequences with L_b > K; scores also depends on filtered_select below.
 * (With rank_mode VOTES or
 * MAX_SCORE the workspace also holds one ranking key per candidate position and the
 * unified ranked list; they are internal.) */
typedef struct {
    size_t  scores_offset;
    int64_t ld_scores;
    size_t  rho_head_offset;
    int32_t k;                      /* topk_per_head after resolving 0 -> K-W */
    size_t  total_bytes;
    int32_t filtered_select;        /* 1: a selection LAYER of this size (cusa_select_layer, a SELECT layer of
                                       cusa_decode_step) keeps only the scores that can reach a head's top-k
                                       and writes no score array; `scores` is then defined after cusa_select
                                       only.  rho_head, idx and cnt are the same either way. */
    size_t  second_chance_offset;   /* filtered_select = 1: an int32 there holds, after such a layer, how many
                                       heads' thresholds failed and were scored and ranked again (a
                                       diagnostic: the result does not depend on it) */
} cusa_ws_layout;

/* Bytes of device workspace any of the calls below needs for `params` and
 * sequences up to max_seq_len.  Workspace must be 256-byte aligned; its content
 * need not be preserved between calls.  Error: INVALID_ARG. */
cusa_status cusa_workspace_bytes(const cusa_params* params, int32_t max_seq_len, size_t* bytes);
cusa_status cusa_workspace_layout(const cusa_params* params, int32_t max_seq_len, cusa_ws_layout* layout);

/* Token selection of a selection layer (Alg. 1, the lines that build rho;
 * Sec. 3.2 and 3.3).  For each sequence b with L = seq_lens[b]:
 *   L <= K : rho = {0 .. L-1}
 *   else   : P = q.K^T (unscaled, binary32, summed left to right over d) for
 *            tokens [0, L-W); every head ranks its min(k, L-W-n_sink) best tokens
 *            of [n_sink, L-W) by (score descending, position ascending); the
 *            ranked lists are unified per rank_mode and the first K-W-n_sink
 *            distinct tokens kept; the n_sink first and the W last positions
 *            are added.
 * q    device bf16 [batch][n_q_heads][128], this layer's query.
 * idx  device int32 [batch][budget]: rho ascending; entries >= cnt[b] unspecified.
 * cnt  device int32 [batch]: |rho| = min(K, L_b).
 * Errors: INVALID_ARG, UNSUPPORTED (max_seq_len - W above 1 179 648,
 * the positions the selection's on-chip bitmap covers), WORKSPACE_TOO_SMALL, LAUNCH. */
cusa_status cusa_select(const cusa_params* params, const void* q, const cusa_kv* kv,
                        int32_t* idx, int32_t* cnt, void* ws, size_t ws_bytes, void* stream);

/* SparseAttention(q, C[rho]) of Alg. 1: Eq. 1 restricted to the positions
 * idx[b][0 .. cnt[b]) (the same set for every head), on this layer's own K/V.
 * idx entries must lie in [0, seq_lens[b]); cnt[b] in [1, budget].
 * out  device bf16 [batch][n_q_heads][128]. */
cusa_status cusa_sparse_attn(const cusa_params* params, const void* q, const cusa_kv* kv,
                             const int32_t* idx, const int32_t* cnt, void* out,
                             void* ws, size_t ws_bytes, void* stream);

/* cusa_sparse_attn for callers that cannot allocate device memory or hand over a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * kernels and the same result bit for bit, with the split-K partials in a static device array
 * that is part of the library image (cusa_noalloc_max_scratch_bytes() bytes per GPU the library
 * runs on, held until the process ends).  Arguments as cusa_sparse_attn, minus the workspace.
 * Allocates nothing, frees nothing, synchronises nothing.
 * Errors: as cusa_sparse_attn; UNSUPPORTED when the partials of this problem (batch * n_q_heads *
 * splits * 520 bytes, splits as the launch plan cuts min(budget, max_seq_len) tokens) do not fit
 * the array.  All calls on one GPU share that GPU's array: calls whose kernels may overlap (two
 * streams, two threads) race on it and must be serialised by the caller. */
size_t      cusa_noalloc_max_scratch_bytes(void);
cusa_status cusa_sparse_attn_noalloc(const cusa_params* params, const void* q, const cusa_kv* kv,
                                     const int32_t* idx, const int32_t* cnt, void* out, void* stream);

/* Head-to-head selection and its sparse attention: the per-head variant the paper
 * compares CUSA with (Sec. 3.2 and the generalization figure; the per-head-index
 * kernel of the kernel-metrics table).  Every head keeps its OWN token set: its
 * first K-W ranked picks (same scores and ranking as cusa_select) plus the last W
 * positions; L <= K: all tokens.
 * idx_head  device int32 [batch][n_q_heads][budget]: each head's set, ascending.
 * cnt       device int32 [batch]: min(K, L_b), the size of every head's set.
 * cusa_sparse_attn_per_head is Eq. 1 restricted, for head h, to idx_head[b][h][0 .. cnt[b]);
 * nothing is shared inside a GQA group, each head loads its own K/V rows.
 * Errors as cusa_select / cusa_sparse_attn. */
cusa_status cusa_select_per_head(const cusa_params* params, const void* q, const cusa_kv* kv,
                                 int32_t* idx_head, int32_t* cnt, void* ws, size_t ws_bytes, void* stream);
cusa_status cusa_sparse_attn_per_head(const cusa_params* params, const void* q, const cusa_kv* kv,
                                      const int32_t* idx_head, const int32_t* cnt, void* out,
                                      void* ws, size_t ws_bytes, void* stream);

/* Attention recall of Eq. 3 for a given token set: recall[b][h] = (softmax mass of head h
 * on the set) / (its mass on all L_b tokens) = sum_{t in set} exp(s_t) / sum_{t < L_b} exp(s_t)
 * with s_t = sm_scale * q_h.k_t.  Two attention passes (over the set, over all tokens) keep
 * their softmax denominators; a diagnostic, not a step of Alg. 1.
 * idx, cnt      as in cusa_sparse_attn (idx_per_head = 0) or as in
 *               cusa_sparse_attn_per_head (idx_per_head = 1).
 * recall        device float [batch][n_q_heads]. */
cusa_status cusa_attention_recall(const cusa_params* params, const void* q, const cusa_kv* kv,
                                  const int32_t* idx, const int32_t* cnt, int32_t idx_per_head,
                                  float* recall, void* ws, size_t ws_bytes, void* stream);

/* FullAttention(q, C[:]) of Alg. 1 (Eq. 1 over all L_b tokens); also the
 * baseline the sparse path is compared with.  budget, window and topk_per_head
 * do not enter the result, but params is validated as a whole (so they must
 * still be consistent) and sizes the workspace.  out as in cusa_sparse_attn. */
cusa_status cusa_full_attn(const cusa_params* params, const void* q, const cusa_kv* kv,
                           void* out, void* ws, size_t ws_bytes, void* stream);

/* A selection layer in one call (the selection branch of Alg. 1): out = FullAttention(q, C[:])
 * and rho = the selection of cusa_select, from one pass over K (the pass that computes the
 * output also writes the scores -- or, for a layer with many scores, only those above a
 * per-head threshold guessed from a sample; heads whose guess fails are scored and ranked again,
 * so the result does not depend on it: cusa_ws_layout.filtered_select).  idx and cnt as in
 * cusa_select (bit for bit the same rho);
 * out as in cusa_full_attn up to binary32 rounding order.  This is what cusa_decode_step runs
 * for a SELECT layer; a caller that drives the layers itself uses it instead of
 * cusa_full_attn followed by cusa_select, which read K twice. */
cusa_status cusa_select_layer(const cusa_params* params, const void* q, const cusa_kv* kv, void* out,
                              int32_t* idx, int32_t* cnt, void* ws, size_t ws_bytes, void* stream);

/* Attention part of one decode step of Alg. 1 over n_layers layers.
 * layer_kind  host int32[n_layers] of cusa_layer_kind.  FULL: full attention.
 *             SELECT: full attention for this layer's output, then rho is rebuilt
 *             from this layer's q and K (the scores P are written by the same pass
 *             over K that computes the output, bit for bit those of cusa_select;
 *             the output agrees with cusa_full_attn up to binary32 rounding order).
 *             SPARSE: sparse attention over the current rho.  A SPARSE layer with no SELECT layer before it in this
 *             call is INVALID_ARG (Alg. 1 starts with rho empty).
 * q_layers    host array of n_layers device pointers, each bf16 [batch][H][128].
 * kv_layers   host array of n_layers cache views.
 * out_layers  host array of n_layers device pointers, each bf16 [batch][H][128].
 * idx, cnt    device, as in cusa_select; hold the latest rho on return. */
cusa_status cusa_decode_step(const cusa_params* params, int32_t n_layers, const int32_t* layer_kind,
                             const void* const* q_layers, const cusa_kv* kv_layers,
                             void* const* out_layers, int32_t* idx, int32_t* cnt,
                             void* ws, size_t ws_bytes, void* stream);

const char* cusa_strerror(cusa_status status);

/* Digest of the sources this binary was compiled from (16 hex digits); a loader compares it
 * with the sources it sees to tell a stale binary. */
const char* cusa_build_id(void);

/* ---- per-kernel timing (benchmark support; not part of the method) ---------
 * While enabled, every kernel the library enqueues is launched with a start and a
 * stop event that the runtime fills from the dispatch's own begin and end time
 * stamps (hipExtLaunchKernelGGL), i.e. the duration a kernel trace reports.
 * cusa_profile_read waits for those events and returns, for kernel id i < n, the
 * number of launches and the summed milliseconds since the last reset.  Enabling
 * costs host time per launch and creates events, so it must not be on under graph
 * capture.  cusa_profile_num_kernels returns the number of kernel ids.
 * The facility holds process-wide state behind a mutex (event pool, pending records, totals);
 * with it off the library keeps no state beyond the once-per-device set-up described above. */
int32_t     cusa_profile_num_kernels(void);
const char* cusa_profile_kernel_name(int32_t id);
void        cusa_profile_enable(int32_t on);
void        cusa_profile_reset(void);
cusa_status cusa_profile_read(int32_t n, int64_t* calls, double* total_ms);

/* Streaming-read probe (benchmark support; not part of the method): enqueues one kernel that
 * reads `bytes` bytes (a multiple of 16 is read; at least 16) of device memory `src` (16-byte
 * aligned) with plain coalesced 16-byte loads and folds them; `sink` is 4 bytes of device memory
 * the kernel may write.  Timed through the facility above (kernel "probe_stream_read_kernel"),
 * it gives the read rate a pure streaming pass reaches on the machine -- the practical ceiling
 * beside the nominal HBM peak.  Errors: INVALID_ARG, LAUNCH. */
cusa_status cusa_probe_stream_read(const void* src, size_t bytes, void* sink, void* stream);

/* Traffic probes (benchmark support): one kernel with the memory access pattern of an attention
 * kernel and none of its arithmetic; a wave reads 32 KiB tiles with 32 loads of 16 bytes per lane
 * in flight (streaming loads, as the attention kernels use for K and V).  pattern 0: nothing else, a
 * plain streaming read of `bytes`.  pattern 1: the tiles are 256-byte rows gathered, ascending with irregular gaps, from a
 * region four times their size (what sparse attention reads; bytes / 4 are read).  pattern 2:
 * streams `bytes` and writes 1/32 of that volume as 256-byte runs right away (a scoring pass that
 * stores every tile's scores).  pattern 3: streams `bytes` and writes the same volume in workgroup
 * bursts of 32 KiB.  src: device, 16-byte aligned, `bytes` (at least 1 MiB; 4 MiB for pattern 1;
 * whole MiB are used).  dst: device, 16-byte aligned, at least bytes / 32 + 512 KiB for patterns 2
 * and 3 (16 bytes for patterns 0 and 1).  Timed through the profiling facility (kernels
 * "probe_traffic_kernel<...>").  Errors: INVALID_ARG, LAUNCH. */
cusa_status cusa_probe_traffic(int32_t pattern, const void* src, size_t bytes, void* dst, size_t dst_bytes,
                               void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CUSA_H */
