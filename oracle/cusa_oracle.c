/*
 * CPU oracle for the decode-time hot path of Cross-Head Unified Sparse
 * Attention (CUSA): token selection at a selection layer and attention over
 * the selected set.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, by-eye-checkable
 * statement of what the paper's method computes.  Only the test-suite, the
 * smoke check and the benchmark's cpu_baseline leg may call it; the product
 * library never does, and the two share no code.
 *
 * Notation follows the paper: L context length (current token included),
 * H query heads, G key/value heads, g = H/G, d head dimension, K token
 * budget, W = K*r recency window, k per-head top-k, rho the selected set.
 *
 * All K/V/q values are bf16 bit patterns (uint16_t), row-major, logical view
 * of ONE sequence: q[H][d], Kc[G][L][d], Vc[G][L][d].
 *
 * Pins (see tests, all CPU): dense attention against an independent float64
 * softmax(QK^T/sqrt(d))V; scores against a scalar float32 re-derivation and the
 * float64 dot product; per-head top-k against a stable full sort; the union
 * against a dictionary brute force and the structural invariants of Alg. 1.
 * The CHOICE among the global-ranking readings (rank_mode) is
 * "parity unpinned": the paper prints no worked example that fixes it.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- bf16 <-> binary32/binary64 ---------------------------------------- */

static float bf16_to_f32(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Round a double to the nearest bf16 (8 significand bits), ties to even, in
 * one rounding.  Subnormal bf16 results are not produced by this path's
 * outputs; they are flushed to signed zero. */
static uint16_t f64_to_bf16_rne(double x) {
    if (isnan(x)) return 0x7fc0;
    if (isinf(x)) return x > 0 ? 0x7f80 : 0xff80;
    if (x == 0.0) return signbit(x) ? 0x8000 : 0x0000;
    int e;
    double m = frexp(x, &e);          /* x = m * 2^e, 0.5 <= |m| < 1       */
    double r = nearbyint(ldexp(m, 8)); /* 8 significant bits, RNE (default) */
    float f = (float)ldexp(r, e - 8); /* exact in binary32                 */
    if (isinf(f)) return x > 0 ? 0x7f80 : 0xff80;
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if (((u >> 23) & 0xff) == 0) return (uint16_t)((u >> 16) & 0x8000);
    return (uint16_t)(u >> 16);
}

int cusa_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- paged cache view --------------------------------------------------- */

/* Materialise one sequence's logical [G][L][d] view from a paged pool laid
 * out [n_pages][G][page_size][d]; block_table[p] is the pool page holding
 * logical tokens p*page_size .. p*page_size+page_size-1. */
void cusa_oracle_resolve_paged(const uint16_t *pool, const int32_t *block_table,
                               int G, int page_size, int d, int L,
                               uint16_t *out) {
    for (int kv = 0; kv < G; ++kv)
        for (int t = 0; t < L; ++t) {
            int64_t page = block_table[t / page_size];
            int64_t src = ((page * G + kv) * page_size + t % page_size) * (int64_t)d;
            int64_t dst = ((int64_t)kv * L + t) * d;
            memcpy(out + dst, pool + src, sizeof(uint16_t) * (size_t)d);
        }
}

/* ---- Alg. 1, selection layer: P := q . C.K^T ----------------------------- */

/* P[h][t] for t in [0, Lc): the UNSCALED query-key product of head h with
 * key t of its KV head (h / g).  binary32, accumulated left to right over
 * the head dimension:  acc = 0;  acc = fl(acc + q_i * k_i), i = 0..d-1.
 * A bf16*bf16 product has a 16-bit significand and is exact in binary32, so
 * the only rounding is the one per addition.  P has row stride ldp. */
void cusa_oracle_scores(const uint16_t *q, const uint16_t *Kc, int H, int G,
                        int d, int L, int Lc, float *P, int64_t ldp) {
    int g = H / G;
#pragma omp parallel for schedule(static)
    for (int h = 0; h < H; ++h) {
        const uint16_t *qh = q + (int64_t)h * d;
        const uint16_t *Kh = Kc + (int64_t)(h / g) * L * d;
        for (int t = 0; t < Lc; ++t) {
            const uint16_t *kt = Kh + (int64_t)t * d;
            float acc = 0.0f;
            for (int i = 0; i < d; ++i) {
                float p = bf16_to_f32(qh[i]) * bf16_to_f32(kt[i]);
                acc = acc + p;
            }
            P[(int64_t)h * ldp + t] = acc;
        }
    }
}

/* ---- Sec. 3.2 / Alg. 1: per-head TopKIndices ------------------------------ */

typedef struct {
    float s;
    int32_t pos;
} scored_t;

/* Larger score first; equal scores (+0 and -0 are equal): lower position first. */
static int cmp_scored(const void *a, const void *b) {
    const scored_t *x = (const scored_t *)a, *y = (const scored_t *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->pos > y->pos) - (x->pos < y->pos);
}

/* rho_head[h][j], j = 0..k_eff-1: positions of the k_eff best candidates of
 * head h among [0, Lc), rank 0 = best.  The caller passes k_eff = min(k, Lc). */
void cusa_oracle_topk(const float *P, int64_t ldp, int H, int Lc, int k_eff,
                      int32_t *rho_head) {
#pragma omp parallel for schedule(dynamic)
    for (int h = 0; h < H; ++h) {
        scored_t *a = (scored_t *)malloc(sizeof(scored_t) * (size_t)(Lc > 0 ? Lc : 1));
        for (int t = 0; t < Lc; ++t) {
            a[t].s = P[(int64_t)h * ldp + t];
            a[t].pos = t;
        }
        qsort(a, (size_t)Lc, sizeof(scored_t), cmp_scored);
        for (int j = 0; j < k_eff; ++j) rho_head[(int64_t)h * k_eff + j] = a[j].pos;
        free(a);
    }
}

/* ---- Alg. 1: UnionFlatten, global rank, prefix, Recent ------------------- */

typedef struct {
    int32_t pos;
    int32_t votes;      /* number of heads proposing the token            */
    int32_t best_rank;  /* smallest per-head rank among the proposals     */
    float max_score;    /* largest P[h][pos] among the proposing heads    */
} cand_t;

static int cmp_votes(const void *a, const void *b) {
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->votes != y->votes) return y->votes - x->votes;
    if (x->best_rank != y->best_rank) return x->best_rank - y->best_rank;
    return (x->pos > y->pos) - (x->pos < y->pos);
}

static int cmp_maxscore(const void *a, const void *b) {
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->max_score > y->max_score) return -1;
    if (x->max_score < y->max_score) return 1;
    return (x->pos > y->pos) - (x->pos < y->pos);
}

static int cmp_i32(const void *a, const void *b) {
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* Builds rho for one sequence.
 *   L <= K           : rho = {0..L-1}  (budget covers the context).
 *   otherwise        : rho = unified[: K-W]  U  {L-W .. L-1}.
 * "unified" is the duplicate-free list of all heads' picks in global rank
 * order.  rank_mode selects the reading of "globally ranked":
 *   0  first occurrence in the rank-major flattening of rho_head
 *      (all rank-0 picks in head order, then all rank-1 picks, ...);
 *   1  number of proposing heads (desc), best per-head rank, position;
 *   2  largest proposing-head score (desc), position.
 * idx receives rho ascending by position; returns |rho|. */
int cusa_oracle_unify(const int32_t *rho_head, const float *P, int64_t ldp,
                      int H, int k_eff, int L, int K, int W, int rank_mode,
                      int32_t *idx) {
    if (L <= K) {
        for (int t = 0; t < L; ++t) idx[t] = t;
        return L;
    }
    int n_hist = K - W;
    int n = 0;
    int Lc = L - W;
    if (n_hist > 0 && k_eff > 0) {
        if (rank_mode == 0) {
            uint8_t *seen = (uint8_t *)calloc((size_t)Lc, 1);
            for (int j = 0; j < k_eff && n < n_hist; ++j)
                for (int h = 0; h < H && n < n_hist; ++h) {
                    int32_t t = rho_head[(int64_t)h * k_eff + j];
                    if (!seen[t]) {
                        seen[t] = 1;
                        idx[n++] = t;
                    }
                }
            free(seen);
        } else {
            int32_t *slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)Lc);
            for (int t = 0; t < Lc; ++t) slot[t] = -1;
            cand_t *c = (cand_t *)malloc(sizeof(cand_t) * (size_t)H * (size_t)k_eff);
            int nc = 0;
            for (int h = 0; h < H; ++h)
                for (int j = 0; j < k_eff; ++j) {
                    int32_t t = rho_head[(int64_t)h * k_eff + j];
                    float s = P ? P[(int64_t)h * ldp + t] : 0.0f;
                    if (slot[t] < 0) {
                        slot[t] = nc;
                        c[nc].pos = t;
                        c[nc].votes = 1;
                        c[nc].best_rank = j;
                        c[nc].max_score = s;
                        ++nc;
                    } else {
                        cand_t *e = &c[slot[t]];
                        e->votes += 1;
                        if (j < e->best_rank) e->best_rank = j;
                        if (s > e->max_score) e->max_score = s;
                    }
                }
            qsort(c, (size_t)nc, sizeof(cand_t), rank_mode == 1 ? cmp_votes : cmp_maxscore);
            for (int i = 0; i < nc && n < n_hist; ++i) idx[n++] = c[i].pos;
            free(c);
            free(slot);
        }
    }
    for (int t = L - W; t < L; ++t) idx[n++] = t;
    qsort(idx, (size_t)n, sizeof(int32_t), cmp_i32);
    return n;
}

/* ---- Eq. 1 (dense) and its restriction to rho (sparse) -------------------- */

/* o_h = softmax(sm_scale * q_h . K[T]^T) V[T] over the token list T = idx[0..n)
 * (idx == NULL: T = 0..n-1), everything in binary64; out_bf16 is the
 * round-to-nearest-even bf16 of the binary64 result, out_f64 (optional) the
 * unrounded one. */
void cusa_oracle_attention(const uint16_t *q, const uint16_t *Kc, const uint16_t *Vc,
                           int H, int G, int d, int L, const int32_t *idx, int n,
                           double sm_scale, uint16_t *out_bf16, double *out_f64) {
    int g = H / G;
#pragma omp parallel for schedule(static)
    for (int h = 0; h < H; ++h) {
        const uint16_t *qh = q + (int64_t)h * d;
        const uint16_t *Kh = Kc + (int64_t)(h / g) * L * d;
        const uint16_t *Vh = Vc + (int64_t)(h / g) * L * d;
        double *z = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        double *o = (double *)calloc((size_t)d, sizeof(double));
        double m = -INFINITY;
        for (int j = 0; j < n; ++j) {
            int64_t t = idx ? idx[j] : j;
            const uint16_t *kt = Kh + t * d;
            double acc = 0.0;
            for (int i = 0; i < d; ++i)
                acc += (double)bf16_to_f32(qh[i]) * (double)bf16_to_f32(kt[i]);
            z[j] = sm_scale * acc;
            if (z[j] > m) m = z[j];
        }
        double denom = 0.0;
        for (int j = 0; j < n; ++j) {
            int64_t t = idx ? idx[j] : j;
            double e = exp(z[j] - m);
            denom += e;
            const uint16_t *vt = Vh + t * d;
            for (int i = 0; i < d; ++i) o[i] += e * (double)bf16_to_f32(vt[i]);
        }
        for (int i = 0; i < d; ++i) {
            double v = n > 0 ? o[i] / denom : 0.0;
            if (out_f64) out_f64[(int64_t)h * d + i] = v;
            if (out_bf16) out_bf16[(int64_t)h * d + i] = f64_to_bf16_rne(v);
        }
        free(o);
        free(z);
    }
}

/* ---- Eq. 3: attention recall of a token set ------------------------------- */

/* recall[h] = sum_{t in rho} softmax(W_h)[t] / sum_t softmax(W_h)[t], where
 * W_h = sm_scale * q_h . K^T over all L tokens (binary64). */
void cusa_oracle_recall(const uint16_t *q, const uint16_t *Kc, int H, int G, int d,
                        int L, const int32_t *idx, int n, double sm_scale,
                        double *recall) {
    int g = H / G;
#pragma omp parallel for schedule(static)
    for (int h = 0; h < H; ++h) {
        const uint16_t *qh = q + (int64_t)h * d;
        const uint16_t *Kh = Kc + (int64_t)(h / g) * L * d;
        double *z = (double *)malloc(sizeof(double) * (size_t)L);
        double m = -INFINITY;
        for (int t = 0; t < L; ++t) {
            double acc = 0.0;
            for (int i = 0; i < d; ++i)
                acc += (double)bf16_to_f32(qh[i]) * (double)bf16_to_f32(Kh[(int64_t)t * d + i]);
            z[t] = sm_scale * acc;
            if (z[t] > m) m = z[t];
        }
        double all = 0.0, sel = 0.0;
        for (int t = 0; t < L; ++t) all += exp(z[t] - m);
        for (int j = 0; j < n; ++j) sel += exp(z[idx[j]] - m);
        recall[h] = sel / all;
        free(z);
    }
}
