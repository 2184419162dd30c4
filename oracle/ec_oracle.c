/*
 * Elastic Cache -- CPU oracle (TEST INFRASTRUCTURE, not a product path).
 *
 * A plain, slow, fp64 implementation of the per-layer KV-cache compression and
 * of the decode attention over the compressed cache, written from the paper
 * (Sec. 3.3 "One Sequence, Two Policies", Eq. 1-3, Alg. 1, and the
 * "Implementation Details" paragraph of Sec. 4.1).  It exists so that the GPU
 * library can be checked against it; only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may call it.  It shares no code, headers or
 * tables with the GPU library.
 *
 * Layout everywhere: dense row-major, [B,H,T,D] for prompt tensors (sequence on
 * axis 2, as Alg. 1 reads it), [B,H,cap,D] for caches, positions are 0-based.
 * All floating point is double.  Integer outputs are int32.
 *
 * No blocking, fusion or reordering: every function is the definition written
 * out as loops.  OpenMP only distributes independent (batch, head) problems.
 *
 * Readings of the paper taken here (the paper is silent or garbled there):
 *  - Eq. 1's denominator runs over all keys n' <= m (standard causal softmax);
 *    a `scale` factor multiplies the dot product (scale = 1 is the literal Eq. 1).
 *  - importance is the column sum over queries (Sec. 3.3, I_n = sum_m A_mn);
 *    layer-wise importance is the mean over heads.
 *  - N_I is an integer argument; callers use ceil(gamma*T) (Alg. 1's del_num).
 *  - ties in the top-N_I choice go to the lower index.
 *  - Eq. 2's last bucket starts one past the previous midpoint so that buckets
 *    partition 0..T-1; "nearest anchor, tie to the earlier anchor" is the same
 *    partition and is what oracle_assign_nearest computes exhaustively.
 *  - Eq. 3 mean includes the anchor's own vector, each member weight 1.
 *  - a later multi-token pass (chat history: Sec. 3.3 applies the compression to
 *    all concatenated inputs; Alg. 1 is entered with a non-empty past and gen_len
 *    > 1): the chunk's queries attend the P cached rows in full and the chunk
 *    causally; the importance of every row of [cache | chunk] is its column sum
 *    over THIS pass's queries (Alg. 1 assigns S, it does not accumulate); rows are
 *    merged by the plain mean of Eq. 3 over row indices of the concatenated
 *    sequence.  A count-weighted mean (each row weighted by the number of
 *    original tokens it already stands for) is offered beside it as an extension.
 *  - decode order: append the new row, attend over all rows, then remove one row.
 *  - "Frequency" discard policy during generation (the Frequency Cache of Sec. 4.1
 *    Baselines, ablation row of Table 3a): every cached row carries the attention
 *    mass it has received so far (layer-wise: the head mean, like the prompt
 *    metric); each generated token adds its attention row to it; when a row must
 *    go, the row with the least mass goes.  The paper leaves open: where a new
 *    row's count starts (here: at the mass it receives from its own query), which
 *    rows are exempt (here: the first protect_first and the newest protect_recent
 *    rows, arguments), and ties (here: the lowest index).  The comparison is made
 *    on fp32 values, the precision the counts are kept in.
 *  - retention test: evict iff the cache is longer than ceil(gamma*n) (Alg. 1's
 *    int(seq_len - n(1-r)) >= 1); truncation location = R rows before the newest
 *    row (R = 25 in Sec. 4.1), or an absolute location N_tl (Sec. 3.3 text).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------- */
/* Sec. 3.3, Eq. 1 and the importance definition that follows it.             */
/*                                                                           */
/* q,k,v [B,H,T,D].  For every head: A = causal row-softmax(scale * q k^T).  */
/* out   [B,H,T,D]  = A v            (may be NULL)                           */
/* lse   [B,H,T]    = log sum_{n<=m} exp(s_mn)   (may be NULL)               */
/* head_imp [B,H,T] = sum_m A_mn     (per-head importance I_n^{i,j})         */
/* score [B,G,T]: G == H -> head_imp; G == 1 -> mean over heads (I_n^i).     */
/* attn  [B,H,T,T] full matrix dump for tiny tests (may be NULL).            */
/* ------------------------------------------------------------------------- */
int oracle_prefill_score(const double *q, const double *k, const double *v,
                         int B, int H, int T, int D, double scale, int G,
                         double *out, double *lse, double *score, double *attn)
{
    if (B < 1 || H < 1 || T < 1 || D < 1 || (G != 1 && G != H)) return 1;
    double *head_imp = (double *)calloc((size_t)B * H * T, sizeof(double));
    if (!head_imp) return 2;
    int fail = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * H; ++bh) {
        const double *qh = q + (size_t)bh * T * D;
        const double *kh = k + (size_t)bh * T * D;
        const double *vh = v + (size_t)bh * T * D;
        double *imp = head_imp + (size_t)bh * T;
        double *row = (double *)malloc((size_t)T * sizeof(double));
        if (!row) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        for (int m = 0; m < T; ++m) {
            /* s_mn for n <= m */
            double smax = -INFINITY;
            for (int n = 0; n <= m; ++n) {
                double dot = 0.0;
                for (int d = 0; d < D; ++d) dot += qh[(size_t)m * D + d] * kh[(size_t)n * D + d];
                row[n] = scale * dot;
                if (row[n] > smax) smax = row[n];
            }
            double denom = 0.0;
            for (int n = 0; n <= m; ++n) {
                row[n] = exp(row[n] - smax);
                denom += row[n];
            }
            if (lse) lse[(size_t)bh * T + m] = smax + log(denom);
            for (int n = 0; n <= m; ++n) row[n] /= denom; /* A_mn */
            for (int n = 0; n <= m; ++n) imp[n] += row[n];
            if (attn) {
                double *arow = attn + ((size_t)bh * T + m) * T;
                for (int n = 0; n < T; ++n) arow[n] = (n <= m) ? row[n] : 0.0;
            }
            if (out) {
                double *o = out + ((size_t)bh * T + m) * D;
                for (int d = 0; d < D; ++d) o[d] = 0.0;
                for (int n = 0; n <= m; ++n)
                    for (int d = 0; d < D; ++d) o[d] += row[n] * vh[(size_t)n * D + d];
            }
        }
        free(row);
    }

    if (!fail) {
        if (G == H) {
            memcpy(score, head_imp, (size_t)B * H * T * sizeof(double));
        } else {
            for (int b = 0; b < B; ++b)
                for (int n = 0; n < T; ++n) {
                    double acc = 0.0;
                    for (int h = 0; h < H; ++h) acc += head_imp[((size_t)b * H + h) * T + n];
                    score[(size_t)b * T + n] = acc / (double)H;
                }
        }
    }
    free(head_imp);
    return fail ? 2 : 0;
}

/* ------------------------------------------------------------------------- */
/* Sec. 3.3 "select the top N_I tokens in I_n, indices in ascending order",   */
/* with the first `protect_first` and last `protect_last` positions always    */
/* kept (Sec. 4.1 Implementation Details).  Scores are compared as fp32       */
/* values; among equal scores the lower index wins.  NaN is outside the       */
/* domain.                                                                   */
/* score [B,G,T] float -> anchor_idx [B,G,n_anchor] int32 ascending.          */
/* ------------------------------------------------------------------------- */
typedef struct {
    float s;
    int32_t i;
} cand_t;

static int cand_before(const void *a, const void *b)
{
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->s > y->s) return -1; /* higher score first */
    if (x->s < y->s) return 1;
    return (x->i > y->i) - (x->i < y->i); /* then lower index */
}

static int int_ascending(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

int oracle_select_anchors(const float *score, int B, int G, int T, int n_anchor,
                          int protect_first, int protect_last, int32_t *anchor_idx)
{
    if (B < 1 || G < 1 || T < 1 || n_anchor < 1 || n_anchor > T) return 1;
    if (protect_first < 0 || protect_last < 0 || protect_first + protect_last > n_anchor) return 1;
    const int n_free = n_anchor - protect_first - protect_last;
    for (int bg = 0; bg < B * G; ++bg) {
        const float *s = score + (size_t)bg * T;
        int32_t *dst = anchor_idx + (size_t)bg * n_anchor;
        cand_t *c = (cand_t *)malloc((size_t)T * sizeof(cand_t));
        if (!c) return 2;
        int nc = 0, nd = 0;
        for (int t = 0; t < T; ++t) {
            if (t < protect_first || t >= T - protect_last)
                dst[nd++] = t;
            else {
                c[nc].s = s[t];
                c[nc].i = t;
                ++nc;
            }
        }
        qsort(c, (size_t)nc, sizeof(cand_t), cand_before);
        for (int j = 0; j < n_free; ++j) dst[nd++] = c[j].i;
        qsort(dst, (size_t)n_anchor, sizeof(int32_t), int_ascending);
        free(c);
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Alg. 1's Nearest(throw_idx, keep_idx), written exhaustively: every         */
/* position goes to the anchor at the smallest |t - t_k|, tie to the smaller  */
/* k.  anchor_idx [B,G,n] ascending -> assign [B,G,T] (bucket number),        */
/* counts [B,G,n].                                                           */
/* ------------------------------------------------------------------------- */
int oracle_assign_nearest(const int32_t *anchor_idx, int B, int G, int T, int n_anchor,
                          int32_t *assign, int32_t *counts)
{
    if (B < 1 || G < 1 || T < 1 || n_anchor < 1 || n_anchor > T) return 1;
    for (int bg = 0; bg < B * G; ++bg) {
        const int32_t *a = anchor_idx + (size_t)bg * n_anchor;
        int32_t *as = assign + (size_t)bg * T;
        int32_t *cn = counts + (size_t)bg * n_anchor;
        for (int kk = 0; kk < n_anchor; ++kk) cn[kk] = 0;
        for (int t = 0; t < T; ++t) {
            int best = 0;
            long bestd = labs((long)t - (long)a[0]);
            for (int kk = 1; kk < n_anchor; ++kk) {
                long d = labs((long)t - (long)a[kk]);
                if (d < bestd) {
                    bestd = d;
                    best = kk;
                }
            }
            as[t] = best;
            cn[best] += 1;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Eq. 2: bucket k = { floor((t_{k-1}+t_k)/2)+1 .. floor((t_k+t_{k+1})/2) },  */
/* the first bucket starting at 0 and the last ending at T-1.                 */
/* anchor_idx [B,G,n] -> lo,hi [B,G,n] inclusive bounds.                      */
/* ------------------------------------------------------------------------- */
int oracle_bucket_bounds(const int32_t *anchor_idx, int B, int G, int T, int n_anchor,
                         int32_t *lo, int32_t *hi)
{
    if (B < 1 || G < 1 || T < 1 || n_anchor < 1 || n_anchor > T) return 1;
    for (int bg = 0; bg < B * G; ++bg) {
        const int32_t *a = anchor_idx + (size_t)bg * n_anchor;
        for (int kk = 0; kk < n_anchor; ++kk) {
            size_t o = (size_t)bg * n_anchor + kk;
            lo[o] = (kk == 0) ? 0 : (a[kk - 1] + a[kk]) / 2 + 1;
            hi[o] = (kk == n_anchor - 1) ? T - 1 : (a[kk] + a[kk + 1]) / 2;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Eq. 3 + Alg. 1's gather: per head, cache row k = mean of the rows assigned */
/* to bucket k.  x [B,H,T,D], assign [B,G,T] (G in {1,H}) -> cache [B,H,cap,D]*/
/* rows 0..n_anchor-1 (other rows untouched).                                 */
/* ------------------------------------------------------------------------- */
int oracle_merge_compact(const double *x, const int32_t *assign, int B, int H, int G, int T,
                         int D, int n_anchor, int cap, double *cache)
{
    if (B < 1 || H < 1 || T < 1 || D < 1 || (G != 1 && G != H)) return 1;
    if (n_anchor < 1 || n_anchor > T || cap < n_anchor) return 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * H; ++bh) {
        int b = bh / H, h = bh % H;
        const int32_t *as = assign + ((size_t)b * G + (G == 1 ? 0 : h)) * T;
        const double *xh = x + (size_t)bh * T * D;
        double *ch = cache + (size_t)bh * cap * D;
        for (int kk = 0; kk < n_anchor; ++kk) {
            double *row = ch + (size_t)kk * D;
            int cnt = 0;
            for (int d = 0; d < D; ++d) row[d] = 0.0;
            for (int t = 0; t < T; ++t) {
                if (as[t] != kk) continue;
                for (int d = 0; d < D; ++d) row[d] += xh[(size_t)t * D + d];
                ++cnt;
            }
            for (int d = 0; d < D; ++d) row[d] /= (double)cnt;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* "Cache Eviction" ablation (Table 3b; Sec. 3.2 Cache Eviction v.s. Cache     */
/* Merging): keep the anchors' own rows, drop everything else.                */
/* x [B,H,T,D], anchor_idx [B,G,n] -> cache [B,H,cap,D] rows 0..n-1.           */
/* ------------------------------------------------------------------------- */
int oracle_evict_compact(const double *x, const int32_t *anchor_idx, int B, int H, int G, int T,
                         int D, int n_anchor, int cap, double *cache)
{
    if (B < 1 || H < 1 || T < 1 || D < 1 || (G != 1 && G != H)) return 1;
    if (n_anchor < 1 || n_anchor > T || cap < n_anchor) return 1;
    for (int bh = 0; bh < B * H; ++bh) {
        int b = bh / H, h = bh % H;
        const int32_t *a = anchor_idx + ((size_t)b * G + (G == 1 ? 0 : h)) * n_anchor;
        for (int kk = 0; kk < n_anchor; ++kk)
            for (int d = 0; d < D; ++d)
                cache[((size_t)bh * cap + kk) * D + d] = x[((size_t)bh * T + a[kk]) * D + d];
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Multi-token pass over an existing compressed cache (Sec. 3.3: encoding     */
/* covers system prompt, instruction and chat history; Alg. 1's gen_len > 1   */
/* branch with a non-empty past: attn is gen_len x seq_len).                  */
/*                                                                           */
/* q [B,H,Tq,D]: the chunk's queries.  k,v [B,H,L,D], L = P + Tq: P cached     */
/* rows followed by the chunk's own rows.  Query m sees rows n <= P + m.      */
/* out [B,H,Tq,D] (may be NULL), lse [B,H,Tq] (may be NULL),                   */
/* score [B,G,L]: column sums over the Tq queries (G == 1: head mean).        */
/* ------------------------------------------------------------------------- */
int oracle_chunk_score(const double *q, const double *k, const double *v, int B, int H, int Tq,
                       int P, int D, double scale, int G, double *out, double *lse,
                       double *score)
{
    if (B < 1 || H < 1 || Tq < 1 || P < 0 || D < 1 || (G != 1 && G != H)) return 1;
    const int L = P + Tq;
    double *head_imp = (double *)calloc((size_t)B * H * L, sizeof(double));
    if (!head_imp) return 2;
    int fail = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * H; ++bh) {
        const double *qh = q + (size_t)bh * Tq * D;
        const double *kh = k + (size_t)bh * L * D;
        const double *vh = v + (size_t)bh * L * D;
        double *imp = head_imp + (size_t)bh * L;
        double *row = (double *)malloc((size_t)L * sizeof(double));
        if (!row) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        for (int m = 0; m < Tq; ++m) {
            const int last = P + m; /* newest row this query may see */
            double smax = -INFINITY;
            for (int n = 0; n <= last; ++n) {
                double dot = 0.0;
                for (int d = 0; d < D; ++d) dot += qh[(size_t)m * D + d] * kh[(size_t)n * D + d];
                row[n] = scale * dot;
                if (row[n] > smax) smax = row[n];
            }
            double denom = 0.0;
            for (int n = 0; n <= last; ++n) {
                row[n] = exp(row[n] - smax);
                denom += row[n];
            }
            if (lse) lse[(size_t)bh * Tq + m] = smax + log(denom);
            for (int n = 0; n <= last; ++n) {
                row[n] /= denom;
                imp[n] += row[n];
            }
            if (out) {
                double *o = out + ((size_t)bh * Tq + m) * D;
                for (int d = 0; d < D; ++d) o[d] = 0.0;
                for (int n = 0; n <= last; ++n)
                    for (int d = 0; d < D; ++d) o[d] += row[n] * vh[(size_t)n * D + d];
            }
        }
        free(row);
    }

    if (!fail) {
        if (G == H) {
            memcpy(score, head_imp, (size_t)B * H * L * sizeof(double));
        } else {
            for (int b = 0; b < B; ++b)
                for (int n = 0; n < L; ++n) {
                    double acc = 0.0;
                    for (int h = 0; h < H; ++h) acc += head_imp[((size_t)b * H + h) * L + n];
                    score[(size_t)b * L + n] = acc / (double)H;
                }
        }
    }
    free(head_imp);
    return fail ? 2 : 0;
}

/* ------------------------------------------------------------------------- */
/* Count-weighted merge (extension beside Eq. 3, for re-merging rows that      */
/* already stand for several tokens): cache row k = sum_t w_t x_t / sum_t w_t  */
/* over the rows t of bucket k.  x [B,H,T,D], assign [B,G,T], w [B,G,T] int32  */
/* positive weights -> cache [B,H,cap,D] rows 0..n_anchor-1 and                */
/* wsum [B,G,n_anchor] (may be NULL).  With every w = 1 this is Eq. 3.         */
/* ------------------------------------------------------------------------- */
int oracle_merge_weighted(const double *x, const int32_t *assign, const int32_t *w, int B, int H,
                          int G, int T, int D, int n_anchor, int cap, double *cache,
                          int32_t *wsum)
{
    if (B < 1 || H < 1 || T < 1 || D < 1 || (G != 1 && G != H)) return 1;
    if (n_anchor < 1 || n_anchor > T || cap < n_anchor) return 1;
    for (int bh = 0; bh < B * H; ++bh) {
        int b = bh / H, h = bh % H;
        size_t bg = (size_t)b * G + (G == 1 ? 0 : h);
        const int32_t *as = assign + bg * T;
        const int32_t *wt = w + bg * T;
        const double *xh = x + (size_t)bh * T * D;
        double *ch = cache + (size_t)bh * cap * D;
        for (int kk = 0; kk < n_anchor; ++kk) {
            double *row = ch + (size_t)kk * D;
            long long tot = 0;
            for (int d = 0; d < D; ++d) row[d] = 0.0;
            for (int t = 0; t < T; ++t) {
                if (as[t] != kk) continue;
                if (wt[t] < 1) return 1;
                for (int d = 0; d < D; ++d) row[d] += (double)wt[t] * xh[(size_t)t * D + d];
                tot += wt[t];
            }
            for (int d = 0; d < D; ++d) row[d] /= (double)tot;
            if (wsum && (G == H || h == 0)) wsum[bg * n_anchor + kk] = (int32_t)tot;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Retention test + truncation location (Sec. 3.3 Output Generation, Alg. 1). */
/* n_seen: tokens seen so far including the one just appended.                */
/* len_after_append: cache rows including the new one.                        */
/* gamma = gamma_num / gamma_den.                                             */
/* budget_mode 0: keep ceil(gamma * n_seen) rows (Alg. 1's del_num test);     */
/* budget_mode 1: constant size, evict whenever len_after_append > fixed_len. */
/* trunc_mode 0: idx = len_after_append - 1 - recent (recent = 25, Sec. 4.1); */
/* trunc_mode 1: idx = n_tl (absolute truncation location, Sec. 3.3).         */
/* Row protect_first.. never below; the newest row is never the victim: if no */
/* legal victim exists nothing is evicted.  Returns idx or -1.                */
/* ------------------------------------------------------------------------- */
int oracle_evict_index(int64_t n_seen, int len_after_append, int gamma_num, int gamma_den,
                       int budget_mode, int fixed_len, int trunc_mode, int recent, int n_tl,
                       int protect_first)
{
    int64_t target;
    if (budget_mode == 0)
        target = ((int64_t)gamma_num * n_seen + gamma_den - 1) / gamma_den; /* ceil */
    else
        target = fixed_len;
    if ((int64_t)len_after_append <= target) return -1;
    int idx = (trunc_mode == 0) ? len_after_append - 1 - recent : n_tl;
    if (idx < protect_first) idx = protect_first;
    if (idx >= len_after_append - 1) return -1;
    return idx;
}

/* ------------------------------------------------------------------------- */
/* One output-generation step for one layer (Sec. 3.1 Output Generation,      */
/* Sec. 3.3 fixed-point elimination).                                        */
/* q,k_new,v_new [B,H,D]; k_cache,v_cache [B,H,cap,D] with cache_len valid    */
/* rows; pos [B,G,cap] (original position of every row) or NULL.              */
/* 1. row cache_len <- (k_new, v_new), pos <- new_pos                         */
/* 2. out = softmax(scale * q . K^T) V over rows 0..cache_len  (plain, no     */
/*    count weighting); probs [B,H,cache_len+1] optional dump                 */
/* 3. if evict_idx >= 0 remove that row (rows behind it move up by one)       */
/* ------------------------------------------------------------------------- */
int oracle_decode_step(const double *q, const double *k_new, const double *v_new,
                       double *k_cache, double *v_cache, int32_t *pos, int B, int H, int G,
                       int D, int cap, int cache_len, int evict_idx, int32_t new_pos,
                       double scale, double *out, double *probs)
{
    if (B < 1 || H < 1 || D < 1 || (G != 1 && G != H)) return 1;
    if (cache_len < 0 || cache_len + 1 > cap) return 1;
    if (evict_idx < -1 || evict_idx > cache_len) return 1;
    const int n = cache_len + 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * H; ++bh) {
        double *kc = k_cache + (size_t)bh * cap * D;
        double *vc = v_cache + (size_t)bh * cap * D;
        const double *qv = q + (size_t)bh * D;
        memcpy(kc + (size_t)cache_len * D, k_new + (size_t)bh * D, (size_t)D * sizeof(double));
        memcpy(vc + (size_t)cache_len * D, v_new + (size_t)bh * D, (size_t)D * sizeof(double));

        double *p = (double *)malloc((size_t)n * sizeof(double));
        double smax = -INFINITY;
        for (int j = 0; j < n; ++j) {
            double dot = 0.0;
            for (int d = 0; d < D; ++d) dot += qv[d] * kc[(size_t)j * D + d];
            p[j] = scale * dot;
            if (p[j] > smax) smax = p[j];
        }
        double denom = 0.0;
        for (int j = 0; j < n; ++j) {
            p[j] = exp(p[j] - smax);
            denom += p[j];
        }
        double *o = out + (size_t)bh * D;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        for (int j = 0; j < n; ++j) {
            p[j] /= denom;
            for (int d = 0; d < D; ++d) o[d] += p[j] * vc[(size_t)j * D + d];
        }
        if (probs) memcpy(probs + (size_t)bh * n, p, (size_t)n * sizeof(double));
        free(p);

        if (evict_idx >= 0) {
            size_t tail = (size_t)(cache_len - evict_idx) * D;
            memmove(kc + (size_t)evict_idx * D, kc + (size_t)(evict_idx + 1) * D, tail * sizeof(double));
            memmove(vc + (size_t)evict_idx * D, vc + (size_t)(evict_idx + 1) * D, tail * sizeof(double));
        }
    }
    if (pos) {
        for (int bg = 0; bg < B * G; ++bg) {
            int32_t *pp = pos + (size_t)bg * cap;
            pp[cache_len] = new_pos;
            if (evict_idx >= 0)
                memmove(pp + evict_idx, pp + evict_idx + 1,
                        (size_t)(cache_len - evict_idx) * sizeof(int32_t));
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Frequency policy, part 1 (Sec. 4.1 Baselines "Frequency Cache ... records   */
/* how often each key-value pair is accessed ... continuously updates the      */
/* frequency counts throughout the generation"): add one generation step's     */
/* attention row to the per-row mass.                                         */
/* probs [B,H,n] (this step's softmax rows), freq [B,G,cap] updated in place: */
/* rows 0..n-2 += mass, row n-1 (the row just appended) = its mass.           */
/* G == 1: mass = mean over heads; G == H: the head's own probability.        */
/* ------------------------------------------------------------------------- */
int oracle_freq_accumulate(const double *probs, int B, int H, int G, int n, int cap, double *freq)
{
    if (B < 1 || H < 1 || n < 1 || n > cap || (G != 1 && G != H)) return 1;
    for (int b = 0; b < B; ++b)
        for (int g = 0; g < G; ++g)
            for (int j = 0; j < n; ++j) {
                double mass;
                if (G == H) {
                    mass = probs[((size_t)b * H + g) * n + j];
                } else {
                    mass = 0.0;
                    for (int h = 0; h < H; ++h) mass += probs[((size_t)b * H + h) * n + j];
                    mass /= (double)H;
                }
                double *f = freq + ((size_t)b * G + g) * cap + j;
                *f = (j == n - 1) ? mass : *f + mass;
            }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Frequency policy, part 2 ("selects the least frequently accessed key-value  */
/* pairs for eviction"): per (b,g) the victim is the row of least mass among   */
/* rows protect_first .. len-1-protect_recent, the lowest index among equals,  */
/* compared as fp32 values.  The row is removed from k_cache, v_cache          */
/* [B,H,cap,D], pos [B,G,cap] (may be NULL) and freq [B,G,cap] float; rows     */
/* behind it move up by one.  victim [B,G] receives the index.                 */
/* ------------------------------------------------------------------------- */
int oracle_evict_min(float *freq, double *k_cache, double *v_cache, int32_t *pos, int B, int H,
                     int G, int D, int cap, int len, int protect_first, int protect_recent,
                     int32_t *victim)
{
    if (B < 1 || H < 1 || D < 1 || (G != 1 && G != H) || len < 1 || len > cap) return 1;
    if (protect_first < 0 || protect_recent < 0 || protect_first + protect_recent >= len) return 1;
    for (int b = 0; b < B; ++b)
        for (int g = 0; g < G; ++g) {
            float *f = freq + ((size_t)b * G + g) * cap;
            int best = protect_first;
            for (int j = protect_first + 1; j <= len - 1 - protect_recent; ++j)
                if (f[j] < f[best]) best = j;
            victim[(size_t)b * G + g] = best;
            for (int j = best; j + 1 < len; ++j) f[j] = f[j + 1];
            if (pos) {
                int32_t *p = pos + ((size_t)b * G + g) * cap;
                for (int j = best; j + 1 < len; ++j) p[j] = p[j + 1];
            }
            for (int h = (G == H ? g : 0); h < (G == H ? g + 1 : H); ++h) {
                double *kc = k_cache + ((size_t)b * H + h) * cap * D;
                double *vc = v_cache + ((size_t)b * H + h) * cap * D;
                memmove(kc + (size_t)best * D, kc + (size_t)(best + 1) * D,
                        (size_t)(len - 1 - best) * D * sizeof(double));
                memmove(vc + (size_t)best * D, vc + (size_t)(best + 1) * D,
                        (size_t)(len - 1 - best) * D * sizeof(double));
            }
        }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* "Mean" importance metric of the ablation (Table 3d) next to the default    */
/* "Sum": the column mass divided by the number of queries that can see the   */
/* key.  In a pass of Tq queries over P cached rows + the chunk (P = 0: the   */
/* prompt pass) row n is seen by queries m >= max(0, n - P), i.e. by           */
/* Tq - max(0, n - P) of them.  score [B,G,P+Tq], in place.                   */
/* ------------------------------------------------------------------------- */
int oracle_importance_mean(double *score, int B, int G, int Tq, int P)
{
    if (B < 1 || G < 1 || Tq < 1 || P < 0) return 1;
    const int L = P + Tq;
    for (size_t bg = 0; bg < (size_t)B * G; ++bg)
        for (int n = 0; n < L; ++n) {
            int first = n - P;
            if (first < 0) first = 0;
            score[bg * L + n] /= (double)(Tq - first);
        }
    return 0;
}
