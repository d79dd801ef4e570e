/*
 * reform_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, fp64 CPU statement of what the REFORM compress-and-gather hot
 * path computes.  It exists so that tests, the smoke check and the benchmark's
 * CPU-baseline leg have something obviously correct to compare the GPU library
 * against.  The GPU library never includes, links or calls anything in this
 * file, and this file includes nothing from the GPU library.
 *
 * Every routine is the textbook definition written out row by row: no
 * tiling, no online softmax, no fusion.  Inputs arrive as float (bf16 and
 * fp32 inputs widen to float exactly, so the caller's widening changes no
 * bit); all arithmetic is double.
 *
 * Paper passages followed (arXiv 2506.01215):
 *   - Sec. 3.1 "Embedding extraction with recurrent chunked forwarding":
 *     each chunk is forwarded conditioned on the compressed KV cache of the
 *     earlier chunks (Fig. 1 step 1, Alg. 1 ForwardChunk), then the cache is
 *     compressed by attention-based token eviction in the manner of H2O,
 *     retained tokens keeping their order (consecutive position ids).
 *   - Sec. 1 (only the most influential tokens stay in the cache) and Sec. 4 common setup
 *     (always-kept initial/recent tokens, 128-query observation window of
 *     the H2O implementation).
 *   - Sec. 3.2, the concatenation-of-normalised-heads equation, and Sec. 3.3
 *     "Identification of significant inputs" (cosine similarity between
 *     query and context embeddings, max-pooling over the query tokens and
 *     over adjacent tokens, highest scores selected, forced first and last
 *     tokens; gathering the selected inputs for recomputation), Sec. 4.5
 *     (pooling window), App. C.6 "Similarity search".
 *   - Sec. 3.1, position ids made consecutive after compression (rotary keys).
 *
 * Readings taken where the paper gives no formula:
 *   - eviction score of key j in KV head g = sum over the G query heads of
 *     the group and over the observing rows of the post-softmax probability
 *     p_ij (attention mass received); raw sum, no normalisation;
 *   - mask: every cache row is visible, chunk rows are causal with the
 *     diagonal included;
 *   - ties in any top selection go to the lowest index;
 *   - cosine uses the clamp  dot / max(|e||u|, eps);
 *   - the pooling window is clipped at the ends of the context;
 *   - rotary pairing is the half-split one (element c with c + rot/2);
 *   - a zero head vector stays zero when an embedding segment is normalised.
 *
 * Parity status: every routine below is pinned by CPU tests against brute
 * force, closed forms, invariants and library routines (tests/test_oracle_*).
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

/* Thread count of the calling thread's later parallel loops (a test that already
 * spreads rows over its own threads sets 1).  No arithmetic depends on it.   */
void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------------ */
/* One attention row, straight from the definition (Sec. 3.1, Fig. 1 step 1):
 *   s_j   = scale * <q, k_j>           for j = 0 .. nvis-1
 *   p_j   = exp(s_j - max s) / sum_j exp(s_j - max s)
 *   o     = sum_j p_j v_j
 *   lse   = max s + log(sum_j exp(s_j - max s))
 * p (length nvis) is left in `p` for the caller.                            */
static void attention_row(const float *q, const float *k, const float *v,
                          int d, int nvis, double scale,
                          double *p, double *o, double *lse)
{
    double m = -INFINITY;
    for (int j = 0; j < nvis; ++j) {
        const float *kj = k + (size_t)j * d;
        double s = 0.0;
        for (int c = 0; c < d; ++c) s += (double)q[c] * (double)kj[c];
        s *= scale;
        p[j] = s;
        if (s > m) m = s;
    }
    double l = 0.0;
    for (int j = 0; j < nvis; ++j) { p[j] = exp(p[j] - m); l += p[j]; }
    for (int c = 0; c < d; ++c) o[c] = 0.0;
    for (int j = 0; j < nvis; ++j) {
        p[j] /= l;
        const float *vj = v + (size_t)j * d;
        for (int c = 0; c < d; ++c) o[c] += p[j] * (double)vj[c];
    }
    *lse = m + log(l);
}

/* Chunk attention over [cache || chunk] plus the eviction score.
 *
 * q      [Hq][Ct][d]     queries of the chunk
 * k, v   [Hkv][cap][d]   rows [0,M) = retained cache, rows [M,M+Ct) = chunk
 * out    [Hq][Ct][d]     attention output               (may be NULL)
 * lse    [Hq][Ct]        log-sum-exp of the scaled logits (may be NULL)
 * score  [Hkv][cap]      entries [0,M+Ct): attention mass key j received from
 *                        the last W rows of the chunk, summed over the
 *                        G = Hq/Hkv query heads of the group.  Overwritten
 *                        unless accumulate != 0.        (may be NULL)
 * Row i (0-based inside the chunk) sees keys j <= M + i.
 * Returns 0, or -1 on a bad argument.                                       */
int oracle_attend_score(const float *q, const float *k, const float *v,
                        int Hq, int Hkv, int d, int M, int Ct, int cap,
                        double scale, int W, int accumulate,
                        double *out, double *lse, double *score)
{
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv || d <= 0 || M < 0 || Ct <= 0 ||
        cap < M + Ct || W < 0 || W > Ct)
        return -1;
    if (W == 0) W = Ct;
    const int G = Hq / Hkv;
    const int n = M + Ct;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int g = 0; g < Hkv; ++g) {
        double *p = (double *)malloc(sizeof(double) * (size_t)n);
        double *o = (double *)malloc(sizeof(double) * (size_t)d);
        if (!p || !o) {
#pragma omp atomic write
            bad = 1;
            free(p); free(o); continue;
        }
        const float *kg = k + (size_t)g * cap * d;
        const float *vg = v + (size_t)g * cap * d;
        double *sg = score ? score + (size_t)g * cap : NULL;
        if (sg && !accumulate)
            for (int j = 0; j < n; ++j) sg[j] = 0.0;
        for (int hh = 0; hh < G; ++hh) {
            const int h = g * G + hh;
            for (int i = 0; i < Ct; ++i) {
                const float *qi = q + ((size_t)h * Ct + i) * d;
                const int nvis = M + i + 1;
                double l;
                attention_row(qi, kg, vg, d, nvis, scale, p, o, &l);
                if (out)
                    memcpy(out + ((size_t)h * Ct + i) * d, o, sizeof(double) * (size_t)d);
                if (lse) lse[(size_t)h * Ct + i] = l;
                if (sg && i >= Ct - W)
                    for (int j = 0; j < nvis; ++j) sg[j] += p[j];
            }
        }
        free(p); free(o);
    }
    return bad ? -2 : 0;
}

/* Same definition for a caller-chosen list of rows only (used to check
 * sampled outputs at sizes where the full pass would take hours).
 * rows_h[r], rows_i[r] name query head and chunk row of sample r.
 * out [nrows][d], lse [nrows].  If score != NULL ([Hkv][cap], zeroed here),
 * it receives the attention mass of the SAMPLED rows only:
 *     score[g][j] = sum over samples r with rows_h[r]/G == g of p_{r,j}.    */
int oracle_attend_rows(const float *q, const float *k, const float *v,
                       int Hq, int Hkv, int d, int M, int Ct, int cap,
                       double scale, const int32_t *rows_h, const int32_t *rows_i,
                       int nrows, double *out, double *lse, double *score)
{
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv || d <= 0 || M < 0 || Ct <= 0 || cap < M + Ct)
        return -1;
    const int G = Hq / Hkv;
    const int n = M + Ct;
    int bad = 0;
    for (int r = 0; r < nrows; ++r)
        if (rows_h[r] < 0 || rows_h[r] >= Hq || rows_i[r] < 0 || rows_i[r] >= Ct) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int g = 0; g < Hkv; ++g) {
        double *p = (double *)malloc(sizeof(double) * (size_t)n);
        if (!p) {
#pragma omp atomic write
            bad = 1;
            continue;
        }
        double *sg = score ? score + (size_t)g * cap : NULL;
        if (sg)
            for (int j = 0; j < n; ++j) sg[j] = 0.0;
        for (int r = 0; r < nrows; ++r) {
            const int h = rows_h[r], i = rows_i[r];
            if (h / G != g) continue;
            const int nvis = M + i + 1;
            attention_row(q + ((size_t)h * Ct + i) * d, k + (size_t)g * cap * d,
                          v + (size_t)g * cap * d, d, nvis, scale, p,
                          out + (size_t)r * d, lse + r);
            if (sg)
                for (int j = 0; j < nvis; ++j) sg[j] += p[j];
        }
        free(p);
    }
    return bad ? -2 : 0;
}

/* ------------------------------------------------------------------------ */
/* Selection of the `keep` largest of x[0..n), ties to the lowest index.
 * Definition: sort indices by (value descending, index ascending), take the
 * first `keep`, then list them in ascending index order.                    */
typedef struct { double val; int32_t idx; } oracle_pair;

static int cmp_val_desc_idx_asc(const void *a, const void *b)
{
    const oracle_pair *x = (const oracle_pair *)a, *y = (const oracle_pair *)b;
    if (x->val > y->val) return -1;
    if (x->val < y->val) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* out_idx[keep], ascending.  Returns 0 or -1.                               */
int oracle_topk_lowest_index(const double *x, int64_t n, int64_t keep, int32_t *out_idx)
{
    if (n < 0 || keep < 0 || keep > n) return -1;
    oracle_pair *a = (oracle_pair *)malloc(sizeof(oracle_pair) * (size_t)(n ? n : 1));
    if (!a) return -2;
    for (int64_t j = 0; j < n; ++j) { a[j].val = x[j]; a[j].idx = (int32_t)j; }
    qsort(a, (size_t)n, sizeof(oracle_pair), cmp_val_desc_idx_asc);
    for (int64_t r = 0; r < keep; ++r) out_idx[r] = a[r].idx;
    qsort(out_idx, (size_t)keep, sizeof(int32_t), cmp_i32);
    free(a);
    return 0;
}

/* Heavy-hitter retention for one KV head (Sec. 3.1; Sec. 1; Sec. 4 setup):
 * among n = M + Ct candidate slots keep the B with the largest score; the
 * first n_sink and the last n_recent slots are always kept and count inside
 * B.  If n <= B everything is kept.  kept[min(n,B)] ascending.
 * Returns the number kept, or -1 on a bad argument.                         */
int oracle_evict_select(const double *score, int n, int B, int n_sink, int n_recent,
                        int32_t *kept)
{
    if (n < 0 || B < 0 || n_sink < 0 || n_recent < 0 || n_sink + n_recent > B) return -1;
    if (n <= B) {
        for (int j = 0; j < n; ++j) kept[j] = j;
        return n;
    }
    double *key = (double *)malloc(sizeof(double) * (size_t)n);
    if (!key) return -2;
    for (int j = 0; j < n; ++j)
        key[j] = (j < n_sink || j >= n - n_recent) ? INFINITY : score[j];
    int rc = oracle_topk_lowest_index(key, n, B, kept);
    free(key);
    return rc ? rc : B;
}

/* Order-preserving compaction (Sec. 3.1: retained tokens get consecutive
 * position ids): row r of the result is row kept[r] of the input, for
 * K, V (row length d), score and pos of one KV head.  Goes through a
 * temporary, never in place.  Any of k, v, score, pos may be NULL.          */
int oracle_compact_rows(float *k, float *v, double *score, int32_t *pos,
                        int d, const int32_t *kept, int n_kept)
{
    if (n_kept < 0 || d <= 0) return -1;
    size_t rows = (size_t)(n_kept ? n_kept : 1);
    float *tk = (float *)malloc(sizeof(float) * rows * d);
    float *tv = (float *)malloc(sizeof(float) * rows * d);
    double *ts = (double *)malloc(sizeof(double) * rows);
    int32_t *tp = (int32_t *)malloc(sizeof(int32_t) * rows);
    if (!tk || !tv || !ts || !tp) { free(tk); free(tv); free(ts); free(tp); return -2; }
    for (int r = 0; r < n_kept; ++r) {
        const size_t s = (size_t)kept[r];
        if (k) memcpy(tk + (size_t)r * d, k + s * d, sizeof(float) * (size_t)d);
        if (v) memcpy(tv + (size_t)r * d, v + s * d, sizeof(float) * (size_t)d);
        if (score) ts[r] = score[s];
        if (pos) tp[r] = pos[s];
    }
    if (k) memcpy(k, tk, sizeof(float) * (size_t)n_kept * d);
    if (v) memcpy(v, tv, sizeof(float) * (size_t)n_kept * d);
    if (score) memcpy(score, ts, sizeof(double) * (size_t)n_kept);
    if (pos) memcpy(pos, tp, sizeof(int32_t) * (size_t)n_kept);
    free(tk); free(tv); free(ts); free(tp);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Cosine similarity of every context embedding with every query embedding
 * (Sec. 3.3; App. C.6):  sim[q][t] = <e_t,u_q> / max(|e_t| |u_q|, eps).
 * emb [N][D], qry [nq][D], sim [nq][N].                                     */
int oracle_cosine(const float *emb, const float *qry, int64_t N, int D, int nq,
                  double eps, double *sim)
{
    if (N < 0 || D <= 0 || nq <= 0) return -1;
    for (int qi = 0; qi < nq; ++qi) {
        const float *u = qry + (size_t)qi * D;
        double un = 0.0;
        for (int c = 0; c < D; ++c) un += (double)u[c] * (double)u[c];
        un = sqrt(un);
#pragma omp parallel for schedule(static)
        for (int64_t t = 0; t < N; ++t) {
            const float *e = emb + (size_t)t * D;
            double dot = 0.0, en = 0.0;
            for (int c = 0; c < D; ++c) {
                dot += (double)e[c] * (double)u[c];
                en += (double)e[c] * (double)e[c];
            }
            double den = sqrt(en) * un;
            if (den < eps) den = eps;
            sim[(size_t)qi * N + t] = dot / den;
        }
    }
    return 0;
}

/* Union of the per-query top-k lists, each index widened by +-radius
 * (clipped to [0,N)), plus the forced first n_head and last n_tail rows
 * (Sec. 3.3: the first and last tokens are always kept; the neighbourhood
 * keeps gathered spans contiguous).  Output ascending, no duplicates.
 * topk [nq][k];  out has room for N entries.  Returns the count or -1.      */
int64_t oracle_union_dilate(const int32_t *topk, int nq, int64_t k, int64_t N,
                            int radius, int64_t n_head, int64_t n_tail, int32_t *out)
{
    if (nq < 0 || k < 0 || N < 0 || radius < 0 || n_head < 0 || n_tail < 0) return -1;
    size_t total = (size_t)nq * (size_t)k * (size_t)(2 * radius + 1) +
                   (size_t)n_head + (size_t)n_tail;
    int32_t *all = (int32_t *)malloc(sizeof(int32_t) * (total ? total : 1));
    if (!all) return -2;
    size_t m = 0;
    for (int qi = 0; qi < nq; ++qi)
        for (int64_t r = 0; r < k; ++r) {
            const int64_t t = topk[(size_t)qi * k + r];
            for (int64_t dlt = -radius; dlt <= radius; ++dlt) {
                const int64_t u = t + dlt;
                if (u >= 0 && u < N) all[m++] = (int32_t)u;
            }
        }
    for (int64_t t = 0; t < n_head && t < N; ++t) all[m++] = (int32_t)t;
    for (int64_t t = 0; t < n_tail && t < N; ++t) all[m++] = (int32_t)(N - 1 - t);
    qsort(all, m, sizeof(int32_t), cmp_i32);
    int64_t cnt = 0;
    for (size_t a = 0; a < m; ++a)
        if (a == 0 || all[a] != all[a - 1]) out[cnt++] = all[a];
    free(all);
    return cnt;
}

/* ------------------------------------------------------------------------ */
/* Significance score of Sec. 3.3 ("Identification of significant inputs"):
 * the similarities are first max-pooled over the query tokens, so that each
 * context token has one score, and then each token's score is max-pooled
 * with its adjacent tokens -- 128 of them, i.e. a centred window of 129
 * (Sec. 4.5 "Pooling kernel size"; Table 6a compares windows 5, 17, 129).
 *   s_t      = max_q sim[q][t]
 *   pooled_t = max { s_u : |u - t| <= (window-1)/2, 0 <= u < N }
 * Reading: the window is clipped at the two ends of the context (no padding
 * value takes part in the maximum).  sim [nq][N], pooled [N]; window odd.   */
int oracle_pool_scores(const double *sim, int nq, int64_t N, int window, double *pooled)
{
    if (nq <= 0 || N < 0 || window < 1 || (window % 2) == 0) return -1;
    const int64_t h = (window - 1) / 2;
    double *s = (double *)malloc(sizeof(double) * (size_t)(N ? N : 1));
    if (!s) return -2;
    for (int64_t t = 0; t < N; ++t) {
        double m = sim[t];
        for (int qi = 1; qi < nq; ++qi)
            if (sim[(size_t)qi * N + t] > m) m = sim[(size_t)qi * N + t];
        s[t] = m;
    }
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < N; ++t) {
        const int64_t lo = t - h < 0 ? 0 : t - h;
        const int64_t hi = t + h > N - 1 ? N - 1 : t + h;
        double m = s[lo];
        for (int64_t u = lo + 1; u <= hi; ++u)
            if (s[u] > m) m = s[u];
        pooled[t] = m;
    }
    free(s);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* One segment of the cross-layer context embedding (Sec. 3.2 "Combining
 * multiple heads": e_comb = concat{ e_i / ||e_i|| : i in selected heads };
 * Alg. 1 `emb.SaveSelected(qkv)`): the selected head's state of every token
 * of the chunk, L2-normalised, written into columns [col, col+d) of the
 * tokens' embedding rows.
 * Reading: a zero vector has no direction; the norm is clamped from below by
 * eps, so it stays zero instead of producing NaN.
 * src: n_rows vectors of d floats, src_stride floats apart;
 * emb: rows of emb_stride doubles; the segment of row r is emb[r*emb_stride+col ..].  */
int oracle_embed_segment(const float *src, int64_t n_rows, int d, int64_t src_stride,
                         double *emb, int64_t emb_stride, int64_t col, double eps)
{
    if (n_rows < 0 || d <= 0 || col < 0 || col + d > emb_stride || !(eps > 0.0)) return -1;
    for (int64_t r = 0; r < n_rows; ++r) {
        const float *x = src + (size_t)r * src_stride;
        double ss = 0.0;
        for (int c = 0; c < d; ++c) ss += (double)x[c] * (double)x[c];
        double nrm = sqrt(ss);
        if (nrm < eps) nrm = eps;
        double *e = emb + (size_t)r * emb_stride + col;
        for (int c = 0; c < d; ++c) e[c] = (double)x[c] / nrm;
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Position reassignment after compression (Sec. 3.1: after compression the
 * tokens of the compressed cache get consecutive position ids).  For a cache
 * that stores rotary-embedded keys this means: the key that sat at slot
 * kept[r] (position id kept[r] under the numbering of the chunk just
 * forwarded) now sits at slot r and must carry position id r, i.e. it is
 * rotated by delta = r - kept[r] <= 0 positions.
 * Reading (the paper names no rotary convention): the half-split pairing of
 * the models it evaluates (Mistral, Qwen2.5): element c is paired with
 * element c + rot/2, c in [0, rot/2), frequency theta^(-2c/rot); elements
 * beyond `rot` are not rotated:
 *     x'_c       = x_c cos(a) - x_{c+rot/2} sin(a)
 *     x'_{c+rot/2} = x_{c+rot/2} cos(a) + x_c sin(a),   a = delta * theta^(-2c/rot)
 * k: rows already compacted, [n_rows][d] floats of one head; kept [n_rows];
 * out [n_rows][d] doubles.                                                   */
int oracle_rerotate_keys(const float *k, const int32_t *kept, int64_t n_rows, int d, int rot,
                         double theta, double *out)
{
    if (n_rows < 0 || d <= 0 || rot < 0 || rot > d || (rot % 2) || !(theta > 0.0)) return -1;
    const int half = rot / 2;
    for (int64_t r = 0; r < n_rows; ++r) {
        const float *x = k + (size_t)r * d;
        double *y = out + (size_t)r * d;
        const double delta = (double)r - (double)kept[r];
        for (int c = 0; c < d; ++c) y[c] = (double)x[c];
        for (int c = 0; c < half; ++c) {
            const double a = delta * pow(theta, -2.0 * (double)c / (double)rot);
            const double cs = cos(a), sn = sin(a);
            const double x0 = (double)x[c], x1 = (double)x[c + half];
            y[c] = x0 * cs - x1 * sn;
            y[c + half] = x1 * cs + x0 * sn;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Gathering the inputs that are recomputed (Sec. 3.3 "On-Demand Cache
 * Recomputation"; Alg. 1 `relevant_inputs <- GatherRelevant(input, emb)`):
 * the rows of the input-embedding table named by the selected token indices,
 * in the given (ascending) order.  table [n_table][row_bytes] raw bytes,
 * out [n_idx][row_bytes].  Returns 0, or -1 on an index outside the table.   */
int oracle_gather_rows(const unsigned char *table, int64_t n_table, int64_t row_bytes,
                       const int32_t *idx, int64_t n_idx, unsigned char *out)
{
    if (n_table < 0 || row_bytes <= 0 || n_idx < 0) return -1;
    for (int64_t i = 0; i < n_idx; ++i) {
        if (idx[i] < 0 || idx[i] >= n_table) return -1;
        memcpy(out + (size_t)i * row_bytes, table + (size_t)idx[i] * row_bytes, (size_t)row_bytes);
    }
    return 0;
}
