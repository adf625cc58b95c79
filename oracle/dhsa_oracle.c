/*
 * DHSA prefill oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, fp64 CPU statement of what the DHSA prefill path computes
 * (Dynamic Hierarchical Sparse Attention, arXiv 2510.24606).  Only the tests,
 * the smoke check and the benchmark's cpu_baseline leg may call it; the HIP
 * library never does, and shares no code, header, table or helper with it.
 *
 * Every function follows the paper's steps in the paper's order and notation:
 *   pooling            Sec. 3.3, Eq. 4 (restated in App. D, ablation paragraph)
 *   chunk similarity   Sec. 3.3 (S_c = Q_c K_c^T, unscaled); Alg. 1 step "chunk-level similarity"
 *   ranking/selection  Sec. 3.1 Step 2; Alg. 1 loop over ranked chunks, clip, append,
 *                      stop at >= N_b, hard truncate, sort
 *   attention          Alg. 2 (gather + {0,-inf} causal mask + softmax) and
 *                      Alg. 3 (tiled online softmax); App. C "Backend implementations"
 *   boundary finalisation  Sec. 3.2 "Inference Pipeline"; App. "Inference of the Boundary
 *                      Predictor": threshold, sort by score, greedy non-maximum suppression
 *   recall diagnostic  App. "Theoretical Analysis", Setup and Notation: per-row recall of a
 *                      selected set against the top-k keys by attention score
 *
 * Readings taken where the paper is silent or has two forms:
 *   - queries are pooled over the same dynamic chunks as keys (Sec. 3.1/3.3), and
 *     the index set is built per query ROW: Alg. 1 with q_max = i + 1 for row i,
 *     scores taken from the row's chunk;
 *   - Argsort is stable: equal scores -> lower chunk id first (hence lower key index);
 *   - GQA: routing per query head h against the pooled keys of kv-head h / G;
 *   - floating point: all sums in fp64 over the exactly-upcast inputs.
 * The functions whose names end in _blocks state Alg. 1 as printed instead: queries
 * pooled over fixed row blocks of B_r rows (q_i = sqrt(B_r) AvgPool(Q_i), the mean
 * taken over the rows the block really has), one index list per row block with
 * q_max = the block's end, every key chunk ranked, and the causal mask applied
 * per token inside attention (Alg. 2 / Alg. 3); a row that sees none of its
 * block's keys gets zeros.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py (closed
 * forms, brute force on tiny inputs, library special cases).  The paper prints
 * no worked numeric example, so end-to-end values are pinned only through those.
 *
 * Layout: X[h][i][d] with d contiguous (float, the exact upcast of the
 * workload's values); B[0..N_c] int32 with B[0] = 0 < ... < B[N_c] = L; chunk k
 * holds tokens [B[k], B[k+1]).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define API __attribute__((visibility("default")))

API int dhsa_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- Sec. 3.3, Eq. 4: x_{C_k} = (sqrt(len_k) / len_k) * sum_{i in [b_k, b_{k+1})} x_i ---- */
API int dhsa_oracle_pool(const float *X, int H, int64_t L, int D, const int32_t *B, int N_c,
                         double *Xc /* [H][N_c][D] */) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int h = 0; h < H; ++h) {
        for (int k = 0; k < N_c; ++k) {
            double len = (double)(B[k + 1] - B[k]);
            for (int d = 0; d < D; ++d) {
                double sum = 0.0;
                for (int64_t i = B[k]; i < B[k + 1]; ++i)
                    sum += (double)X[((int64_t)h * L + i) * D + d];
                Xc[((int64_t)h * N_c + k) * D + d] = (sqrt(len) / len) * sum;
            }
        }
    }
    return 0;
}

/* ---- The ablation "without robust chunk representation" (App. D): plain average
 * pooling, x_{C_k} = (1 / len_k) * sum of the chunk's vectors. ---- */
API int dhsa_oracle_pool_mean(const float *X, int H, int64_t L, int D, const int32_t *B, int N_c,
                              double *Xc /* [H][N_c][D] */) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int h = 0; h < H; ++h) {
        for (int k = 0; k < N_c; ++k) {
            double len = (double)(B[k + 1] - B[k]);
            for (int d = 0; d < D; ++d) {
                double sum = 0.0;
                for (int64_t i = B[k]; i < B[k + 1]; ++i)
                    sum += (double)X[((int64_t)h * L + i) * D + d];
                Xc[((int64_t)h * N_c + k) * D + d] = sum / len;
            }
        }
    }
    return 0;
}

/* pooling = 0: Eq. 4; 1: plain average (the ablation) */
static int pool_by_mode(int pooling, const float *X, int H, int64_t L, int D, const int32_t *B, int N_c,
                        double *Xc) {
    return pooling ? dhsa_oracle_pool_mean(X, H, L, D, B, N_c, Xc) : dhsa_oracle_pool(X, H, L, D, B, N_c, Xc);
}

/* ---- Sec. 3.3: (S_c)_{l,k} = < q_{C_l}, k_{C_k} >, one row l, every key chunk k ---- */
API int dhsa_oracle_score_row(const double *qc /* [D] */, const double *Kc /* [N_c][D] */, int N_c,
                              int D, double *S_row /* [N_c] */) {
    for (int k = 0; k < N_c; ++k) {
        double s = 0.0;
        for (int d = 0; d < D; ++d) s += qc[d] * Kc[(int64_t)k * D + d];
        S_row[k] = s;
    }
    return 0;
}

/* Full S_c for every query head; kv-head of query head h is h / G (GQA). */
API int dhsa_oracle_scores(const double *Qc /* [H_q][N_c][D] */, const double *Kc /* [H_kv][N_c][D] */,
                           int H_q, int H_kv, int N_c, int D, double *Sc /* [H_q][N_c][N_c] */) {
    int G = H_q / H_kv;
#pragma omp parallel for collapse(2) schedule(static)
    for (int h = 0; h < H_q; ++h)
        for (int l = 0; l < N_c; ++l)
            dhsa_oracle_score_row(Qc + ((int64_t)h * N_c + l) * D, Kc + (int64_t)(h / G) * N_c * D, N_c, D,
                                  Sc + ((int64_t)h * N_c + l) * N_c);
    return 0;
}

/* ---- Alg. 1, "rank key chunks by chunk-level similarity (descending)" ----
 * Stable merge sort of chunk ids by score, larger first; equal scores keep
 * ascending id (so -0.0 and +0.0 tie).  Scores are assumed finite. */
static void merge_sort_desc(const double *S, int32_t *a, int32_t *tmp, int n) {
    if (n < 2) return;
    int m = n / 2;
    merge_sort_desc(S, a, tmp, m);
    merge_sort_desc(S, a + m, tmp, n - m);
    int i = 0, j = m, o = 0;
    while (i < m && j < n) {
        if (S[a[j]] > S[a[i]]) tmp[o++] = a[j++]; /* strictly larger moves ahead */
        else tmp[o++] = a[i++];                   /* ties: left (lower id) first  */
    }
    while (i < m) tmp[o++] = a[i++];
    while (j < n) tmp[o++] = a[j++];
    memcpy(a, tmp, (size_t)n * sizeof(int32_t));
}

API int dhsa_oracle_rank(const double *S_row, int N_c, int32_t *pi /* [N_c] */) {
    int32_t *tmp = (int32_t *)malloc((size_t)N_c * sizeof(int32_t));
    if (!tmp) return 1;
    for (int k = 0; k < N_c; ++k) pi[k] = k;
    merge_sort_desc(S_row, pi, tmp, N_c);
    free(tmp);
    return 0;
}

static int cmp_i32(const void *a, const void *b) {
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* ---- Alg. 1, inner loop: walk ranked chunks, clip to q_max, append, stop at
 * >= N_b, hard-truncate to N_b, sort ascending.  Returns |I|. ---- */
API int dhsa_oracle_select(const int32_t *pi, const int32_t *B, int N_c, int64_t q_max, int N_b,
                           int32_t *I /* capacity N_b */) {
    /* the appended list may overshoot N_b by up to one chunk before truncation */
    int64_t cap = (int64_t)N_b + (int64_t)B[N_c];
    int32_t *list = (int32_t *)malloc((size_t)cap * sizeof(int32_t));
    if (!list) return -1;
    int64_t n = 0;
    for (int r = 0; r < N_c; ++r) {
        int j = pi[r];
        int64_t s = B[j], e = B[j + 1];
        if (s > q_max) s = q_max;
        if (e > q_max) e = q_max;
        if (s >= e) continue;
        for (int64_t t = s; t < e; ++t) list[n++] = (int32_t)t;
        if (n >= N_b) break;
    }
    if (n > N_b) n = N_b;
    qsort(list, (size_t)n, sizeof(int32_t), cmp_i32);
    memcpy(I, list, (size_t)n * sizeof(int32_t));
    free(list);
    return (int)n;
}

/* ---- Sec. 3.1 Step 2 read at token-pair level (second, independent form):
 * pair (i, j) inherits (S_c)_{c(i), c(j)}; j > i is masked; each row keeps its
 * N_b best pairs, larger score first, equal scores -> lower key index.
 * O(L^2 log L): tiny L only. ---- */
typedef struct { double s; int32_t j; } pair_t;
static int cmp_pair(const void *a, const void *b) {
    const pair_t *x = (const pair_t *)a, *y = (const pair_t *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->j > y->j) - (x->j < y->j);
}
API int dhsa_oracle_select_pairs(const double *Sc_h /* [N_c][N_c] */, const int32_t *B, int N_c, int N_b,
                                 int32_t *I /* [L][N_b], -1 padded */, int32_t *cnt /* [L] */) {
    int64_t L = B[N_c];
    int32_t *chunk_of = (int32_t *)malloc((size_t)L * sizeof(int32_t));
    pair_t *row = (pair_t *)malloc((size_t)L * sizeof(pair_t));
    if (!chunk_of || !row) return 1;
    for (int k = 0; k < N_c; ++k)
        for (int64_t i = B[k]; i < B[k + 1]; ++i) chunk_of[i] = k;
    for (int64_t i = 0; i < L; ++i) {
        int64_t n = 0;
        for (int64_t j = 0; j <= i; ++j) { /* j > i masked out */
            row[n].s = Sc_h[(int64_t)chunk_of[i] * N_c + chunk_of[j]];
            row[n].j = (int32_t)j;
            ++n;
        }
        qsort(row, (size_t)n, sizeof(pair_t), cmp_pair);
        if (n > N_b) n = N_b;
        for (int64_t t = 0; t < n; ++t) I[i * N_b + t] = row[t].j;
        qsort(I + i * N_b, (size_t)n, sizeof(int32_t), cmp_i32);
        for (int64_t t = n; t < N_b; ++t) I[i * N_b + t] = -1;
        cnt[i] = (int32_t)n;
    }
    free(chunk_of);
    free(row);
    return 0;
}

/* ---- Alg. 2 for one query row i: gather K[I], V[I]; mask = 0 if i >= I[v]
 * else -inf; softmax((q K_sel^T) * scale + mask) V_sel.  A row whose keys are
 * all masked gets zeros. ---- */
API int dhsa_oracle_attend_row(const float *q /* [D] */, const float *Kg /* [L][D] */,
                               const float *Vg /* [L][D] */, const int32_t *I, int cnt, int64_t i, int D,
                               double scale, double *o /* [D] */) {
    double *s = (double *)malloc((size_t)(cnt > 0 ? cnt : 1) * sizeof(double));
    if (!s) return 1;
    double m = -INFINITY;
    for (int v = 0; v < cnt; ++v) {
        double acc = 0.0;
        for (int d = 0; d < D; ++d) acc += (double)q[d] * (double)Kg[(int64_t)I[v] * D + d];
        s[v] = (i >= I[v]) ? acc * scale : -INFINITY;
        if (s[v] > m) m = s[v];
    }
    for (int d = 0; d < D; ++d) o[d] = 0.0;
    if (m == -INFINITY) { free(s); return 0; }
    double denom = 0.0;
    for (int v = 0; v < cnt; ++v) { s[v] = exp(s[v] - m); denom += s[v]; }
    for (int v = 0; v < cnt; ++v) {
        double p = s[v] / denom;
        for (int d = 0; d < D; ++d) o[d] += p * (double)Vg[(int64_t)I[v] * D + d];
    }
    free(s);
    return 0;
}

/* ---- Alg. 3 for one row block [q_s, q_e) sharing one index list: stream I in
 * column tiles of B_c, causal mask by absolute position, online (m, l, O_sum),
 * normalise at the end. ---- */
API int dhsa_oracle_attend_block_tiled(const float *Qh /* [L][D] */, const float *Kg, const float *Vg,
                                       const int32_t *I, int cnt, int64_t q_s, int64_t q_e, int D,
                                       double scale, int B_c, double *O /* [q_e-q_s][D] */) {
    int rows = (int)(q_e - q_s);
    double *m = (double *)malloc((size_t)rows * sizeof(double));
    double *l = (double *)malloc((size_t)rows * sizeof(double));
    double *S = (double *)malloc((size_t)rows * (size_t)B_c * sizeof(double));
    if (!m || !l || !S) return 1;
    for (int u = 0; u < rows; ++u) {
        m[u] = -INFINITY;
        l[u] = 0.0;
        for (int d = 0; d < D; ++d) O[(int64_t)u * D + d] = 0.0;
    }
    for (int t = 0; t < cnt; t += B_c) {
        int w = (t + B_c <= cnt) ? B_c : cnt - t;
        const int32_t *J = I + t;
        for (int u = 0; u < rows; ++u)
            for (int v = 0; v < w; ++v) {
                double acc = 0.0;
                for (int d = 0; d < D; ++d)
                    acc += (double)Qh[(q_s + u) * D + d] * (double)Kg[(int64_t)J[v] * D + d];
                S[(int64_t)u * B_c + v] = ((q_s + u) < J[v]) ? -INFINITY : acc * scale;
            }
        for (int u = 0; u < rows; ++u) {
            double m_new = m[u];
            for (int v = 0; v < w; ++v)
                if (S[(int64_t)u * B_c + v] > m_new) m_new = S[(int64_t)u * B_c + v];
            if (m_new == -INFINITY) continue; /* nothing visible yet */
            double alpha = exp(m[u] - m_new);
            double rowsum = 0.0;
            for (int d = 0; d < D; ++d) O[(int64_t)u * D + d] *= alpha;
            for (int v = 0; v < w; ++v) {
                double p = exp(S[(int64_t)u * B_c + v] - m_new);
                rowsum += p;
                for (int d = 0; d < D; ++d) O[(int64_t)u * D + d] += p * (double)Vg[(int64_t)J[v] * D + d];
            }
            l[u] = l[u] * alpha + rowsum;
            m[u] = m_new;
        }
    }
    for (int u = 0; u < rows; ++u)
        for (int d = 0; d < D; ++d) O[(int64_t)u * D + d] = (l[u] > 0.0) ? O[(int64_t)u * D + d] / l[u] : 0.0;
    free(m); free(l); free(S);
    return 0;
}

/* ---- Chunk-level view of the Alg. 1 walk for query chunk l (all its rows share
 * the ranking; they differ only in how much of chunk l itself is visible).
 * For each key chunk k <= l: where it sits relative to chunk l in the ranking
 * (0 before, 1 = chunk l itself, 2 after) and how many tokens of OTHER visible
 * chunks were appended before the walk reaches it.  Row i (with v = i+1-b_l
 * visible tokens of chunk l) has appended before[k] + (pos[k]==2 ? v : 0)
 * tokens when it reaches chunk k.  Chunks k > l are never visible: pos = 3. ---- */
API int dhsa_oracle_chunk_walk(const int32_t *pi, const int32_t *B, int N_c, int l,
                               int32_t *before /* [N_c] */, int8_t *pos /* [N_c] */) {
    int64_t appended = 0;
    int seen_l = 0;
    for (int r = 0; r < N_c; ++r) {
        int k = pi[r];
        if (k > l) { before[k] = -1; pos[k] = 3; continue; }
        before[k] = (int32_t)appended;
        if (k == l) { pos[k] = 1; seen_l = 1; }
        else { pos[k] = seen_l ? 2 : 0; appended += B[k + 1] - B[k]; }
    }
    return 0;
}

/* ---- Drivers ------------------------------------------------------------ */

static int chunk_of_row(const int32_t *B, int N_c, int64_t i) {
    int lo = 0, hi = N_c; /* B[lo] <= i < B[hi] */
    while (hi - lo > 1) {
        int mid = (lo + hi) / 2;
        if (B[mid] <= i) lo = mid; else hi = mid;
    }
    return lo;
}

/* Routing for a list of rows, every query head: I_{h,i} = Alg. 1 with
 * q_max = i + 1 and the scores of row i's chunk.  Optionally also the per-rank
 * scores are not returned; only index sets. */
API int dhsa_oracle_route_rows(const float *Q, const float *K, int H_q, int H_kv, int64_t L, int D,
                               const int32_t *B, int N_c, int N_b, int pooling, const int64_t *rows, int n_rows,
                               int32_t *I_out /* [H_q][n_rows][N_b], -1 padded */,
                               int32_t *cnt_out /* [H_q][n_rows] */) {
    int G = H_q / H_kv;
    double *Qc = (double *)malloc((size_t)H_q * N_c * D * sizeof(double));
    double *Kc = (double *)malloc((size_t)H_kv * N_c * D * sizeof(double));
    if (!Qc || !Kc) return 1;
    pool_by_mode(pooling, Q, H_q, L, D, B, N_c, Qc);
    pool_by_mode(pooling, K, H_kv, L, D, B, N_c, Kc);
    int err = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int h = 0; h < H_q; ++h)
        for (int t = 0; t < n_rows; ++t) {
            int64_t i = rows[t];
            int l = chunk_of_row(B, N_c, i);
            double *S_row = (double *)malloc((size_t)N_c * sizeof(double));
            int32_t *pi = (int32_t *)malloc((size_t)N_c * sizeof(int32_t));
            if (!S_row || !pi) { err = 1; free(S_row); free(pi); continue; }
            dhsa_oracle_score_row(Qc + ((int64_t)h * N_c + l) * D, Kc + (int64_t)(h / G) * N_c * D, N_c, D, S_row);
            dhsa_oracle_rank(S_row, N_c, pi);
            int32_t *I = I_out + ((int64_t)h * n_rows + t) * N_b;
            int n = dhsa_oracle_select(pi, B, N_c, i + 1, N_b, I);
            if (n < 0) { err = 1; n = 0; }
            for (int x = n; x < N_b; ++x) I[x] = -1;
            cnt_out[(int64_t)h * n_rows + t] = n;
            free(S_row); free(pi);
        }
    free(Qc); free(Kc);
    return err;
}

/* The whole path for a list of rows: route (above), then Alg. 2 per row. */
API int dhsa_oracle_prefill_rows(const float *Q, const float *K, const float *V, int H_q, int H_kv,
                                 int64_t L, int D, const int32_t *B, int N_c, int N_b, int pooling, double scale,
                                 const int64_t *rows, int n_rows, double *O_out /* [H_q][n_rows][D] */,
                                 int32_t *I_out /* [H_q][n_rows][N_b] */, int32_t *cnt_out) {
    int G = H_q / H_kv;
    int err = dhsa_oracle_route_rows(Q, K, H_q, H_kv, L, D, B, N_c, N_b, pooling, rows, n_rows, I_out, cnt_out);
    if (err) return err;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int h = 0; h < H_q; ++h)
        for (int t = 0; t < n_rows; ++t) {
            int64_t i = rows[t];
            int g = h / G;
            if (dhsa_oracle_attend_row(Q + ((int64_t)h * L + i) * D, K + (int64_t)g * L * D,
                                       V + (int64_t)g * L * D, I_out + ((int64_t)h * n_rows + t) * N_b,
                                       cnt_out[(int64_t)h * n_rows + t], i, D, scale,
                                       O_out + ((int64_t)h * n_rows + t) * D))
                err = 1;
        }
    return err;
}

/* Chunk-level walk state for every query chunk of one query head (used to
 * check a compact routing plan on ALL rows at full size): rem[l][k] = N_b -
 * before[k] for the walk of query chunk l; pos as in dhsa_oracle_chunk_walk.
 * Also, per query chunk, the smallest score gap between two adjacently ranked
 * visible chunks whose order can change some row's index set (near-tie
 * accounting): a pair (r, r+1) matters iff some row takes a token of rank r and
 * not every row takes both chunks whole. */
API int dhsa_oracle_plan_head(const double *Qc_h /* [N_c][D] */, const double *Kc_g /* [N_c][D] */,
                              const int32_t *B, int N_c, int D, int N_b,
                              int32_t *rem /* [N_c][N_c] */, int8_t *pos /* [N_c][N_c] */,
                              double *cut_gap /* [N_c] */) {
    int err = 0;
#pragma omp parallel for schedule(dynamic, 4)
    for (int l = 0; l < N_c; ++l) {
        double *S_row = (double *)malloc((size_t)N_c * sizeof(double));
        int32_t *pi = (int32_t *)malloc((size_t)N_c * sizeof(int32_t));
        int32_t *before = (int32_t *)malloc((size_t)N_c * sizeof(int32_t));
        if (!S_row || !pi || !before) { err = 1; free(S_row); free(pi); free(before); continue; }
        dhsa_oracle_score_row(Qc_h + (int64_t)l * D, Kc_g, N_c, D, S_row);
        dhsa_oracle_rank(S_row, N_c, pi);
        int8_t *pos_l = pos + (int64_t)l * N_c;
        dhsa_oracle_chunk_walk(pi, B, N_c, l, before, pos_l);
        for (int k = 0; k < N_c; ++k) rem[(int64_t)l * N_c + k] = (pos_l[k] == 3) ? 0 : N_b - before[k];
        /* near-tie accounting over the visible chunks in rank order */
        int len_l = B[l + 1] - B[l];
        double gap = INFINITY;
        int prev = -1;
        for (int r = 0; r < N_c; ++r) {
            int k = pi[r];
            if (k > l) continue;
            if (prev >= 0) {
                /* tokens of `prev` and `k` taken by the first (v=1) and last (v=len_l) row */
                int any_prev = 0, full_both = 1;
                for (int e = 0; e < 2; ++e) {
                    int v = e ? len_l : 1;
                    int64_t room_p = (int64_t)N_b - before[prev] - (pos_l[prev] == 2 ? v : 0);
                    int64_t room_k = (int64_t)N_b - before[k] - (pos_l[k] == 2 ? v : 0);
                    int64_t len_p = (prev == l) ? v : B[prev + 1] - B[prev];
                    int64_t len_k = (k == l) ? v : B[k + 1] - B[k];
                    if (room_p > 0) any_prev = 1;
                    if (room_p < len_p || room_k < len_k) full_both = 0;
                }
                if (any_prev && !full_both) {
                    double g = fabs(S_row[prev] - S_row[k]);
                    if (g < gap) gap = g;
                }
            }
            prev = k;
        }
        cut_gap[l] = gap;
        free(S_row); free(pi); free(before);
    }
    return err;
}


/* ======================= Alg. 1 as printed: fixed row blocks ======================= */

/* ---- Alg. 1 step "row-block query representations": q_i = sqrt(B_r) * AvgPool(Q_i),
 * Q_i = Q[i B_r : min((i+1) B_r, L)).  AvgPool is the mean over the rows the block has
 * (the last block may be short); the factor is sqrt of the nominal B_r as printed. ---- */
API int dhsa_oracle_pool_blocks(const float *X, int H, int64_t L, int D, int B_r,
                                double *Xq /* [H][N_r][D] */) {
    int64_t N_r = (L + B_r - 1) / B_r;
#pragma omp parallel for collapse(2) schedule(static)
    for (int h = 0; h < H; ++h) {
        for (int64_t i = 0; i < N_r; ++i) {
            int64_t q_s = i * B_r, q_e = (i + 1) * B_r < L ? (i + 1) * B_r : L;
            for (int d = 0; d < D; ++d) {
                double sum = 0.0;
                for (int64_t r = q_s; r < q_e; ++r) sum += (double)X[((int64_t)h * L + r) * D + d];
                Xq[((int64_t)h * N_r + i) * D + d] = sqrt((double)B_r) * (sum / (double)(q_e - q_s));
            }
        }
    }
    return 0;
}

/* Plain average of a row block (the ablation without the sqrt(B_r) factor of the robust representation). */
API int dhsa_oracle_pool_blocks_mean(const float *X, int H, int64_t L, int D, int B_r,
                                     double *Xq /* [H][N_r][D] */) {
    int64_t N_r = (L + B_r - 1) / B_r;
#pragma omp parallel for collapse(2) schedule(static)
    for (int h = 0; h < H; ++h) {
        for (int64_t i = 0; i < N_r; ++i) {
            int64_t q_s = i * B_r, q_e = (i + 1) * B_r < L ? (i + 1) * B_r : L;
            for (int d = 0; d < D; ++d) {
                double sum = 0.0;
                for (int64_t r = q_s; r < q_e; ++r) sum += (double)X[((int64_t)h * L + r) * D + d];
                Xq[((int64_t)h * N_r + i) * D + d] = sum / (double)(q_e - q_s);
            }
        }
    }
    return 0;
}

/* ---- Alg. 1 for one row block i of one head: S_c[i, :] over ALL key chunks,
 * Argsort (stable, descending), walk with q_max = min((i+1) B_r, L).  Returns |I_i|. ---- */
API int dhsa_oracle_select_block(const double *q_i /* [D] */, const double *Kc_g /* [N_c][D] */,
                                 const int32_t *B, int N_c, int D, int64_t q_max, int N_b,
                                 int32_t *I /* capacity N_b */) {
    double *S_row = (double *)malloc((size_t)N_c * sizeof(double));
    int32_t *pi = (int32_t *)malloc((size_t)N_c * sizeof(int32_t));
    if (!S_row || !pi) { free(S_row); free(pi); return -1; }
    dhsa_oracle_score_row(q_i, Kc_g, N_c, D, S_row);
    int n = dhsa_oracle_rank(S_row, N_c, pi) ? -1 : dhsa_oracle_select(pi, B, N_c, q_max, N_b, I);
    free(S_row); free(pi);
    return n;
}

/* ---- Second, independent form of the block selection (tiny L): every key token
 * j < q_max inherits the score of (row block i, chunk of j); keep the N_b best,
 * larger score first, equal scores -> lower key index; sort ascending. ---- */
API int dhsa_oracle_select_pairs_blocks(const double *Sb_h /* [N_r][N_c] */, const int32_t *B, int N_c,
                                        int B_r, int N_b, int32_t *I /* [N_r][N_b], -1 padded */,
                                        int32_t *cnt /* [N_r] */) {
    int64_t L = B[N_c];
    int64_t N_r = (L + B_r - 1) / B_r;
    int32_t *chunk_of = (int32_t *)malloc((size_t)L * sizeof(int32_t));
    pair_t *row = (pair_t *)malloc((size_t)L * sizeof(pair_t));
    if (!chunk_of || !row) return 1;
    for (int k = 0; k < N_c; ++k)
        for (int64_t j = B[k]; j < B[k + 1]; ++j) chunk_of[j] = k;
    for (int64_t i = 0; i < N_r; ++i) {
        int64_t q_max = (i + 1) * B_r < L ? (i + 1) * B_r : L;
        int64_t n = 0;
        for (int64_t j = 0; j < q_max; ++j) {
            row[n].s = Sb_h[i * N_c + chunk_of[j]];
            row[n].j = (int32_t)j;
            ++n;
        }
        qsort(row, (size_t)n, sizeof(pair_t), cmp_pair);
        if (n > N_b) n = N_b;
        for (int64_t t = 0; t < n; ++t) I[i * N_b + t] = row[t].j;
        qsort(I + i * N_b, (size_t)n, sizeof(int32_t), cmp_i32);
        for (int64_t t = n; t < N_b; ++t) I[i * N_b + t] = -1;
        cnt[i] = (int32_t)n;
    }
    free(chunk_of);
    free(row);
    return 0;
}

/* Index lists of a list of row blocks, every query head (GQA as above). */
API int dhsa_oracle_route_blocks(const float *Q, const float *K, int H_q, int H_kv, int64_t L, int D,
                                 const int32_t *B, int N_c, int B_r, int N_b, int pooling, const int64_t *blocks,
                                 int n_blocks, int32_t *I_out /* [H_q][n_blocks][N_b], -1 padded */,
                                 int32_t *cnt_out /* [H_q][n_blocks] */) {
    int G = H_q / H_kv;
    int64_t N_r = (L + B_r - 1) / B_r;
    double *Qb = (double *)malloc((size_t)H_q * N_r * D * sizeof(double));
    double *Kc = (double *)malloc((size_t)H_kv * N_c * D * sizeof(double));
    if (!Qb || !Kc) return 1;
    if (pooling) dhsa_oracle_pool_blocks_mean(Q, H_q, L, D, B_r, Qb);
    else dhsa_oracle_pool_blocks(Q, H_q, L, D, B_r, Qb);
    pool_by_mode(pooling, K, H_kv, L, D, B, N_c, Kc);
    int err = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int h = 0; h < H_q; ++h)
        for (int t = 0; t < n_blocks; ++t) {
            int64_t i = blocks[t];
            int64_t q_max = (i + 1) * B_r < L ? (i + 1) * B_r : L;
            int32_t *I = I_out + ((int64_t)h * n_blocks + t) * N_b;
            int n = dhsa_oracle_select_block(Qb + ((int64_t)h * N_r + i) * D, Kc + (int64_t)(h / G) * N_c * D, B,
                                             N_c, D, q_max, N_b, I);
            if (n < 0) { err = 1; n = 0; }
            for (int x = n; x < N_b; ++x) I[x] = -1;
            cnt_out[(int64_t)h * n_blocks + t] = n;
        }
    free(Qb); free(Kc);
    return err;
}

/* The whole block-form path for a list of rows: the index list of each row's
 * block (Alg. 1), then Alg. 2 for the row with its causal mask. */
API int dhsa_oracle_prefill_rows_blocks(const float *Q, const float *K, const float *V, int H_q, int H_kv,
                                        int64_t L, int D, const int32_t *B, int N_c, int B_r, int N_b,
                                        int pooling, double scale, const int64_t *rows, int n_rows,
                                        double *O_out /* [H_q][n_rows][D] */,
                                        int32_t *I_out /* [H_q][n_rows][N_b]: the list of the row's block */,
                                        int32_t *cnt_out) {
    int G = H_q / H_kv;
    int64_t *blocks = (int64_t *)malloc((size_t)(n_rows > 0 ? n_rows : 1) * sizeof(int64_t));
    if (!blocks) return 1;
    for (int t = 0; t < n_rows; ++t) blocks[t] = rows[t] / B_r;
    int err = dhsa_oracle_route_blocks(Q, K, H_q, H_kv, L, D, B, N_c, B_r, N_b, pooling, blocks, n_rows, I_out,
                                       cnt_out);
    free(blocks);
    if (err) return err;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int h = 0; h < H_q; ++h)
        for (int t = 0; t < n_rows; ++t) {
            int64_t i = rows[t];
            int g = h / G;
            if (dhsa_oracle_attend_row(Q + ((int64_t)h * L + i) * D, K + (int64_t)g * L * D,
                                       V + (int64_t)g * L * D, I_out + ((int64_t)h * n_rows + t) * N_b,
                                       cnt_out[(int64_t)h * n_rows + t], i, D, scale,
                                       O_out + ((int64_t)h * n_rows + t) * D))
                err = 1;
        }
    return err;
}

/* Per row block of one query head: how many tokens of each key chunk the block's
 * list holds (they are the chunk's first take[i][k] tokens; 0 = not listed), for
 * checking a compact plan on ALL blocks at full size; and the smallest score gap
 * between two adjacently ranked visible chunks whose order changes the list
 * (rank r is taken and ranks r, r+1 are not both taken whole). */
API int dhsa_oracle_plan_blocks_head(const double *Qb_h /* [N_r][D] */, const double *Kc_g /* [N_c][D] */,
                                     const int32_t *B, int N_c, int D, int B_r, int N_b,
                                     int32_t *take /* [N_r][N_c] */, double *cut_gap /* [N_r] */) {
    int64_t L = B[N_c];
    int64_t N_r = (L + B_r - 1) / B_r;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t i = 0; i < N_r; ++i) {
        double *S_row = (double *)malloc((size_t)N_c * sizeof(double));
        int32_t *pi = (int32_t *)malloc((size_t)N_c * sizeof(int32_t));
        if (!S_row || !pi) { err = 1; free(S_row); free(pi); continue; }
        int64_t q_max = (i + 1) * B_r < L ? (i + 1) * B_r : L;
        dhsa_oracle_score_row(Qb_h + i * D, Kc_g, N_c, D, S_row);
        dhsa_oracle_rank(S_row, N_c, pi);
        int32_t *tk = take + i * N_c;
        for (int k = 0; k < N_c; ++k) tk[k] = 0;
        int64_t appended = 0;
        double gap = INFINITY;
        int prev = -1;
        int64_t prev_len = 0, prev_take = 0;
        for (int r = 0; r < N_c; ++r) {
            int k = pi[r];
            int64_t s = B[k] < q_max ? B[k] : q_max, e = B[k + 1] < q_max ? B[k + 1] : q_max;
            if (s >= e) continue;
            int64_t room = (int64_t)N_b - appended;
            int64_t t = room <= 0 ? 0 : (room < e - s ? room : e - s);
            tk[k] = (int32_t)t;
            if (prev >= 0 && prev_take > 0 && !(prev_take == prev_len && t == e - s)) {
                double g = fabs(S_row[prev] - S_row[k]);
                if (g < gap) gap = g;
            }
            prev = k; prev_len = e - s; prev_take = t;
            appended += e - s;
        }
        cut_gap[i] = gap;
        free(S_row); free(pi);
    }
    return err;
}


/* ======================= Boundary finalisation (threshold + NMS) ======================= */

/* ---- Sec. 3.2 "Inference Pipeline" / App. "Inference of the Boundary Predictor":
 * p[i] is the predictor's score that position i marks the END of a chunk.
 *   1. candidates: the positions whose score exceeds the threshold tau (strictly);
 *   2. sort the candidates by score, descending (equal scores: lower position first);
 *   3. starting with the best, mark a candidate as a boundary and remove every other
 *      candidate within W tokens of it (0 < |j - i| <= W); go on with the best remaining.
 * The boundary set is returned in the half-open convention the rest of the path uses:
 * a chunk that ends at position i ends at index i + 1, so B = {0} u {i + 1 : i kept} u {L},
 * ascending, without repeats (the end of the sequence is always a chunk end).
 * Returns N_c (B has N_c + 1 entries; capacity L + 1), or -1. ---- */
typedef struct { float s; int32_t i; } cand_t;
static void merge_sort_cand(cand_t *a, cand_t *tmp, int64_t n) {
    if (n < 2) return;
    int64_t m = n / 2;
    merge_sort_cand(a, tmp, m);
    merge_sort_cand(a + m, tmp, n - m);
    int64_t i = 0, j = m, o = 0;
    while (i < m && j < n) {
        if (a[j].s > a[i].s) tmp[o++] = a[j++]; /* strictly larger score moves ahead */
        else tmp[o++] = a[i++];                 /* ties: left (lower position) first */
    }
    while (i < m) tmp[o++] = a[i++];
    while (j < n) tmp[o++] = a[j++];
    memcpy(a, tmp, (size_t)n * sizeof(cand_t));
}

API int64_t dhsa_oracle_finalize_boundaries(const float *p, int64_t L, double tau, int W,
                                            int32_t *B /* capacity L + 1 */) {
    cand_t *cand = (cand_t *)malloc((size_t)(L > 0 ? L : 1) * sizeof(cand_t));
    cand_t *tmp = (cand_t *)malloc((size_t)(L > 0 ? L : 1) * sizeof(cand_t));
    char *removed = (char *)calloc((size_t)(L > 0 ? L : 1), 1);
    char *kept = (char *)calloc((size_t)(L > 0 ? L : 1), 1);
    if (!cand || !tmp || !removed || !kept) { free(cand); free(tmp); free(removed); free(kept); return -1; }
    int64_t n = 0;
    for (int64_t i = 0; i < L; ++i)
        if ((double)p[i] > tau) { cand[n].s = p[i]; cand[n].i = (int32_t)i; ++n; }
    merge_sort_cand(cand, tmp, n);
    for (int64_t r = 0; r < n; ++r) {
        int64_t i = cand[r].i;
        if (removed[i]) continue;
        kept[i] = 1;
        int64_t lo = i - W < 0 ? 0 : i - W, hi = i + W > L - 1 ? L - 1 : i + W;
        for (int64_t j = lo; j <= hi; ++j)
            if (j != i) removed[j] = 1;
    }
    int64_t m = 0;
    B[m++] = 0;
    for (int64_t i = 0; i + 1 < L; ++i)
        if (kept[i]) B[m++] = (int32_t)(i + 1);
    B[m++] = (int32_t)L;
    free(cand); free(tmp); free(removed); free(kept);
    return m - 1;
}


/* ======================= Recall against exact top-k attention ======================= */

/* ---- App. "Theoretical Analysis" (Setup and Notation), per-row recall:
 * I*_i = the k keys j <= i with the largest attention scores a_ij (a_ij = exp of
 * the logit, so: the largest logits q_i . k_j; equal logits -> lower index),
 * k = min(k_top, i + 1); Recall_i = |I*_i n I_hat_i| / |I*_i| for a selected set
 * I_hat_i.  Returns |I*_i n I_hat_i| in *hits and |I*_i| in *size.  Logits are
 * summed in fp64 in the order d = 0, 1, ...: the products of the stored values
 * are exact in fp64, so this is the value any fp64 evaluation in that order has. ---- */
API int dhsa_oracle_recall_row(const float *q /* [D] */, const float *Kg /* [L][D] */, int64_t i, int D,
                               const int32_t *I_hat, int cnt, int k_top, int32_t *hits, int32_t *size) {
    int64_t n = i + 1;
    pair_t *row = (pair_t *)malloc((size_t)n * sizeof(pair_t));
    char *in_top = (char *)calloc((size_t)n, 1);
    if (!row || !in_top) { free(row); free(in_top); return 1; }
    for (int64_t j = 0; j < n; ++j) {
        double acc = 0.0;
        for (int d = 0; d < D; ++d) acc += (double)q[d] * (double)Kg[j * D + d];
        row[j].s = acc;
        row[j].j = (int32_t)j;
    }
    qsort(row, (size_t)n, sizeof(pair_t), cmp_pair);   /* logit descending, equal logits by lower index */
    int64_t k = k_top < n ? k_top : n;
    for (int64_t t = 0; t < k; ++t) in_top[row[t].j] = 1;
    int32_t h = 0;
    for (int v = 0; v < cnt; ++v)
        if (I_hat[v] >= 0 && I_hat[v] < n && in_top[I_hat[v]]) ++h;
    *hits = h;
    *size = (int32_t)k;
    free(row); free(in_top);
    return 0;
}

/* Recall of the routed sets of a list of rows of one query head (row form: the row's
 * own set; row-block form, B_r > 0: the keys of its block's list at or below the row). */
API int dhsa_oracle_recall_rows(const float *Q, const float *K, int H_q, int H_kv, int64_t L, int D,
                                const int32_t *B, int N_c, int B_r, int N_b, int pooling, int head,
                                const int64_t *rows, int n_rows, int32_t *hits /* [n_rows] */,
                                int32_t *size /* [n_rows] */) {
    int G = H_q / H_kv;
    int32_t *I = (int32_t *)malloc((size_t)H_q * (size_t)(n_rows > 0 ? n_rows : 1) * N_b * sizeof(int32_t));
    int32_t *cnt = (int32_t *)malloc((size_t)H_q * (size_t)(n_rows > 0 ? n_rows : 1) * sizeof(int32_t));
    if (!I || !cnt) { free(I); free(cnt); return 1; }
    int err;
    if (B_r > 0) {
        int64_t *blocks = (int64_t *)malloc((size_t)(n_rows > 0 ? n_rows : 1) * sizeof(int64_t));
        if (!blocks) { free(I); free(cnt); return 1; }
        for (int t = 0; t < n_rows; ++t) blocks[t] = rows[t] / B_r;
        err = dhsa_oracle_route_blocks(Q, K, H_q, H_kv, L, D, B, N_c, B_r, N_b, pooling, blocks, n_rows, I, cnt);
        free(blocks);
    } else {
        err = dhsa_oracle_route_rows(Q, K, H_q, H_kv, L, D, B, N_c, N_b, pooling, rows, n_rows, I, cnt);
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int t = 0; t < n_rows; ++t) {
        int64_t i = rows[t];
        const int32_t *It = I + ((int64_t)head * n_rows + t) * N_b;
        int c = cnt[(int64_t)head * n_rows + t];
        /* the block's list may hold keys above the row: they are masked in attention, so not retained */
        int32_t *vis = (int32_t *)malloc((size_t)(c > 0 ? c : 1) * sizeof(int32_t));
        int cv = 0;
        if (!vis) { err = 1; continue; }
        for (int v = 0; v < c; ++v)
            if (It[v] <= i) vis[cv++] = It[v];
        if (dhsa_oracle_recall_row(Q + ((int64_t)head * L + i) * D, K + (int64_t)(head / G) * L * D, i, D, vis, cv,
                                   N_b, hits + t, size + t))
            err = 1;
        free(vis);
    }
    free(I); free(cnt);
    return err;
}
