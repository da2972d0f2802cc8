/*
 * SpecPV verification path -- CPU fp64 oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the checker the GPU library is compared against.  It is a
 * plain, slow, definition-by-definition implementation; nothing in the
 * product path may call it (only tests, the smoke check and the bench's
 * cpu_baseline leg do).  It shares no code, tables or helpers with the HIP
 * sources.
 *
 * Every function works on ONE sequence and ONE layer.  All floating-point
 * inputs arrive already widened to double (the widening from fp32 / bf16 is
 * exact), and every intermediate is double.  The only place a narrower
 * precision appears is block selection, where the reduced score is rounded
 * to fp32 before it is ordered, because the selection rule is stated on fp32
 * scores.
 *
 * Layouts (row-major, last index fastest):
 *   K, V      [L ][Hkv][D]   committed context keys / values
 *   Q         [M ][Hq ][D]   one query per draft-tree node and query head
 *   Kd, Vd    [M ][Hkv][D]   keys / values of the draft-tree nodes themselves
 *   kmax,kmin [nb][Hkv][D]   per-block key summaries, nb = ceil(L / B)
 *   parent    [M]            parent[0] = -1, parent[i] < i
 * Query head h reads KV head g = h / G with G = Hq / Hkv (grouped-query
 * attention).  Row r = j*G + (h - g*G) enumerates the M*G query rows of a
 * KV head, node-major.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py
 * (closed forms, hand-worked examples under tests/golden/, brute force on
 * tiny inputs, and reductions to numpy / torch SDPA library routines).  The
 * paper prints no worked numeric example, so agreement with the authors'
 * own numbers is unpinned; agreement with the paper's definitions is pinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_REDUCE_MEAN 0
#define ORACLE_REDUCE_MAX 1
#define ORACLE_REDUCE_LAST 2

/* Section 3.2, eq. 1: the summary of block i is the element-wise maximum and
 * minimum of the keys of the tokens in the block.  A trailing block that is
 * only partly filled is summarised over the tokens it has. */
void oracle_block_summarize(const double *K, int L, int Hkv, int D, int B,
                            double *kmax, double *kmin)
{
    int nb = (L + B - 1) / B;
    for (int i = 0; i < nb; ++i)
        for (int g = 0; g < Hkv; ++g)
            for (int d = 0; d < D; ++d) {
                int t0 = i * B;
                int t1 = (i + 1) * B < L ? (i + 1) * B : L;
                double mx = K[((size_t)t0 * Hkv + g) * D + d];
                double mn = mx;
                for (int t = t0 + 1; t < t1; ++t) {
                    double x = K[((size_t)t * Hkv + g) * D + d];
                    if (x > mx) mx = x;
                    if (x < mn) mn = x;
                }
                kmax[((size_t)i * Hkv + g) * D + d] = mx;
                kmin[((size_t)i * Hkv + g) * D + d] = mn;
            }
}

/* Section 3.2, eq. 2: the score of block i for query row r is the larger of
 * the two inner products  q_r . Kmax_i  and  q_r . Kmin_i  (two full inner
 * products, then one max; no 1/sqrt(D) factor).
 * Output s[g][i][r], r = j*G + hh. */
void oracle_row_scores(const double *Q, int M, int Hq,
                       const double *kmax, const double *kmin, int nb,
                       int Hkv, int D, double *s)
{
    int G = Hq / Hkv;
    int R = M * G;
#pragma omp parallel for collapse(2) schedule(static)
    for (int g = 0; g < Hkv; ++g)
        for (int i = 0; i < nb; ++i)
            for (int j = 0; j < M; ++j)
                for (int hh = 0; hh < G; ++hh) {
                    int h = g * G + hh;
                    const double *q = Q + ((size_t)j * Hq + h) * D;
                    const double *a = kmax + ((size_t)i * Hkv + g) * D;
                    const double *b = kmin + ((size_t)i * Hkv + g) * D;
                    double da = 0.0, db = 0.0;
                    for (int d = 0; d < D; ++d) {
                        da += q[d] * a[d];
                        db += q[d] * b[d];
                    }
                    s[((size_t)g * nb + i) * R + (size_t)j * G + hh] = da > db ? da : db;
                }
}

/* The channel-wise variant of the block score, in the style of the query-aware
 * page selection that Section 3.2 names as the inspiration for its summaries:
 * per channel the larger of  q_r[d] * Kmax_i[d]  and  q_r[d] * Kmin_i[d],
 * summed over the channels.  Unlike eq. 2 this is an upper bound of q_r . k_t
 * for every token t of the block.  Same output layout as oracle_row_scores. */
void oracle_row_scores_channel(const double *Q, int M, int Hq,
                               const double *kmax, const double *kmin, int nb,
                               int Hkv, int D, double *s)
{
    int G = Hq / Hkv;
    int R = M * G;
#pragma omp parallel for collapse(2) schedule(static)
    for (int g = 0; g < Hkv; ++g)
        for (int i = 0; i < nb; ++i)
            for (int j = 0; j < M; ++j)
                for (int hh = 0; hh < G; ++hh) {
                    int h = g * G + hh;
                    const double *q = Q + ((size_t)j * Hq + h) * D;
                    const double *a = kmax + ((size_t)i * Hkv + g) * D;
                    const double *b = kmin + ((size_t)i * Hkv + g) * D;
                    double sum = 0.0;
                    for (int d = 0; d < D; ++d) {
                        double pa = q[d] * a[d], pb = q[d] * b[d];
                        sum += pa > pb ? pa : pb;
                    }
                    s[((size_t)g * nb + i) * R + (size_t)j * G + hh] = sum;
                }
}

/* Section 3.2, eq. 3: the per-row scores of a block are reduced to one score
 * by f in {mean, max, last}.  mean and max run over all M*G rows of the KV
 * head; "last" keeps only the rows of one designated node (the most recently
 * verified token, node `last_node`) and averages over its G query heads.
 * Output scores[g][i]. */
void oracle_reduce_scores(const double *s, int Hkv, int nb, int M, int G,
                          int reduce, int last_node, double *scores)
{
    int R = M * G;
    for (int g = 0; g < Hkv; ++g)
        for (int i = 0; i < nb; ++i) {
            const double *row = s + ((size_t)g * nb + i) * R;
            double out;
            if (reduce == ORACLE_REDUCE_MEAN) {
                double acc = 0.0;
                for (int r = 0; r < R; ++r) acc += row[r];
                out = acc / (double)R;
            } else if (reduce == ORACLE_REDUCE_MAX) {
                out = row[0];
                for (int r = 1; r < R; ++r)
                    if (row[r] > out) out = row[r];
            } else {
                double acc = 0.0;
                for (int hh = 0; hh < G; ++hh) acc += row[(size_t)last_node * G + hh];
                out = acc / (double)G;
            }
            scores[(size_t)g * nb + i] = out;
        }
}

/* Section 3.2 (sink, retrieval and local components of the partial cache).
 * Per KV head: blocks [0, ns) are always kept (sink), blocks [nb-nr, nb) are
 * always kept (local window), and from the candidates in between the k blocks
 * with the largest score are kept.  Scores are rounded to fp32 first; among
 * equal fp32 scores the lower block index wins.  The kept blocks are listed in
 * ascending block order (the partial cache is contiguous in token order).
 * If nb <= ns + k + nr every block is kept.
 * Output sel_idx[g][0..n_sel) padded with -1, sel_count[g]; n_sel = ns+k+nr. */
void oracle_select_blocks(const double *scores, int Hkv, int nb, int ns,
                          int nr, int k, int32_t *sel_idx, int32_t *sel_count)
{
    int n_sel = ns + k + nr;
    char *keep = (char *)malloc((size_t)(nb > 0 ? nb : 1));
    for (int g = 0; g < Hkv; ++g) {
        memset(keep, 0, (size_t)(nb > 0 ? nb : 1));
        if (nb <= n_sel) {
            for (int i = 0; i < nb; ++i) keep[i] = 1;
        } else {
            for (int i = 0; i < ns; ++i) keep[i] = 1;
            for (int i = nb - nr; i < nb; ++i) keep[i] = 1;
            /* k rounds of "take the best candidate not taken yet" */
            for (int round = 0; round < k; ++round) {
                int best = -1;
                float best_s = 0.0f;
                for (int i = ns; i < nb - nr; ++i) {
                    if (keep[i]) continue;
                    float si = (float)scores[(size_t)g * nb + i];
                    if (best < 0 || si > best_s) { /* strict >: lower index wins ties */
                        best = i;
                        best_s = si;
                    }
                }
                if (best < 0) break;
                keep[best] = 1;
            }
        }
        int c = 0;
        for (int i = 0; i < nb; ++i)
            if (keep[i]) sel_idx[(size_t)g * n_sel + c++] = i;
        sel_count[g] = c;
        for (; c < n_sel; ++c) sel_idx[(size_t)g * n_sel + c] = -1;
    }
    free(keep);
}

/* Section 3.2 / 3.3 and the tree decode of Algorithm 1: scaled-dot-product
 * attention of every (node j, query head h) over
 *     the context tokens t < L whose block  t / B  is in the kept list of
 *     KV head g = h / G                       (all blocks if sel_idx == NULL)
 *   + the draft-tree nodes a that are j itself or an ancestor of j.
 * logits z = q . k / sqrt(D);  p = softmax(z);  O = sum p v;
 * LSE = log sum exp z.  psum (optional) receives sum p, which must be 1.
 * sel_idx is [Hkv][n_sel] (entries < 0 are padding), sel_count is [Hkv]. */
void oracle_tree_attention(const double *Q, const double *K, const double *V,
                           const double *Kd, const double *Vd,
                           const int32_t *parent, int M, int Hq, int Hkv,
                           int D, int L, int B, const int32_t *sel_idx,
                           const int32_t *sel_count, int n_sel, double *O,
                           double *lse, double *psum)
{
    int G = Hq / Hkv;
    int nb = (L + B - 1) / B;
    double scale = 1.0 / sqrt((double)D);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int j = 0; j < M; ++j)
        for (int h = 0; h < Hq; ++h) {
            int g = h / G;
            const double *q = Q + ((size_t)j * Hq + h) * D;
            /* 1. which context blocks does this KV head attend to */
            char *keep = (char *)calloc((size_t)(nb > 0 ? nb : 1), 1);
            if (sel_idx == NULL) {
                for (int i = 0; i < nb; ++i) keep[i] = 1;
            } else {
                for (int c = 0; c < sel_count[g]; ++c) {
                    int i = sel_idx[(size_t)g * n_sel + c];
                    if (i >= 0 && i < nb) keep[i] = 1;
                }
            }
            /* 2. which draft nodes: j and its ancestors */
            char *anc = (char *)calloc((size_t)M, 1);
            for (int a = j; a >= 0; a = parent[a]) anc[a] = 1;
            /* 3. logits of all attended keys, in one list */
            size_t cap = (size_t)L + (size_t)M;
            double *z = (double *)malloc(cap * sizeof(double));
            const double **vp = (const double **)malloc(cap * sizeof(double *));
            size_t n = 0;
            for (int t = 0; t < L; ++t) {
                if (!keep[t / B]) continue;
                const double *kk = K + ((size_t)t * Hkv + g) * D;
                double dot = 0.0;
                for (int d = 0; d < D; ++d) dot += q[d] * kk[d];
                z[n] = dot * scale;
                vp[n] = V + ((size_t)t * Hkv + g) * D;
                ++n;
            }
            for (int a = 0; a < M; ++a) {
                if (!anc[a]) continue;
                const double *kk = Kd + ((size_t)a * Hkv + g) * D;
                double dot = 0.0;
                for (int d = 0; d < D; ++d) dot += q[d] * kk[d];
                z[n] = dot * scale;
                vp[n] = Vd + ((size_t)a * Hkv + g) * D;
                ++n;
            }
            /* 4. softmax and weighted sum of values */
            double zmax = z[0];
            for (size_t x = 1; x < n; ++x)
                if (z[x] > zmax) zmax = z[x];
            double denom = 0.0;
            for (size_t x = 0; x < n; ++x) denom += exp(z[x] - zmax);
            double *o = O + ((size_t)j * Hq + h) * D;
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            double ps = 0.0;
            for (size_t x = 0; x < n; ++x) {
                double p = exp(z[x] - zmax) / denom;
                ps += p;
                for (int d = 0; d < D; ++d) o[d] += p * vp[x][d];
            }
            if (lse) lse[(size_t)j * Hq + h] = zmax + log(denom);
            if (psum) psum[(size_t)j * Hq + h] = ps;
            free(z);
            free((void *)vp);
            free(anc);
            free(keep);
        }
}

/* Number of OpenMP threads the loops above run on (for the bench report). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
