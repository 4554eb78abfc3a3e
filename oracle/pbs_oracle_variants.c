/*
 * pbs_oracle_variants.c -- fp64 CPU oracle of the method's VARIANTS that the paper ablates: the alternative proxies
 * for the global importance score and the key-aware query permutation.
 *
 * TEST INFRASTRUCTURE ONLY, like pbs_oracle.c, and just as independent of the HIP library: nothing here is shared
 * with, included by or linked into the product; only tests/, the smoke check and the benchmark's CPU leg may use it.
 * Plain C, one scalar loop per formula, no blocking, OpenMP across independent (batch, head) items only.
 * Inputs are float arrays whose values are already rounded to the storage type; everything is promoted to double.
 *
 * Where the paper leaves a choice open, the reading taken is stated at the function ("parity unpinned": no value the
 * paper prints fixes it; the tests pin the function against the mathematics instead).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------
 * Global importance score from a chosen set of query rows -- the proxies of Section "The Problem of Information
 * Fragmentation" (heuristic 4: "a subset of queries (either a random subset or the last block)") and of the appendix
 * "Task-wise Proxy Sensitivity" (Random-Query-Attn, Avg-Query-Attn, Last-Block-Query-Attn).  Same formula as Eq. 4,
 * with the queries of a GQA group averaged row by row first (appendix "GQA Handling"):
 *
 *   mode 0, query rows given:  Qset[t] = mean over the group's heads of Q[rows[t]],  t = 0 .. m-1
 *                              (rows = the last block gives Eq. 4 itself; rows drawn at random by the caller give
 *                              Random-Query-Attn; a row listed twice counts twice);
 *   mode 1, average query:     Qset = one vector, the mean over ALL n positions of the group-averaged queries
 *                              (reading of "Avg-Query-Attn", which the paper only names: parity unpinned);
 *
 *   s[j] = (1 / |Qset|) * sum_t softmax_j( Qset[t] . K[j] * scale )   over all n keys, no causal mask (as Eq. 4).
 *
 * rows: [m] positions in [0, n), used for every (batch, kv head); ignored in mode 1.  s: [batch, h_kv, n] doubles.
 * ---------------------------------------------------------------------- */
int pbsv_key_scores_proxy(int batch, int h_q, int h_kv, int n, int d, int mode, int m, const int32_t *rows,
                          double scale, const float *Q, const float *K, double *s)
{
    if (h_kv <= 0 || h_q % h_kv != 0 || n <= 0 || d <= 0) return 1;
    if (mode == 0) {
        if (m <= 0 || !rows) return 1;
        for (int t = 0; t < m; ++t) if (rows[t] < 0 || rows[t] >= n) return 1;
    } else if (mode != 1) return 1;
    const int r = h_q / h_kv;
    const int nq = mode == 0 ? m : 1;
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < batch; ++b)
        for (int h = 0; h < h_kv; ++h) {
            double *qset = (double *)malloc(sizeof(double) * (size_t)nq * d);
            double *P = (double *)malloc(sizeof(double) * (size_t)n);
            double *sh = s + ((size_t)b * h_kv + h) * (size_t)n;
            if (!qset || !P) { fail = 1; free(qset); free(P); continue; }
            if (mode == 0) {
                for (int t = 0; t < m; ++t)
                    for (int e = 0; e < d; ++e) {
                        double acc = 0.0;
                        for (int u = 0; u < r; ++u)
                            acc += (double)Q[(((size_t)b * h_q + (size_t)h * r + u) * n + rows[t]) * d + e];
                        qset[(size_t)t * d + e] = acc / (double)r;
                    }
            } else {
                for (int e = 0; e < d; ++e) {
                    double acc = 0.0;
                    for (int pos = 0; pos < n; ++pos) {
                        double g = 0.0;
                        for (int u = 0; u < r; ++u)
                            g += (double)Q[(((size_t)b * h_q + (size_t)h * r + u) * n + pos) * d + e];
                        acc += g / (double)r;
                    }
                    qset[e] = acc / (double)n;
                }
            }
            const float *Kh = K + ((size_t)b * h_kv + h) * (size_t)n * d;
            for (int j = 0; j < n; ++j) sh[j] = 0.0;
            for (int t = 0; t < nq; ++t) {
                double mx = 0.0;
                for (int j = 0; j < n; ++j) {
                    double acc = 0.0;
                    for (int e = 0; e < d; ++e) acc += qset[(size_t)t * d + e] * (double)Kh[(size_t)j * d + e];
                    P[j] = acc * scale;
                    if (j == 0 || P[j] > mx) mx = P[j];
                }
                double sum = 0.0;
                for (int j = 0; j < n; ++j) { P[j] = exp(P[j] - mx); sum += P[j]; }
                for (int j = 0; j < n; ++j) sh[j] += P[j] / sum;
            }
            for (int j = 0; j < n; ++j) sh[j] /= (double)nq;
            free(qset); free(P);
        }
    return fail;
}

/* ------------------------------------------------------------------------
 * Key-aware query permutation of Section "Design Choice: Why Permute Keys but not Queries?":
 *   centroids  Kbar_j = MeanPool(keys of block j),  j = 0 .. T-1  (of the key tensor given: K, or K' when the keys
 *              were permuted first; valid rows only in a partial last block);
 *   every query of a full segment g is assigned to the centroid it is most similar to by cosine similarity, among
 *   the centroids its segment may attend to, j < (g+1)*R capped at T (the columns the extended causal mask admits);
 *   the queries of the segment are then ordered by their assigned centroid, ascending, queries with the same centroid
 *   keeping their original order.  Tokens past the last full segment stay where they are.
 *
 * Readings (the paper gives one sentence, "queries are assigned greedily based on their similarity to the
 * centroids": parity unpinned): "greedily" = every query takes its single best centroid, with no capacity per
 * centroid and no reassignment; the candidate set is the visible region of the segment; ties go to the lowest j.
 * cos(q, Kbar_j) = (q . Kbar_j) / (|q| |Kbar_j|): |q| is the same for every j, so the decision uses
 *     u_j = (q . Kbar_j) * rinv_j,   rinv_j = 1 / sqrt(sum_e Kbar_j[e]^2)   (0 when the centroid is the zero vector),
 * every sum over the features in ascending order with separate multiplications and additions, argmax by strict ">".
 *
 * Gather form with absolute positions, like every index vector of the method: slot p of Q' holds query qidx[p].
 * qidx: [batch, h_q, n] int32; assigned (nullable): [batch, h_q, n] int32, the centroid of every query (-1 in the tail).
 * ---------------------------------------------------------------------- */
typedef struct { int32_t c; int32_t pos; } pbsv_assign;

static int assign_cmp(const void *pa, const void *pb)
{
    const pbsv_assign *a = (const pbsv_assign *)pa, *b = (const pbsv_assign *)pb;
    if (a->c != b->c) return a->c < b->c ? -1 : 1;
    return a->pos < b->pos ? -1 : (a->pos > b->pos ? 1 : 0);
}

/* centroids and their reciprocal norms for every (batch, kv head): Kbar [bh][T][d], rinv [bh][T] */
static int centroids(int nbk, int n, int d, int block, int T, const float *K, double **Kbar_out, double **rinv_out)
{
    double *Kbar = (double *)malloc(sizeof(double) * (size_t)nbk * T * d);
    double *rinv = (double *)malloc(sizeof(double) * (size_t)nbk * T);
    if (!Kbar || !rinv) { free(Kbar); free(rinv); return 2; }
    for (int bh = 0; bh < nbk; ++bh)
        for (int j = 0; j < T; ++j) {
            const int lo = j * block, hi = lo + block < n ? lo + block : n;
            double nsq = 0.0;
            for (int e = 0; e < d; ++e) {
                double acc = 0.0;
                for (int pos = lo; pos < hi; ++pos) acc += (double)K[((size_t)bh * n + pos) * d + e];
                const double mean = acc / (double)(hi - lo);
                Kbar[((size_t)bh * T + j) * d + e] = mean;
                nsq += mean * mean;
            }
            rinv[(size_t)bh * T + j] = nsq > 0.0 ? 1.0 / sqrt(nsq) : 0.0;
        }
    *Kbar_out = Kbar;
    *rinv_out = rinv;
    return 0;
}

/* segment g of one query head: out[0 .. segment) = the segment's positions ordered by (assigned centroid, position);
 * assigned (nullable) is indexed by absolute position.  a: scratch of `segment` entries. */
static void order_segment(int g, int n, int d, int segment, int R, int T, const float *Qh, const double *kb,
                          const double *ri, pbsv_assign *a, int32_t *out, int32_t *assigned)
{
    const int ncand = (g + 1) * R < T ? (g + 1) * R : T;
    (void)n;
    for (int t = 0; t < segment; ++t) {
        const int pos = g * segment + t;
        const float *q = Qh + (size_t)pos * d;
        int best = 0;
        double ubest = 0.0;
        for (int j = 0; j < ncand; ++j) {
            double dot = 0.0;
            for (int e = 0; e < d; ++e) dot += (double)q[e] * kb[(size_t)j * d + e];
            const double u = dot * ri[j];
            if (j == 0 || u > ubest) { ubest = u; best = j; }
        }
        a[t].c = best;
        a[t].pos = pos;
        if (assigned) assigned[pos] = best;
    }
    qsort(a, (size_t)segment, sizeof(pbsv_assign), assign_cmp);
    for (int t = 0; t < segment; ++t) out[t] = a[t].pos;
}

int pbsv_query_permutation(int batch, int h_q, int h_kv, int n, int d, int block, int segment,
                           const float *Q, const float *K, int32_t *qidx, int32_t *assigned)
{
    if (h_kv <= 0 || h_q % h_kv != 0 || n <= 0 || d <= 0 || block <= 0 || segment % block != 0) return 1;
    const int T = (n + block - 1) / block, R = segment / block, G = n / segment, r = h_q / h_kv;
    double *Kbar, *rinv;
    if (centroids(batch * h_kv, n, d, block, T, K, &Kbar, &rinv)) return 2;
    int fail = 0;
#pragma omp parallel for schedule(dynamic)
    for (int bhq = 0; bhq < batch * h_q; ++bhq) {
        const int b = bhq / h_q, hq = bhq % h_q, hk = hq / r;
        const double *kb = Kbar + ((size_t)(b * h_kv + hk) * T) * d;
        const double *ri = rinv + (size_t)(b * h_kv + hk) * T;
        int32_t *out = qidx + (size_t)bhq * n;
        int32_t *as = assigned ? assigned + (size_t)bhq * n : NULL;
        pbsv_assign *a = (pbsv_assign *)malloc(sizeof(pbsv_assign) * (size_t)segment);
        if (!a) { fail = 1; continue; }
        for (int g = 0; g < G; ++g)
            order_segment(g, n, d, segment, R, T, Q + (size_t)bhq * n * d, kb, ri, a, out + (size_t)g * segment, as);
        for (int pos = G * segment; pos < n; ++pos) {
            out[pos] = pos;
            if (as) as[pos] = -1;
        }
        free(a);
    }
    free(Kbar); free(rinv);
    return fail ? 2 : 0;
}

/* The same for ONE full segment g of every query head (what a test at full length can afford): qseg [batch, h_q,
 * segment] = the slice [g*segment, (g+1)*segment) of the qidx that pbsv_query_permutation would write. */
int pbsv_query_permutation_segment(int batch, int h_q, int h_kv, int n, int d, int block, int segment, int g,
                                   const float *Q, const float *K, int32_t *qseg)
{
    if (h_kv <= 0 || h_q % h_kv != 0 || n <= 0 || d <= 0 || block <= 0 || segment % block != 0) return 1;
    const int T = (n + block - 1) / block, R = segment / block, G = n / segment, r = h_q / h_kv;
    if (g < 0 || g >= G) return 1;
    double *Kbar, *rinv;
    if (centroids(batch * h_kv, n, d, block, T, K, &Kbar, &rinv)) return 2;
    int fail = 0;
#pragma omp parallel for schedule(dynamic)
    for (int bhq = 0; bhq < batch * h_q; ++bhq) {
        const int b = bhq / h_q, hq = bhq % h_q, hk = hq / r;
        pbsv_assign *a = (pbsv_assign *)malloc(sizeof(pbsv_assign) * (size_t)segment);
        if (!a) { fail = 1; continue; }
        order_segment(g, n, d, segment, R, T, Q + (size_t)bhq * n * d, Kbar + ((size_t)(b * h_kv + hk) * T) * d,
                      rinv + (size_t)(b * h_kv + hk) * T, a, qseg + (size_t)bhq * segment, NULL);
        free(a);
    }
    free(Kbar); free(rinv);
    return fail ? 2 : 0;
}
