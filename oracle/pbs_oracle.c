/*
 * pbs_oracle.c -- plain, slow, fp64 CPU oracle for the PBS-Attn prefill path.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path links, loads or calls
 * this file; only the tests, the smoke check and the benchmark's cpu_baseline
 * leg do.  It shares no code, header, table or helper with the HIP library.
 *
 * Every function follows one passage of the paper "Sparser Block-Sparse
 * Attention via Token Permutation" (arXiv 2510.21270), cited at the function.
 * Inputs are float arrays that already hold values rounded to the storage
 * type (bf16 or fp32); all arithmetic below is IEEE double, in the order the
 * paper states, with no blocking, fusion or reordering.  OpenMP is used only
 * across independent (head, row) units; it never changes a summation order.
 *
 * Layouts: Q [batch, h_q, n, d]; K, V [batch, h_kv, n, d]; row-major.
 * Query head hq reads kv head hq / (h_q / h_kv).
 * Index vectors are in gather form with absolute positions: slot p of a
 * permuted tensor holds original token idx[p].
 *
 * Pins (see tests/test_oracle_*.py): Theorem 1 against dense causal attention,
 * numpy/scipy library routines for Eq. 4 and Eq. 5, brute-force subset search
 * and hand-worked rows for Algorithm 2, Table 5's causal block totals.
 * Readings that the paper does not fix by a printed value (no mask in Eq. 4,
 * query averaging for GQA, the extended causal mask C, forced on-diagonal
 * blocks, forced first block) are "parity unpinned" beyond those checks.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int ceil_div(int a, int b) { return (a + b - 1) / b; }

/* ------------------------------------------------------------------------
 * Eq. 4 (global importance score) with the shared-permutation GQA strategy of
 * the appendix "GQA Handling": the query vectors of the r = h_q / h_kv heads
 * of a group are averaged row by row, then
 *     s = mean_rows( softmax( Qhat_last_block K^T * scale ) )
 * over ALL n keys (Eq. 4 carries no causal mask).  "Last block" is the last
 * min(block, n) query rows.  s: [batch, h_kv, n] doubles.
 * ---------------------------------------------------------------------- */
int pbso_key_scores(int batch, int h_q, int h_kv, int n, int d, int block,
                    double scale, const float *Q, const float *K, double *s)
{
    if (h_kv <= 0 || h_q % h_kv != 0 || n <= 0 || d <= 0 || block <= 0) return 1;
    const int r = h_q / h_kv;
    const int bl = block < n ? block : n;
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < batch; ++b)
        for (int h = 0; h < h_kv; ++h) {
            double *qhat = (double *)malloc(sizeof(double) * (size_t)bl * d);
            double *L = (double *)malloc(sizeof(double) * (size_t)bl * n);
            if (!qhat || !L) { fail = 1; free(qhat); free(L); continue; }
            /* group-averaged last-block queries */
            for (int row = 0; row < bl; ++row)
                for (int e = 0; e < d; ++e) {
                    double acc = 0.0;
                    for (int t = 0; t < r; ++t) {
                        size_t hq = (size_t)h * r + t;
                        acc += (double)Q[(((size_t)b * h_q + hq) * n + (n - bl + row)) * d + e];
                    }
                    qhat[(size_t)row * d + e] = acc / (double)r;
                }
            const float *Kh = K + ((size_t)b * h_kv + h) * (size_t)n * d;
            /* logits */
            for (int row = 0; row < bl; ++row)
                for (int j = 0; j < n; ++j) {
                    double acc = 0.0;
                    for (int e = 0; e < d; ++e)
                        acc += qhat[(size_t)row * d + e] * (double)Kh[(size_t)j * d + e];
                    L[(size_t)row * n + j] = acc * scale;
                }
            /* row softmax */
            for (int row = 0; row < bl; ++row) {
                double *Lr = L + (size_t)row * n;
                double mx = Lr[0];
                for (int j = 1; j < n; ++j) if (Lr[j] > mx) mx = Lr[j];
                double sum = 0.0;
                for (int j = 0; j < n; ++j) { Lr[j] = exp(Lr[j] - mx); sum += Lr[j]; }
                for (int j = 0; j < n; ++j) Lr[j] /= sum;
            }
            /* mean over the rows */
            double *sh = s + ((size_t)b * h_kv + h) * (size_t)n;
            for (int j = 0; j < n; ++j) {
                double acc = 0.0;
                for (int row = 0; row < bl; ++row) acc += L[(size_t)row * n + j];
                sh[j] = acc / (double)bl;
            }
            free(qhat); free(L);
        }
    return fail;
}

/* ------------------------------------------------------------------------
 * Eq. 5 inside the segmented permutation of Section "Segmented Permutation for
 * Causal Attention": the first floor(n/S)*S tokens form G segments of S; inside
 * segment g the keys are ordered by descending score, equal scores keeping
 * ascending index; the remaining n mod S tokens stay where they are.
 * Gather form: idx[g*S + t] = g*S + (index of the t-th largest score).
 * s, idx: [nbh, n].
 * ---------------------------------------------------------------------- */
typedef struct { double s; int32_t i; } pbso_pair;

static int pair_desc(const void *pa, const void *pb)
{
    const pbso_pair *a = (const pbso_pair *)pa, *b = (const pbso_pair *)pb;
    if (a->s > b->s) return -1;
    if (a->s < b->s) return 1;
    return (a->i > b->i) - (a->i < b->i);
}

int pbso_segment_argsort(int nbh, int n, int segment, const double *s, int32_t *idx)
{
    if (segment <= 0 || n <= 0) return 1;
    const int G = n / segment;
    int fail = 0;
#pragma omp parallel for schedule(dynamic)
    for (int bh = 0; bh < nbh; ++bh) {
        pbso_pair *buf = (pbso_pair *)malloc(sizeof(pbso_pair) * (size_t)segment);
        if (!buf) { fail = 1; continue; }
        const double *sh = s + (size_t)bh * n;
        int32_t *ih = idx + (size_t)bh * n;
        for (int g = 0; g < G; ++g) {
            for (int t = 0; t < segment; ++t) { buf[t].s = sh[g * segment + t]; buf[t].i = t; }
            qsort(buf, (size_t)segment, sizeof(pbso_pair), pair_desc);
            for (int t = 0; t < segment; ++t) ih[g * segment + t] = g * segment + buf[t].i;
        }
        for (int p = G * segment; p < n; ++p) ih[p] = p;
        free(buf);
    }
    return fail;
}

/* Algorithm 1, first step: X' = P X as a row gather, X'[p] = X[idx[p]].  [nbh, n, d]. */
int pbso_gather_rows(int nbh, int n, int d, const float *X, const int32_t *idx, float *Xp)
{
    for (int bh = 0; bh < nbh; ++bh)
        for (int p = 0; p < n; ++p) {
            int32_t src = idx[(size_t)bh * n + p];
            if (src < 0 || src >= n) return 1;
            memcpy(Xp + ((size_t)bh * n + p) * d, X + ((size_t)bh * n + src) * d, sizeof(float) * (size_t)d);
        }
    return 0;
}

/* Algorithm 1, last step / Theorem 1: O = P_sigma^T O', i.e. O[idx[p]] = O'[p].  [nbh, n, d]. */
int pbso_scatter_rows(int nbh, int n, int d, const double *Op, const int32_t *idx, double *O)
{
    for (int bh = 0; bh < nbh; ++bh)
        for (int p = 0; p < n; ++p) {
            int32_t dst = idx ? idx[(size_t)bh * n + p] : p;
            if (dst < 0 || dst >= n) return 1;
            memcpy(O + ((size_t)bh * n + dst) * d, Op + ((size_t)bh * n + p) * d, sizeof(double) * (size_t)d);
        }
    return 0;
}

/* number of key blocks the extended causal mask C lets query block i see
 * (appendix "Block Selection in PBS-Attn": C also admits the on-diagonal
 * segment; past the last full segment it is plain block causality). */
static int allowed_cols(int i, int T, int R, int G)
{
    int g = i / R;
    if (g < G) { int v = (g + 1) * R; return v < T ? v : T; }
    return i + 1;
}

/* ------------------------------------------------------------------------
 * Algorithm 2 (MeanPooling block selection) on the permuted Q', K':
 *   pooled block means (over the valid rows of a partial last block),
 *   a_i = softmax_j( Qbar_i . Kbar_j * scale ) over the columns C allows,
 *   o_i = stable argsort(-a_i), c_i = cumsum(a_i[o_i]),
 *   k = min({t : c_i[t] >= tau} U {n_i}), select o_i[1..k].
 * Then the blocks of the query block's own segment are switched on (they hold
 * causally needed keys after the intra-segment permutation, Section "Effect of
 * Segment Size"); past the last full segment, where nothing is permuted, only
 * the diagonal block is (the "most recent" block of Section "Baselines"); and
 * block 0 when flags bit 0 is set (the forced first block of the same
 * passage).  Forced blocks do not change k.
 * mask: [batch, h_q, T, T] bytes; row_cnt: [batch, h_q, T]; col_idx:
 * [batch, h_q, T, T] ascending, first row_cnt valid, rest -1;
 * probs (nullable): [batch, h_q, T, T] the a_i (0 outside the allowed columns);
 * k_out (nullable): [batch, h_q, T] the k of Algorithm 2 before any forcing.
 * ---------------------------------------------------------------------- */
int pbso_block_mask(int batch, int h_q, int h_kv, int n, int d, int block, int segment,
                    double tau, double scale, unsigned flags,
                    const float *Qp, const float *Kp,
                    uint8_t *mask, int32_t *row_cnt, int32_t *col_idx, double *probs, int32_t *k_out)
{
    if (h_kv <= 0 || h_q % h_kv != 0 || block <= 0 || segment % block != 0) return 1;
    const int T = ceil_div(n, block), R = segment / block, G = n / segment;
    const int r = h_q / h_kv;
    double *Qbar = (double *)malloc(sizeof(double) * (size_t)batch * h_q * T * d);
    double *Kbar = (double *)malloc(sizeof(double) * (size_t)batch * h_kv * T * d);
    if (!Qbar || !Kbar) { free(Qbar); free(Kbar); return 2; }
    /* MeanPool of every block */
    for (int pass = 0; pass < 2; ++pass) {
        const float *X = pass ? Kp : Qp;
        double *Xbar = pass ? Kbar : Qbar;
        const int nh = batch * (pass ? h_kv : h_q);
#pragma omp parallel for collapse(2) schedule(static)
        for (int bh = 0; bh < nh; ++bh)
            for (int i = 0; i < T; ++i) {
                int lo = i * block, hi = lo + block < n ? lo + block : n;
                for (int e = 0; e < d; ++e) {
                    double acc = 0.0;
                    for (int p = lo; p < hi; ++p) acc += (double)X[((size_t)bh * n + p) * d + e];
                    Xbar[((size_t)bh * T + i) * d + e] = acc / (double)(hi - lo);
                }
            }
    }
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int bh = 0; bh < batch * h_q; ++bh)
        for (int i = 0; i < T; ++i) {
            const int b = bh / h_q, hq = bh % h_q, hk = hq / r;
            const int ni = allowed_cols(i, T, R, G);
            double *a = (double *)malloc(sizeof(double) * (size_t)ni);
            pbso_pair *o = (pbso_pair *)malloc(sizeof(pbso_pair) * (size_t)ni);
            if (!a || !o) { fail = 1; free(a); free(o); continue; }
            const double *qb = Qbar + ((size_t)bh * T + i) * d;
            const double *kb = Kbar + ((size_t)(b * h_kv + hk) * T) * d;
            double mx = 0.0;
            for (int j = 0; j < ni; ++j) {
                double acc = 0.0;
                for (int e = 0; e < d; ++e) acc += qb[e] * kb[(size_t)j * d + e];
                a[j] = acc * scale;
                if (j == 0 || a[j] > mx) mx = a[j];
            }
            double sum = 0.0;
            for (int j = 0; j < ni; ++j) { a[j] = exp(a[j] - mx); sum += a[j]; }
            for (int j = 0; j < ni; ++j) a[j] /= sum;
            for (int j = 0; j < ni; ++j) { o[j].s = a[j]; o[j].i = j; }
            qsort(o, (size_t)ni, sizeof(pbso_pair), pair_desc);
            int k = ni;
            double c = 0.0;
            for (int t = 0; t < ni; ++t) {
                c += o[t].s;
                if (c >= tau) { k = t + 1; break; }
            }
            uint8_t *mrow = mask + ((size_t)bh * T + i) * T;
            memset(mrow, 0, (size_t)T);
            for (int t = 0; t < k; ++t) mrow[o[t].i] = 1;
            /* every block of the query block's own (permuted) segment; in the
             * unpermuted tail only the diagonal ("most recent") block */
            const int g = i / R;
            const int flo = (g < G) ? g * R : i;
            for (int j = flo; j < ni; ++j) mrow[j] = 1;
            if (k_out) k_out[(size_t)bh * T + i] = k;
            if ((flags & 1u) && ni > 0) mrow[0] = 1;
            int32_t *crow = col_idx + ((size_t)bh * T + i) * T;
            int cnt = 0;
            for (int j = 0; j < T; ++j) if (mrow[j]) crow[cnt++] = j;
            for (int j = cnt; j < T; ++j) crow[j] = -1;
            row_cnt[(size_t)bh * T + i] = cnt;
            if (probs) {
                double *prow = probs + ((size_t)bh * T + i) * T;
                for (int j = 0; j < T; ++j) prow[j] = j < ni ? a[j] : 0.0;
            }
            free(a); free(o);
        }
    free(Qbar); free(Kbar);
    return fail ? 2 : 0;
}

/* ------------------------------------------------------------------------
 * Algorithm 1, the loop over key blocks for ONE query block (b, hq, i), in the
 * online-softmax form of the appendix "FlashAttention" / "Block-Sparse
 * Attention": only the listed blocks are visited, in the listed (ascending)
 * order; a skipped block leaves (O, m, l) untouched.  Entry (row, col) of a
 * visited block takes part iff the key's original position is not after the
 * query's original position (kidx <= qidx; qidx NULL = identity) and the key
 * slot lies inside n; other entries are -inf.  A row whose running maximum is
 * still -inf after a block has nothing to accumulate yet.
 * out: [block, d] (rows past n untouched); lse: [block] or NULL.
 * ---------------------------------------------------------------------- */
static void attn_row_online(int h_q, int h_kv, int n, int d, int block, double scale,
                            const float *Qp, const float *Kp, const float *Vp,
                            const int32_t *qidx, const int32_t *kidx,
                            int T, const int32_t *row_cnt, const int32_t *col_idx,
                            int b, int hq, int i, double *out, double *lse)
{
    const int r = h_q / h_kv, hk = hq / r;
    const size_t qh = (size_t)b * h_q + hq, kh = (size_t)b * h_kv + hk;
    const int rows = (i * block + block <= n) ? block : n - i * block;
    const int cnt = row_cnt[qh * T + i];
    const int32_t *cols = col_idx + (qh * T + i) * (size_t)T;
    double *S = (double *)malloc(sizeof(double) * (size_t)block);
    for (int rr = 0; rr < rows; ++rr) {
        const int qslot = i * block + rr;
        const int32_t qpos = qidx ? qidx[qh * n + qslot] : qslot;
        const float *q = Qp + (qh * n + qslot) * d;
        double m = -INFINITY, l = 0.0;
        double *O = out + (size_t)rr * d;
        for (int e = 0; e < d; ++e) O[e] = 0.0;
        for (int t = 0; t < cnt; ++t) {
            const int j = cols[t];
            double mblk = -INFINITY;
            for (int c = 0; c < block; ++c) {
                const int kslot = j * block + c;
                if (kslot >= n || kidx[kh * n + kslot] > qpos) { S[c] = -INFINITY; continue; }
                const float *k = Kp + (kh * n + kslot) * d;
                double acc = 0.0;
                for (int e = 0; e < d; ++e) acc += (double)q[e] * (double)k[e];
                S[c] = acc * scale;
                if (S[c] > mblk) mblk = S[c];
            }
            const double mnew = mblk > m ? mblk : m;
            if (mnew == -INFINITY) continue;           /* nothing visible yet */
            const double alpha = (m == -INFINITY) ? 0.0 : exp(m - mnew);
            double rowsum = 0.0;
            for (int e = 0; e < d; ++e) O[e] *= alpha;
            for (int c = 0; c < block; ++c) {
                if (S[c] == -INFINITY) continue;
                const double p = exp(S[c] - mnew);
                rowsum += p;
                const float *v = Vp + (kh * n + (size_t)j * block + c) * d;
                for (int e = 0; e < d; ++e) O[e] += p * (double)v[e];
            }
            l = l * alpha + rowsum;
            m = mnew;
        }
        for (int e = 0; e < d; ++e) O[e] = O[e] / l;   /* diag(l)^-1 O */
        if (lse) lse[rr] = m + log(l);
    }
    free(S);
}

/* The same query block by the plain definition: gather every visible
 * (key, value) of the listed blocks, one max-subtracted softmax, one weighted
 * sum.  This is what the online form must equal up to rounding order. */
static void attn_row_direct(int h_q, int h_kv, int n, int d, int block, double scale,
                            const float *Qp, const float *Kp, const float *Vp,
                            const int32_t *qidx, const int32_t *kidx,
                            int T, const int32_t *row_cnt, const int32_t *col_idx,
                            int b, int hq, int i, double *out, double *lse)
{
    const int r = h_q / h_kv, hk = hq / r;
    const size_t qh = (size_t)b * h_q + hq, kh = (size_t)b * h_kv + hk;
    const int rows = (i * block + block <= n) ? block : n - i * block;
    const int cnt = row_cnt[qh * T + i];
    const int32_t *cols = col_idx + (qh * T + i) * (size_t)T;
    double *S = (double *)malloc(sizeof(double) * (size_t)cnt * block + 8);
    for (int rr = 0; rr < rows; ++rr) {
        const int qslot = i * block + rr;
        const int32_t qpos = qidx ? qidx[qh * n + qslot] : qslot;
        const float *q = Qp + (qh * n + qslot) * d;
        double mx = -INFINITY;
        for (int t = 0; t < cnt; ++t)
            for (int c = 0; c < block; ++c) {
                const int kslot = cols[t] * block + c;
                double v = -INFINITY;
                if (kslot < n && kidx[kh * n + kslot] <= qpos) {
                    const float *k = Kp + (kh * n + kslot) * d;
                    double acc = 0.0;
                    for (int e = 0; e < d; ++e) acc += (double)q[e] * (double)k[e];
                    v = acc * scale;
                    if (v > mx) mx = v;
                }
                S[(size_t)t * block + c] = v;
            }
        double sum = 0.0;
        for (size_t u = 0; u < (size_t)cnt * block; ++u)
            if (S[u] != -INFINITY) { S[u] = exp(S[u] - mx); sum += S[u]; } else S[u] = 0.0;
        double *O = out + (size_t)rr * d;
        for (int e = 0; e < d; ++e) O[e] = 0.0;
        for (int t = 0; t < cnt; ++t)
            for (int c = 0; c < block; ++c) {
                const double p = S[(size_t)t * block + c] / sum;
                if (p == 0.0) continue;
                const float *v = Vp + (kh * n + (size_t)cols[t] * block + c) * d;
                for (int e = 0; e < d; ++e) O[e] += p * (double)v[e];
            }
        if (lse) lse[rr] = mx + log(sum);
    }
    free(S);
}

/* Sampled query blocks: rows[3*u + {0,1,2}] = (b, hq, i); out [nrows, block, d];
 * lse [nrows, block] or NULL; direct != 0 selects the plain-definition form. */
int pbso_attn_rows(int batch, int h_q, int h_kv, int n, int d, int block, double scale,
                   const float *Qp, const float *Kp, const float *Vp,
                   const int32_t *qidx, const int32_t *kidx,
                   const int32_t *row_cnt, const int32_t *col_idx,
                   int nrows, const int32_t *rows, int direct, double *out, double *lse)
{
    if (h_kv <= 0 || h_q % h_kv != 0 || block <= 0) return 1;
    const int T = ceil_div(n, block);
    for (int u = 0; u < nrows; ++u)
        if (rows[3 * u] < 0 || rows[3 * u] >= batch || rows[3 * u + 1] < 0 || rows[3 * u + 1] >= h_q ||
            rows[3 * u + 2] < 0 || rows[3 * u + 2] >= T) return 1;
#pragma omp parallel for schedule(dynamic)
    for (int u = 0; u < nrows; ++u) {
        double *o = out + (size_t)u * block * d;
        double *ls = lse ? lse + (size_t)u * block : NULL;
        if (direct)
            attn_row_direct(h_q, h_kv, n, d, block, scale, Qp, Kp, Vp, qidx, kidx, T, row_cnt, col_idx,
                            rows[3 * u], rows[3 * u + 1], rows[3 * u + 2], o, ls);
        else
            attn_row_online(h_q, h_kv, n, d, block, scale, Qp, Kp, Vp, qidx, kidx, T, row_cnt, col_idx,
                            rows[3 * u], rows[3 * u + 1], rows[3 * u + 2], o, ls);
    }
    return 0;
}

/* Whole tensor: Op [batch, h_q, n, d], lse [batch, h_q, n] or NULL. */
int pbso_attn_fwd(int batch, int h_q, int h_kv, int n, int d, int block, double scale,
                  const float *Qp, const float *Kp, const float *Vp,
                  const int32_t *qidx, const int32_t *kidx,
                  const int32_t *row_cnt, const int32_t *col_idx,
                  int direct, double *Op, double *lse)
{
    if (h_kv <= 0 || h_q % h_kv != 0 || block <= 0) return 1;
    const int T = ceil_div(n, block);
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int bh = 0; bh < batch * h_q; ++bh)
        for (int i = 0; i < T; ++i) {
            double *o = Op + ((size_t)bh * n + (size_t)i * block) * d;
            double *ls = lse ? lse + (size_t)bh * n + (size_t)i * block : NULL;
            if (direct)
                attn_row_direct(h_q, h_kv, n, d, block, scale, Qp, Kp, Vp, qidx, kidx, T, row_cnt, col_idx,
                                bh / h_q, bh % h_q, i, o, ls);
            else
                attn_row_online(h_q, h_kv, n, d, block, scale, Qp, Kp, Vp, qidx, kidx, T, row_cnt, col_idx,
                                bh / h_q, bh % h_q, i, o, ls);
        }
    return 0;
}

/* ------------------------------------------------------------------------
 * Dense causal attention on the ORIGINAL order (appendix "Scaled Dot-Product
 * Attention" with the lower-triangular restriction of Section "Segmented
 * Permutation for Causal Attention"): O[t] = softmax_{u<=t}(q_t.k_u*scale) V.
 * Used only as the right-hand side of Theorem 1.
 * ---------------------------------------------------------------------- */
int pbso_dense_causal(int batch, int h_q, int h_kv, int n, int d, double scale,
                      const float *Q, const float *K, const float *V, double *O)
{
    if (h_kv <= 0 || h_q % h_kv != 0) return 1;
    const int r = h_q / h_kv;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int bh = 0; bh < batch * h_q; ++bh)
        for (int t = 0; t < n; ++t) {
            const size_t kh = (size_t)(bh / h_q) * h_kv + (bh % h_q) / r;
            const float *q = Q + ((size_t)bh * n + t) * d;
            double *w = (double *)malloc(sizeof(double) * (size_t)(t + 1));
            double mx = -INFINITY;
            for (int u = 0; u <= t; ++u) {
                const float *k = K + (kh * n + u) * d;
                double acc = 0.0;
                for (int e = 0; e < d; ++e) acc += (double)q[e] * (double)k[e];
                w[u] = acc * scale;
                if (w[u] > mx) mx = w[u];
            }
            double sum = 0.0;
            for (int u = 0; u <= t; ++u) { w[u] = exp(w[u] - mx); sum += w[u]; }
            double *o = O + ((size_t)bh * n + t) * d;
            for (int e = 0; e < d; ++e) o[e] = 0.0;
            for (int u = 0; u <= t; ++u) {
                const double p = w[u] / sum;
                const float *v = V + (kh * n + u) * d;
                for (int e = 0; e < d; ++e) o[e] += p * (double)v[e];
            }
            free(w);
        }
    return 0;
}

int pbso_num_threads(void)
{
    int nt = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        nt = omp_get_num_threads();
    }
#endif
    return nt;
}
