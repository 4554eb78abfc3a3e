/*
 * pbs.h -- C ABI of the MI355X-native PBS-Attn prefill path.
 *
 * PBS-Attn = Permuted Block-Sparse Attention (arXiv 2510.21270).  One prefill
 * attention forward pass is Algorithm 1 of the paper:
 *
 *   pbs_key_scores      Eq. 4   global importance score of every key
 *   pbs_segment_permute Eq. 5   per-segment descending argsort + K', V' = P_pi K, P_pi V
 *   pbs_block_mask      Alg. 2  mean-pooled cumulative-mass block selection on (Q', K')
 *   pbs_attn_fwd        Alg. 1  online-softmax attention over the selected blocks only
 *   pbs_unpermute       Alg. 1  O = P_sigma^T O'   (Theorem 1)
 *
 * General conventions
 *   - Every tensor pointer is a DEVICE pointer to caller-owned, contiguous,
 *     row-major memory, 16-byte aligned.  The library never allocates, frees
 *     or synchronises; all work is enqueued on `stream` (a hipStream_t passed
 *     as void*, NULL = the default stream) and is complete when the stream is.
 *   - `pbs_problem` itself is a HOST pointer and is read during the call only.
 *   - Arguments are validated on the host before anything is launched; a bad
 *     call returns a status and enqueues nothing.  A failed launch returns
 *     PBS_ERR_HIP.  Nothing throws or aborts.
 *   - Q is [batch, h_q, n, d]; K and V are [batch, h_kv, n, d]; h_q % h_kv == 0
 *     and query head h reads kv head h / (h_q / h_kv)  (grouped-query attention;
 *     one permutation per kv head, the "shared permutation strategy" of the
 *     appendix "GQA Handling"; the replicated default of the paper is the case
 *     h_kv == h_q).
 *   - T = ceil(n / block) blocks; segment % block == 0; R = segment / block;
 *     G = floor(n / segment) full segments; tokens at or beyond G * segment are
 *     never permuted (Section "Segmented Permutation for Causal Attention").
 *   - Index vectors are in gather form with absolute positions: slot p of a
 *     permuted tensor holds original token idx[p], and idx maps every segment
 *     onto itself.
 *   - K' ("Kp") keeps the [batch, h_kv, n, d] layout.  V' is kept as "Vt":
 *     [batch, h_kv, T, block / G, d, G] with G = min(block, 32), i.e. every
 *     key block stored as groups of G consecutive key slots, each group
 *     transposed (feature-major), the slots past n in the last block
 *     zero-filled.  Vt is produced by pbs_segment_permute and consumed by
 *     pbs_attn_fwd; pbs_vt_bytes gives its size.
 *   - Supported: dtype PBS_BF16 or PBS_F32; d in {64, 128}; block in
 *     {16, 32, 64, 128}; segment <= 4096; T <= 4096; any n >= 1.  The matrix-core
 *     attention kernel serves PBS_BF16 with d = 128 and block in {64, 128};
 *     every other supported combination runs on fp32 vector arithmetic.
 *   - Results are deterministic: the same inputs give bit-identical outputs.
 */
#ifndef PBS_H
#define PBS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PBS_OK = 0,
    PBS_ERR_NULL = 1,        /* a required pointer is NULL */
    PBS_ERR_SHAPE = 2,       /* inconsistent sizes (h_q % h_kv, segment % block, n < 1, ...) */
    PBS_ERR_UNSUPPORTED = 3, /* valid problem outside the supported set listed above */
    PBS_ERR_WORKSPACE = 4,   /* ws_bytes smaller than pbs_workspace_bytes(), or ws misaligned */
    PBS_ERR_HIP = 5          /* a kernel launch failed */
} pbs_status;

typedef enum { PBS_F32 = 0, PBS_BF16 = 1 } pbs_dtype;

/*
 * PBS_FLAG_FORCE_FIRST_BLOCK: Algorithm 2 also keeps key block 0 in every row.
 * PBS_FLAG_TOKEN_ORDER_COPY: K', Vt and kidx each carry a second tensor of the same shape in token order (K
 *   itself, V block-transposed without permutation, kidx = 0 .. n-1) in the same allocation, starting
 *   batch * h_kv * T * block rows (K': rows of d elements; kidx: entries; Vt: key slots of d elements, i.e. directly
 *   behind the first tensor) after the start of the permuted one; each buffer therefore holds
 *   batch * h_kv * (T * block + n) rows (Vt: 2 * batch * h_kv * T * block).  pbs_segment_permute writes both; every
 *   other stage reads the first tensor as before, and pbs_attn_fwd may evaluate a query block's own segment from
 *   the second (see there).  The result is the same attention: the order in which keys are summed does not matter
 *   (Theorem 1).
 * PBS_FLAG_RUNNING_MAX_ONLY: pbs_attn_fwd evaluates every query block with the running-maximum recurrence of
 *   Algorithm 1 as printed (m moves and O, l are rescaled); for bf16, d = 128, block = 128 this leaves out the first
 *   pass, which keeps a fixed softmax reference per query.  Same result up to rounding; slower.
 * PBS_FLAG_KBAR_IN_WS: the workspace given to pbs_block_mask already holds the block means of Kp, left there by
 *   the pbs_segment_permute call that wrote this Kp (see its `ws`); pbs_block_mask then does not read Kp at all.
 * PBS_FLAG_INDEX_REMAP: index remapping as the appendix "Memory Overhead" sketches it (the attention kernel retrieves
 *   the keys from the original tensor through the permuted indices): no K' exists.  pbs_segment_permute writes kidx
 *   and Vt only (its Kp argument is ignored and may be NULL; with a workspace it still leaves the block means of the
 *   permuted keys there), pbs_block_mask must then be given PBS_FLAG_KBAR_IN_WS as well, and pbs_attn_fwd takes the
 *   caller's K in place of Kp and gathers the rows kidx[slot] while it stages its tiles.  bf16, d = 128, block 64 or
 *   128 only (PBS_ERR_UNSUPPORTED otherwise, and together with PBS_FLAG_TOKEN_ORDER_COPY); same results as with a
 *   materialised K', bit for bit against PBS_FLAG_RUNNING_MAX_ONLY (it runs on that kernel).  V' stays materialised
 *   as Vt: the second matrix product needs it feature-major.
 */
enum { PBS_FLAG_FORCE_FIRST_BLOCK = 1u, PBS_FLAG_TOKEN_ORDER_COPY = 2u, PBS_FLAG_RUNNING_MAX_ONLY = 4u,
       PBS_FLAG_KBAR_IN_WS = 8u, PBS_FLAG_INDEX_REMAP = 16u };

typedef enum {
    PBS_STAGE_KEY_SCORES = 1,
    PBS_STAGE_SEGMENT_PERMUTE = 2,
    PBS_STAGE_BLOCK_MASK = 3,
    PBS_STAGE_ATTN_FWD = 4,
    PBS_STAGE_UNPERMUTE = 5,
    PBS_STAGE_QUERY_PERMUTE = 6   /* pbs_query_permutation, an ablation outside Algorithm 1's main setting */
} pbs_stage;

typedef struct {
    int32_t batch, h_q, h_kv, n, d;
    int32_t block;    /* B of the paper */
    int32_t segment;  /* S of the paper */
    int32_t dtype;    /* pbs_dtype of Q, K, V, K', Vt, O', O */
    float tau;        /* mass threshold of Alg. 2, compared as (double)tau */
    float scale;      /* logit scale; 0 means 1/sqrt(d) (formed in double where the arithmetic is fp64) */
    uint32_t flags;   /* PBS_FLAG_* */
} pbs_problem;

/* Static string for a status code (never NULL). */
const char *pbs_status_string(pbs_status st);

/* PBS_OK when the problem is inside the supported set, else the status every stage would return. */
pbs_status pbs_validate(const pbs_problem *p);

/* Bytes of scratch a stage needs in `ws` (256-byte aligned device memory); 0 for an invalid problem. */
size_t pbs_workspace_bytes(const pbs_problem *p, int stage);

/* Bytes of the Vt tensor: batch * h_kv * T * d * block elements of the problem's dtype, twice that with
 * PBS_FLAG_TOKEN_ORDER_COPY. */
size_t pbs_vt_bytes(const pbs_problem *p);

/*
 * Eq. 4, with the queries of a GQA group averaged (appendix "GQA Handling"):
 *   Qhat = mean over the group's query heads of the last min(block, n) rows of Q,
 *   scores = mean_rows( softmax_over_all_n_keys( Qhat K^T * scale ) ).
 * No causal mask (Eq. 4 has none).  Q [batch,h_q,n,d] (only the last rows are read), K [batch,h_kv,n,d]
 * -> scores [batch,h_kv,n] float32.  bf16 inputs: matrix cores with an fp32 accumulator and a two-term
 * split of Qhat; fp32 inputs: fp64 accumulation.
 */
pbs_status pbs_key_scores(const pbs_problem *p, const void *Q, const void *K, float *scores,
                          void *ws, size_t ws_bytes, void *stream);

/*
 * The other proxies for the importance score that the paper ablates (Section "The Problem of Information
 * Fragmentation", heuristic 4; appendix "Task-wise Proxy Sensitivity"): the formula of Eq. 4 with another set of
 * query rows standing for all queries.
 *   PBS_PROXY_LAST_BLOCK   the last min(block, n) rows: exactly pbs_key_scores (Last-Block-Query-Attn).
 *   PBS_PROXY_QUERY_ROWS   the m rows at the positions qrows[0 .. m-1] (device memory, int32, the same positions for
 *                          every head; 1 <= m <= 128; a position outside [0, n) is clamped into it; a position listed
 *                          twice counts twice).  With positions drawn at random by the caller: Random-Query-Attn.
 *   PBS_PROXY_AVG_QUERY    one query: the mean over all n positions of the group-averaged query vectors (the reading
 *                          taken of Avg-Query-Attn, which the paper only names); Q is read in full.
 * No causal mask, as in Eq. 4.  Arguments, workspace and precision otherwise as pbs_key_scores.
 * Errors: as pbs_key_scores, plus PBS_ERR_UNSUPPORTED for an unknown proxy, PBS_ERR_NULL / PBS_ERR_SHAPE for a
 * missing qrows / an m outside [1, 128].
 */
typedef enum { PBS_PROXY_LAST_BLOCK = 0, PBS_PROXY_QUERY_ROWS = 1, PBS_PROXY_AVG_QUERY = 2 } pbs_proxy;
pbs_status pbs_key_scores_proxy(const pbs_problem *p, int proxy, const int32_t *qrows, int32_t m, const void *Q,
                                const void *K, float *scores, void *ws, size_t ws_bytes, void *stream);

/*
 * For callers that cannot allocate or pass scratch memory (code under HIP graph capture that owns no workspace,
 * tight serving loops, harnesses that forbid hipMalloc): pbs_key_scores with its scratch memory in a device array
 * that is part of the library image instead of in `ws`.  Same arguments otherwise, same kernels, bit-identical
 * scores.  Allocates nothing and calls no allocating routine.
 *   The array holds pbs_key_scores_static_scratch_bytes() = 4 MiB on every GPU the library runs on, until the
 *   process ends; a problem whose pbs_workspace_bytes(p, PBS_STAGE_KEY_SCORES) is larger is rejected with
 *   PBS_ERR_WORKSPACE and nothing is enqueued (the headline layer, 8 kv heads x 131072 keys, needs 2.6 MiB).
 *   All calls on one GPU share that GPU's array: two calls whose kernels may overlap in time (different streams,
 *   or different host threads without ordering between their streams) race on it; calls on one stream are safe.
 *   Nothing in the array has to be cleared between calls: every word that a call reads it has written before.
 * Errors: as pbs_key_scores, plus PBS_ERR_HIP when the array's address cannot be obtained on the current device.
 */
pbs_status pbs_key_scores_static(const pbs_problem *p, const void *Q, const void *K, float *scores, void *stream);
size_t pbs_key_scores_static_scratch_bytes(void);

/*
 * Eq. 5 inside each full segment: kidx[g*S + t] = g*S + (position of the t-th largest score of segment g),
 * equal scores in ascending position (stable), tail positions kept (identity).  Then Algorithm 1's first
 * step for keys and values: Kp[slot] = K[kidx[slot]], Vt = block-transposed V[kidx[.]].
 *   scores [batch,h_kv,n] float32, or NULL for the identity permutation (the unpermuted MeanPooling
 *     baseline of the appendix "Block Selection in PBS-Attn": K' = K, V' = V).  NaN scores are not supported.
 *   kidx   [batch,h_kv,n] int32, written.
 *   Kp, Vt written; pass both NULL to compute kidx only (K and V may then be NULL too).
 *   ws: optional.  NULL: nothing more.  Otherwise at least pbs_workspace_bytes(p, PBS_STAGE_BLOCK_MASK) bytes,
 *   256-byte aligned (else PBS_ERR_WORKSPACE): the block means of K' that Algorithm 2 starts from are written there
 *   while K' is gathered (the first step of pbs_block_mask moved up one stage, so that K' is not read again for it);
 *   hand the same memory to pbs_block_mask with PBS_FLAG_KBAR_IN_WS set.  Ignored when Kp is NULL.
 */
pbs_status pbs_segment_permute(const pbs_problem *p, const float *scores, const void *K, const void *V,
                               int32_t *kidx, void *Kp, void *Vt, void *ws, size_t ws_bytes, void *stream);

/*
 * Algorithm 1's first step for any [batch, heads, n, d] tensor: Xp[slot] = X[idx[slot]] (Q' = P_sigma Q for a
 * caller-supplied segment-wise sigma; the paper's main setting P_sigma = I needs no call).
 * idx [batch,heads,n] int32 with values in [0, n); an out-of-range entry yields a zero row.
 */
pbs_status pbs_permute_rows(const pbs_problem *p, int32_t heads, const void *X, const int32_t *idx, void *Xp,
                            void *stream);

/*
 * Key-aware query permutation, the ablation of Section "Design Choice: Why Permute Keys but not Queries?" (the
 * paper's main setting keeps P_sigma = I and needs no call).  Centroids Kbar_j = block means of Kc (the keys the
 * queries will attend to: K, or K' when the keys are permuted first; valid rows only in a partial last block).  Every
 * query of a full segment g is assigned to the centroid of highest cosine similarity among those its segment may see,
 * j < (g+1)*R capped at T, ties to the lowest j; sigma orders the queries of the segment by assigned centroid,
 * ascending, queries of one centroid in their original order; tokens past the last full segment keep their place.
 * ("Assigned greedily" is read as: every query takes its single best centroid, no capacity, no reassignment.)
 *   Q [batch,h_q,n,d]; Kc [batch,h_kv,n,d]; qidx [batch,h_q,n] int32 written, gather form with absolute positions:
 *   Q'[slot] = Q[qidx[slot]] (pbs_permute_rows), O[qidx[slot]] = O'[slot] (pbs_unpermute).
 *   ws: pbs_workspace_bytes(p, PBS_STAGE_QUERY_PERMUTE) bytes.  IEEE fp64, features in ascending order, separate
 *   multiplications and additions: the assignment does not depend on the machine.
 * Errors: PBS_ERR_NULL, PBS_ERR_SHAPE (misaligned), PBS_ERR_WORKSPACE, the statuses of pbs_validate, PBS_ERR_HIP.
 */
pbs_status pbs_query_permutation(const pbs_problem *p, const void *Q, const void *Kc, int32_t *qidx, void *ws,
                                 size_t ws_bytes, void *stream);

/*
 * Algorithm 2 on the permuted (Q', K'), per query head:
 *   block means (valid rows only in a partial last block);
 *   a_i = softmax_j(Qbar_i . Kbar_j * scale) over the columns the extended causal mask C admits:
 *         j < (g(i)+1)*R for a query block inside full segment g(i), j <= i past the last full segment;
 *   stable descending sort (ties: lowest j), cumulative sum, k = min({t : c[t] >= tau} U {n_i}), first k kept.
 * All of this is IEEE fp64 in the order of the definition (block means: rows ascending for fp32 storage; for bf16
 * storage any order gives the exact sum; logits: features ascending), so that the discrete result does not depend
 * on how a machine rounds lower precision.  Where the evaluation differs from a plain left-to-right one with
 * separate multiplications and additions, it does so by single roundings: the logits use fused multiply-adds (the
 * same bits whenever the products are exact, as they are for block means of bf16 values unless one column of a block
 * spreads over more than about ten binades), and two sums are formed in a tree order (the softmax denominator and
 * the partial masses the threshold search compares with tau).  A selection can then differ from the plain
 * evaluation only if a cumulative mass lies within a few 1e-16 of tau.  Then the blocks of the
 * query block's own segment are switched on (Section "Effect of Segment Size": they cannot be skipped); past the
 * last full segment only the diagonal block; and block 0 when PBS_FLAG_FORCE_FIRST_BLOCK is set (Section
 * "Baselines").  Forced blocks do not change k.
 *   mask_bits [batch,h_q,T,ceil(T/64)] uint64, bit (j & 63) of word (j >> 6) of row i = M[i][j];
 *   row_cnt   [batch,h_q,T] int32; col_idx [batch,h_q,T,T] int32, the first row_cnt[i] entries of row i are the
 *   selected j ascending, the rest is left untouched.
 */
pbs_status pbs_block_mask(const pbs_problem *p, const void *Qp, const void *Kp, uint64_t *mask_bits,
                          int32_t *row_cnt, int32_t *col_idx, void *ws, size_t ws_bytes, void *stream);

/*
 * Algorithm 1's main loop: for every query block i, over the listed key blocks only (a block that is not
 * listed leaves the running (O, m, l) untouched): S = Q'_i K'_j^T * scale, online softmax, O'_i = diag(l)^-1 O.
 * Inside the query block's own segment, and in the unpermuted tail, entry (row, col) takes part only if the
 * key's original position is not after the query's: kidx[j*block+col] <= qidx[i*block+row]; key slots >= n never
 * take part.  Listed blocks outside the columns C admits are ignored.  A query row that sees no key at all gets
 * a zero output row and lse = -inf (cannot happen when the diagonal block is listed).
 *   Qp [batch,h_q,n,d]; Kp [batch,h_kv,n,d]; Vt as above; qidx [batch,h_q,n] or NULL (identity);
 *   kidx [batch,h_kv,n]; row_cnt, col_idx as written by pbs_block_mask (any order of the listed blocks is
 *   accepted); Op [batch,h_q,n,d] written; lse [batch,h_q,n] float32 or NULL: log-sum-exp of the visible,
 *   listed logits of every query row.
 *   ws: pbs_workspace_bytes(p, PBS_STAGE_ATTN_FWD) bytes, 256-byte aligned device memory (0 bytes, and ws may be NULL,
 *   unless dtype is bf16 with d = 128 and block = 128).  For that shape the call launches two kernels on the stream:
 *   one that keeps a fixed softmax reference per query and writes one int32 flag per query block into ws (1 = some
 *   probability outgrew the reference by more than 2^64), and one that recomputes the flagged query blocks with the
 *   running-maximum recurrence of Algorithm 1.  The contents of ws need not be initialised and mean nothing afterwards.
 *   With PBS_FLAG_RUNNING_MAX_ONLY every query block of that shape goes through the second kernel alone.
 *   With PBS_FLAG_TOKEN_ORDER_COPY (Kp, Vt, kidx carry their token-order copies), qidx == NULL and that same shape, a
 *   query block inside a full segment whose list ends with all R blocks of its own segment, ascending (as
 *   pbs_block_mask writes them), takes these R blocks from the token-order copy instead: the blocks before the
 *   diagonal in full, the diagonal block under the causal test, none after it.  These are the same visible keys,
 *   so O' and lse are the same up to the rounding order of the sums; every other list is processed as listed.
 */
pbs_status pbs_attn_fwd(const pbs_problem *p, const void *Qp, const void *Kp, const void *Vt,
                        const int32_t *qidx, const int32_t *kidx, const int32_t *row_cnt, const int32_t *col_idx,
                        void *Op, float *lse, void *ws, size_t ws_bytes, void *stream);

/*
 * Algorithm 1's last step (Theorem 1): O[qidx[slot]] = Op[slot].  qidx NULL (P_sigma = I, the paper's main
 * setting) makes this a plain copy, or nothing at all when O == Op.  Op, O [batch,h_q,n,d]; O must not
 * partially overlap Op.
 */
pbs_status pbs_unpermute(const pbs_problem *p, const void *Op, const int32_t *qidx, void *O, void *stream);

/*
 * Coverage tooling for the block-selection objective of Section "The Problem of Information Fragmentation" (the
 * attention mass, softmax over every visible key, that falls into the selected blocks); not a step of Algorithm 1.
 * pbs_admitted_lists writes the lists that name every key block the extended causal mask C admits (appendix "Block
 * Selection in PBS-Attn"): row_cnt[b,h,i] = (g(i)+1)*R capped at T inside full segment g(i), i+1 past the last full
 * segment; col_idx[b,h,i,0..row_cnt) = 0, 1, ...  (shapes as for pbs_block_mask; the rest of col_idx is untouched).
 * pbs_mass_covered combines the log-sum-exp outputs of two pbs_attn_fwd calls, one over a selection and one over the
 * admitted lists: covered[b,h,slot] = exp(lse_listed - lse_admitted), 0 where lse_listed is -inf.  All three
 * [batch,h_q,n] float32; covered may alias either input.
 * Errors: PBS_ERR_NULL, the statuses of pbs_validate, PBS_ERR_HIP.
 */
pbs_status pbs_admitted_lists(const pbs_problem *p, int32_t *row_cnt, int32_t *col_idx, void *stream);
pbs_status pbs_mass_covered(const pbs_problem *p, const float *lse_listed, const float *lse_admitted, float *covered,
                            void *stream);

/*
 * Measurement aids, not steps of Algorithm 1.
 * pbs_mfma_rate_probe launches a kernel that does nothing but bf16 matrix instructions (four waves per SIMD on 256
 * compute units, operands in registers, no other instruction in the loop) for `iters` rounds of 32 instructions, with
 * all-zero operands (random_operands = 0) or pseudo-random ones.  The caller times the launch on `stream`; *flop (host
 * memory) receives the number of floating-point operations it performs.  The instruction rate per clock is the same
 * in both cases; the clock the chip grants under matrix load depends on the operand bits, so the rate with random
 * operands is the matrix rate a kernel working on real data can approach.
 *   sink: device memory, sink_floats >= 262144 float32, overwritten; afterwards sink[0] = shader clock in MHz that one
 *   wave of the launch saw, sink[1] = that wave's clocks per matrix instruction (four waves share a SIMD: 4 x 32 in a
 *   long run).  iters in [1, 2^22].
 * pbs_shader_clock_meter launches one wave that compares the shader-clock counter with the constant 100 MHz counter
 * for about `micros` microseconds (1 .. 2 000 000) and writes out[0] = shader clock in MHz, out[1] = microseconds
 * watched (device memory, 2 floats).  Launched on a second stream beside another kernel it reports that kernel's clock.
 * Errors: PBS_ERR_NULL, PBS_ERR_SHAPE (a size or count out of range), PBS_ERR_HIP.
 */
pbs_status pbs_mfma_rate_probe(int random_operands, int iters, float *sink, size_t sink_floats, double *flop,
                               void *stream);
pbs_status pbs_shader_clock_meter(float *out, int micros, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* PBS_H */
