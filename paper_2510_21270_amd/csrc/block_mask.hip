// pbs_block_mask: Algorithm 2 (MeanPooling block selection) on the permuted (Q', K') plus the forced blocks.
//
// Everything that decides the discrete result runs in IEEE fp64 in the order of the definition, so the mask does not
// depend on how a machine rounds lower precision (the logits use fused multiply-adds: the same bits as separate
// operations whenever the products of two block means are exact, which 15 + 15 significant bits plus the exponent
// spread inside a block's column usually are):
//   1. pool_kernel     block means of K' (HBM-bound), stored d-major ([head][e][T]) so that the next kernel reads
//                      them coalesced.  A sum of up to 128 bf16 values is exact in fp64 in any order (8 significant
//                      bits each; the exponents of one column would have to spread over more than 38 binades to lose
//                      a bit), so bf16 inputs are summed in whatever order loads best.  fp32 values have 24 significant
//                      bits and no such slack: they are added one row after the other, in ascending order, which
//                      is the order of the plain definition.
//   2. select_kernel   block means of its own Q' blocks, then logits of up to four query heads of one group against
//                      the allowed columns, softmax, the mass threshold by bisection (one wave per row), forced
//                      blocks, then bit-mask words by wave ballot and the ascending column list by prefix popcount.
#include "pbs_host.h"

namespace pbs {

// ---------------------------------------------------------------------------------------------
// grid = (T, heads); E = input element type.  TRANSPOSED: write out[head][e][Ts] (row stride Ts >= T) instead of
// out[head][i][e].
// 256 threads: thread (cg = tid % cpr, rg = tid / cpr) sums its 16-byte column group over rows rg, rg+RG, ...
// ---------------------------------------------------------------------------------------------
template <typename E, bool TRANSPOSED>
__global__ __launch_bounds__(256) void pool_kernel(const E *__restrict__ X, double *__restrict__ out, int n, int d,
                                                   int block, int T, int Ts)
{
    constexpr int VEC = 16 / sizeof(E);
    typedef E vec_t __attribute__((ext_vector_type(VEC)));
    __shared__ double red[256 * VEC];                       // [rg][cg][VEC] flattened as tid * VEC
    const int i = blockIdx.x;
    const size_t head = blockIdx.y;
    const int cpr = d / VEC;                                // 8..32
    const int RG = 256 / cpr;
    const int cg = threadIdx.x % cpr, rg = threadIdx.x / cpr;
    const int lo = i * block, hi = min(n, lo + block);
    if constexpr (sizeof(E) == 4) {
        // fp32 storage: thread e owns column e and adds its rows in ascending order
        if ((int)threadIdx.x < d) {
            const int e = threadIdx.x;
            double s = 0.0;
            for (int row = lo; row < hi; ++row) s += (double)ElemTraits<E>::to_float(X[(head * n + row) * (size_t)d + e]);
            const double mean = s / (double)(hi - lo);
            if (TRANSPOSED) out[(head * d + e) * (size_t)Ts + i] = mean;
            else out[(head * T + i) * (size_t)d + e] = mean;
        }
        return;
    }
    double acc[VEC];
#pragma unroll
    for (int u = 0; u < VEC; ++u) acc[u] = 0.0;
    // four independent 16-byte loads in flight per thread (bf16: the sums are exact in fp64 whatever the order)
    constexpr int U = 4;
    for (int row = lo + rg; row < hi; row += U * RG) {
        vec_t v[U];
#pragma unroll
        for (int q = 0; q < U; ++q) {
            v[q] = vec_t{};
            if (row + q * RG < hi)
                v[q] = *reinterpret_cast<const vec_t *>(X + (head * n + row + q * RG) * (size_t)d + cg * VEC);
        }
#pragma unroll
        for (int q = 0; q < U; ++q)
            if (row + q * RG < hi)
#pragma unroll
                for (int u = 0; u < VEC; ++u) acc[u] += (double)ElemTraits<E>::to_float(v[q][u]);
    }
#pragma unroll
    for (int u = 0; u < VEC; ++u) red[threadIdx.x * VEC + u] = acc[u];
    __syncthreads();
    if ((int)threadIdx.x < d) {
        const int e = threadIdx.x, c = e / VEC, u = e % VEC;
        double s = 0.0;
        for (int q = 0; q < RG; ++q) s += red[(q * cpr + c) * VEC + u];
        const double mean = s / (double)(hi - lo);
        if (TRANSPOSED) out[(head * d + e) * (size_t)Ts + i] = mean;
        else out[(head * T + i) * (size_t)d + e] = mean;
    }
}

// ---------------------------------------------------------------------------------------------
// Selection.  One workgroup per (kv head, chunk of RB query heads of its group, query block i): the RB rows
// share the allowed columns and the pooled keys.  The logits are register-tiled: a thread owns four neighbouring
// columns of all RB rows, so the two 16-byte loads that bring one feature of its four pooled keys and the (at most)
// two 16-byte LDS reads that bring that feature of the RB pooled queries feed 4 * RB fused multiply-adds; every sum
// runs over the features in ascending order.  After the
// logits, wave w owns row w and finishes it alone (no workgroup barriers): softmax, then the smallest
// probability v* that is still kept, found by bisection instead of a sort.
//
// The kept set of Algorithm 2 is the shortest prefix of the order (probability descending, column ascending)
// whose mass reaches tau.  With M(v) = sum of the probabilities >= v, v* is the largest v with M(v) >= tau:
// every probability above v* is kept, and of the columns that tie at v* the first m by column index, m being
// the number of additions of v* to M(> v*) that reach tau.  The bisection runs over the bit patterns of the
// non-negative doubles between the smallest and the largest probability and stops as soon as a single
// element, or a single bit pattern, is left in the bracket.
// ---------------------------------------------------------------------------------------------
struct MassCount {
    double mass;
    int cnt;
};

// mass and number of the row's probabilities >= v; pr is padded with -1 up to a multiple of 64
__device__ inline MassCount mass_at_least(const double *pr, int ni64, int lane, double v)
{
    double acc = 0.0;
    int cnt = 0;
    for (int j0 = 0; j0 < ni64; j0 += 64) {
        const double x = pr[j0 + lane];
        const bool ge = x >= v;
        acc += ge ? x : 0.0;
        cnt += __popcll(__ballot(ge));
    }
    return {wave_sum_dpp(acc), cnt};
}

// QB query blocks (i0 = QB * blockIdx.x and the next ones) of RB query heads per workgroup: RT = RB * QB rows, one wave
// each.  Neighbouring query blocks see the same pooled keys (the later one a few more columns), so with QB = 2 a
// 16-byte load of pooled keys feeds twice the multiply-adds and the logits need half the round trips to L2.
// Query blocks are taken from the last one down: the long rows start first, the short ones fill the tail.
constexpr int kPairedLds = 64 * 1024;

template <int RB, int QB, typename E>
__global__ __launch_bounds__(64 * RB * QB) __attribute__((amdgpu_waves_per_eu(1, 4)))
void select_kernel(const E *__restrict__ Qp,           // [bhq][n][d]
                   const double *__restrict__ KbarT,   // [bhkv][d][Ts]
                   uint64_t *__restrict__ mask_bits, int32_t *__restrict__ row_cnt, int32_t *__restrict__ col_idx,
                   Geo g, int chunks, int Tpad, int Ts)
{
    constexpr int RT = RB * QB;                                      // rows (= waves) of the workgroup
    constexpr int THREADS = 64 * RT;
    constexpr int CT = 4 / QB;                                       // columns per thread: 4 * 64 * RB per pass
    constexpr int FD = 4 * QB;                                       // features per register buffer
    static_assert(QB == 1 || QB == 2, "column tile is one or two 16-byte loads");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    double *prob = reinterpret_cast<double *>(smem_raw);             // [RT][Tpad]
    __shared__ __align__(16) double qs[128][RT];                     // block means of the RT query rows, feature-major

    const int i0 = (g.T - 1) / QB * QB - QB * (int)blockIdx.x;       // first query block of this workgroup
    const int bhk = blockIdx.y / chunks, chunk = blockIdx.y % chunks;
    const int b = bhk / g.h_kv, hk = bhk % g.h_kv;
    const int rows = min(RB, g.r - chunk * RB);                      // query heads handled here
    const int bhq0 = b * g.h_q + hk * g.r + chunk * RB;
    const int tid = threadIdx.x;
    const int w = tid >> 6, lane = tid & 63;
    const int wq = w / RB, wh = w % RB;                              // this wave's query block (i0 + wq) and head
    const int i = i0 + wq;
    const bool active = i < g.T && wh < rows;
    const int nblk = min(QB, g.T - i0);                              // query blocks present
    const int ni_all = allowed_cols(i0 + nblk - 1, g);               // the last one sees the most columns

    // Block mean of query block i of head wh, by wave w (sums of storage values in fp64; 16-byte column groups,
    // sixteen loads in flight per lane, then the row groups of the wave are added up).  Pooling Q' here instead of in
    // a kernel of its own lets the 1 GiB read of Q' overlap with the arithmetic of other workgroups.
    // fp32 storage: every lane owns columns and adds their rows in ascending order (see the note at the top).
    if constexpr (sizeof(E) == 4) {
        const int lo = i * g.block, hi = min(g.n, lo + g.block);
        if (active) {
            const E *X = Qp + (size_t)(bhq0 + wh) * g.n * g.d;
            for (int e = lane; e < g.d; e += 64) {
                double s = 0.0;
                for (int row = lo; row < hi; ++row) s += (double)ElemTraits<E>::to_float(X[(size_t)row * g.d + e]);
                qs[e][w] = s / (double)(hi - lo);
            }
        }
    } else {
        constexpr int VEC = 16 / sizeof(E);
        typedef E vec_t __attribute__((ext_vector_type(VEC)));
        const int cpr = g.d / VEC;                                   // 8 .. 32 column groups
        const int RG = 64 / cpr;                                     // row groups of a wave
        const int cg = lane % cpr, rg = lane / cpr;
        const int lo = i * g.block, hi = min(g.n, lo + g.block);
        double acc[VEC];
#pragma unroll
        for (int u = 0; u < VEC; ++u) acc[u] = 0.0;
        if (active) {
            // (a block of 128 rows of 256 bytes is two rounds): the read of Q' is the one large HBM stream of this
            // kernel and a workgroup does nothing else while it waits for it
            constexpr int U = 16;
            const E *X = Qp + (size_t)(bhq0 + wh) * g.n * g.d + cg * VEC;
            for (int r0 = lo + rg; r0 < hi; r0 += U * RG) {
                vec_t v[U];
#pragma unroll
                for (int q = 0; q < U; ++q) {
                    v[q] = vec_t{};
                    if (r0 + q * RG < hi) v[q] = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(X + (size_t)(r0 + q * RG) * g.d));
                }
#pragma unroll
                for (int q = 0; q < U; ++q)
                    if (r0 + q * RG < hi)
#pragma unroll
                        for (int u = 0; u < VEC; ++u) acc[u] += (double)ElemTraits<E>::to_float(v[q][u]);
            }
        }
        for (int o = cpr; o < 64; o <<= 1)
#pragma unroll
            for (int u = 0; u < VEC; ++u) acc[u] += __shfl_xor(acc[u], o, 64);
        if (rg == 0 && active)
#pragma unroll
            for (int u = 0; u < VEC; ++u) qs[cg * VEC + u][w] = acc[u] / (double)(hi - lo);
    }
    __syncthreads();

    // logits: fused multiply-adds in the order e = 0..d-1; columns j .. j + CT - 1 of every row per thread (columns at
    // or beyond a row's own count are computed from whatever the padded Kbar rows hold and never read; rows that are
    // not there from whatever qs holds).  Two register buffers of FD features each, filled alternately: the loads of
    // one are in flight while the other is multiplied (scheduling barriers keep the compiler from moving a buffer's
    // loads down to its use).
    const double *kt = KbarT + (size_t)bhk * g.d * Ts;
    typedef double double2v __attribute__((ext_vector_type(2)));
    for (int j = CT * tid; j < ni_all; j += CT * THREADS) {
        double acc[RT][CT];
#pragma unroll
        for (int row = 0; row < RT; ++row)
#pragma unroll
            for (int c = 0; c < CT; ++c) acc[row][c] = 0.0;
        double kva[FD][CT], kvb[FD][CT];
        auto fetch = [&](double (&kv)[FD][CT], int e) {
            const int ec = e < g.d ? e : g.d - FD;             // past the end: re-read the last features (unused)
#pragma unroll
            for (int u = 0; u < FD; ++u) {
                const double *src = kt + (size_t)(ec + u) * Ts + j;
                const double2v lo2 = *reinterpret_cast<const double2v *>(src);
                kv[u][0] = lo2[0];
                kv[u][1] = lo2[1];
                if constexpr (CT == 4) {
                    const double2v hi2 = *reinterpret_cast<const double2v *>(src + 2);
                    kv[u][2] = hi2[0];
                    kv[u][3] = hi2[1];
                }
            }
        };
        auto multiply = [&](const double (&kv)[FD][CT], int e) {
#pragma unroll
            for (int u = 0; u < FD; ++u)
#pragma unroll
                for (int row = 0; row < RT; ++row) {
                    const double q = qs[e + u][row];
#pragma unroll
                    for (int c = 0; c < CT; ++c) acc[row][c] = __builtin_fma(q, kv[u][c], acc[row][c]);
                }
        };
        fetch(kva, 0);
        for (int e = 0; e < g.d; e += 2 * FD) {                // d is 64 or 128
            fetch(kvb, e + FD);
            __builtin_amdgcn_sched_barrier(0);
            multiply(kva, e);
            __builtin_amdgcn_sched_barrier(0);
            fetch(kva, e + 2 * FD);
            __builtin_amdgcn_sched_barrier(0);
            multiply(kvb, e + FD);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int row = 0; row < RT; ++row)
#pragma unroll
            for (int c = 0; c < CT; ++c)
                if (j + c < ni_all) prob[row * Tpad + j + c] = __dmul_rn(acc[row][c], g.scale64);
    }
    __syncthreads();

    // from here on wave w works alone on its row
    if (!active) return;
    const int row = w;
    const int ni = allowed_cols(i, g);
    double *pr = prob + row * Tpad;
    const int ni64 = (ni + 63) & ~63;
    double lmax = -INFINITY;
    for (int j = lane; j < ni; j += 64) lmax = fmax(lmax, pr[j]);
    lmax = wave_max(lmax);
    double lsum = 0.0, emin = INFINITY;
    for (int j = lane; j < ni; j += 64) {
        const double ev = exp(pr[j] - lmax);
        pr[j] = ev;
        lsum += ev;
        emin = fmin(emin, ev);
    }
    lsum = wave_sum_dpp(lsum);
    emin = -wave_max(-emin);
    for (int j0 = 0; j0 < ni64; j0 += 64) {
        const int j = j0 + lane;
        pr[j] = j < ni ? pr[j] / lsum : -1.0;                // padding never counts
    }
    const double pmax = 1.0 / lsum, pmin = emin / lsum;      // exp(0) = 1 is the largest numerator

    // vstar: smallest kept probability; above: mass and count of the probabilities > vstar; ties: columns at vstar
    double vstar, above = 0.0;
    int n_above = 0, n_tie;
    int m;                                                   // ties kept, lowest columns first
    if (!(g.tau > 0.0)) {                                    // the first cumulative sum already reaches tau
        vstar = pmax;
        n_tie = mass_at_least(pr, ni64, lane, pmax).cnt;
        m = 1;
    } else {
        const MassCount all = mass_at_least(pr, ni64, lane, pmin);
        if (all.mass < g.tau) {                              // never reached: everything is kept
            vstar = -0.5;
            n_above = ni;
            n_tie = 0;
            m = 0;
        } else {
            // invariant: M(lo) >= tau > M(hi); lo and hi are bit patterns of non-negative doubles
            long long lo = __double_as_longlong(pmin), hi = __double_as_longlong(pmax) + 1;
            int cnt_lo = all.cnt;
            while (hi - lo > 1 && cnt_lo - n_above > 1) {
                const long long mid = lo + ((hi - lo) >> 1);
                const MassCount mc = mass_at_least(pr, ni64, lane, __longlong_as_double(mid));
                if (mc.mass >= g.tau) { lo = mid; cnt_lo = mc.cnt; }
                else { hi = mid; n_above = mc.cnt; above = mc.mass; }
            }
            n_tie = cnt_lo - n_above;
            if (hi - lo > 1) {                               // one element left in [lo, hi): it is vstar
                const double hid = __longlong_as_double(hi);
                double best = -1.0;
                for (int j0 = 0; j0 < ni64; j0 += 64) {
                    const double x = pr[j0 + lane];
                    best = fmax(best, x < hid ? x : -1.0);
                }
                vstar = wave_max(best);
            } else {
                vstar = __longlong_as_double(lo);
            }
            double c = above;
            m = 0;
            do { c += vstar; ++m; } while (c < g.tau && m < n_tie);
        }
    }

    // forced blocks and output: mask words by ballot, ascending column list by prefix popcount
    const int seg = i / g.R;
    const int flo = seg < g.G ? seg * g.R : i;
    const int W = (g.T + 63) >> 6;
    const size_t orow = (size_t)(bhq0 + wh) * g.T + i;
    uint64_t *mrow = mask_bits + orow * W;
    int32_t *crow = col_idx + orow * g.T;
    const uint64_t below = (1ull << lane) - 1ull;
    int base = 0, ties_seen = 0;
    for (int w = 0; w < W; ++w) {
        const int j = w * 64 + lane;
        const double x = j < ni ? pr[j] : -1.0;
        const uint64_t tie_word = __ballot(x == vstar);
        const int tie_rank = ties_seen + __popcll(tie_word & below);
        ties_seen += __popcll(tie_word);
        bool on = false;
        if (j < ni)
            on = x > vstar || (x == vstar && tie_rank < m) || j >= flo ||
                 (j == 0 && (g.flags & PBS_FLAG_FORCE_FIRST_BLOCK));
        const uint64_t word = __ballot(on);
        if (lane == 0) mrow[w] = word;
        if (on) crow[base + __popcll(word & below)] = j;
        base += __popcll(word);
    }
    if (lane == 0) row_cnt[orow] = base;
}

template <int RB, int QB, typename E>
static pbs_status launch_select_qb(const E *Qp, const double *KbarT, uint64_t *mask_bits, int32_t *row_cnt,
                                   int32_t *col_idx, const Geo &g, hipStream_t s)
{
    const int chunks = (g.r + RB - 1) / RB;
    const int Tpad = (g.T + 63) & ~63;
    const int Ts = kbar_stride(g.T);
    const size_t lds = (size_t)RB * QB * Tpad * sizeof(double);
    static std::atomic<unsigned long long> lds_raised{0};
    if (lds > 32 * 1024) {
        const pbs_status st = raise_lds_limit(reinterpret_cast<const void *>(&select_kernel<RB, QB, E>),
                                              QB == 1 ? RB * kMaxT * (int)sizeof(double) : kPairedLds, lds_raised);
        if (st != PBS_OK) return st;
    }
    return launch((select_kernel<RB, QB, E>), dim3((g.T + QB - 1) / QB, g.batch * g.h_kv * chunks), dim3(64 * RB * QB),
                  lds, s, Qp, KbarT, mask_bits, row_cnt, col_idx, g, chunks, Tpad, Ts);
}

// two query blocks per workgroup while their logits fit 64 KiB of LDS (two such workgroups per compute unit)
template <int RB, typename E>
static pbs_status launch_select(const E *Qp, const double *KbarT, uint64_t *mask_bits, int32_t *row_cnt,
                                int32_t *col_idx, const Geo &g, hipStream_t s)
{
    const int Tpad = (g.T + 63) & ~63;
    if ((size_t)RB * 2 * Tpad * sizeof(double) <= (size_t)kPairedLds)
        return launch_select_qb<RB, 2>(Qp, KbarT, mask_bits, row_cnt, col_idx, g, s);
    return launch_select_qb<RB, 1>(Qp, KbarT, mask_bits, row_cnt, col_idx, g, s);
}

// Block means of K' into KbarT ([kv head][feature][kbar_stride(T)] fp64); also called by pbs_segment_permute for the
// shapes its gather kernel does not pool on the way.
pbs_status launch_pool_keys(const pbs_problem *p, const Geo &g, const void *Kp, double *KbarT, hipStream_t s)
{
    const int nk = g.batch * g.h_kv;
    if (p->dtype == PBS_BF16)
        return launch((pool_kernel<bf16_t, true>), dim3(g.T, nk), dim3(256), 0, s, (const bf16_t *)Kp, KbarT, g.n, g.d,
                      g.block, g.T, kbar_stride(g.T));
    return launch((pool_kernel<float, true>), dim3(g.T, nk), dim3(256), 0, s, (const float *)Kp, KbarT, g.n, g.d, g.block,
                  g.T, kbar_stride(g.T));
}

// Block means of the keys K, row-major ([kv head][block][feature] fp64): the centroids of the query permutation.
pbs_status launch_pool_keys_rowmajor(const pbs_problem *p, const Geo &g, const void *K, double *Kbar, hipStream_t s)
{
    const int nk = g.batch * g.h_kv;
    if (p->dtype == PBS_BF16)
        return launch((pool_kernel<bf16_t, false>), dim3(g.T, nk), dim3(256), 0, s, (const bf16_t *)K, Kbar, g.n, g.d,
                      g.block, g.T, g.T);
    return launch((pool_kernel<float, false>), dim3(g.T, nk), dim3(256), 0, s, (const float *)K, Kbar, g.n, g.d, g.block,
                  g.T, g.T);
}

size_t ws_block_mask(const pbs_problem *p)
{
    const Geo g = make_geo(p);
    // pooled K', fp64, feature-major, rows padded to kbar_stride(T) columns
    return align_up((size_t)g.batch * g.h_kv * kbar_stride(g.T) * g.d * sizeof(double), kWsAlign);
}

}  // namespace pbs

using namespace pbs;

extern "C" pbs_status pbs_block_mask(const pbs_problem *p, const void *Qp, const void *Kp, uint64_t *mask_bits,
                                     int32_t *row_cnt, int32_t *col_idx, void *ws, size_t ws_bytes, void *stream)
{
    pbs_status st = validate(p);
    if (st != PBS_OK) return st;
    if (!Qp || !Kp || !mask_bits || !row_cnt || !col_idx) return PBS_ERR_NULL;
    if (!aligned16(Qp) || !aligned16(Kp)) return PBS_ERR_SHAPE;
    if ((st = check_ws(p, PBS_STAGE_BLOCK_MASK, ws, ws_bytes)) != PBS_OK) return st;
    const Geo g = make_geo(p);
    hipStream_t s = (hipStream_t)stream;
    double *KbarT = reinterpret_cast<double *>(ws);
    if (!(p->flags & PBS_FLAG_KBAR_IN_WS) && (st = launch_pool_keys(p, g, Kp, KbarT, s)) != PBS_OK) return st;
    if (p->dtype == PBS_BF16) {
        const bf16_t *Q = (const bf16_t *)Qp;
        if (g.r >= 3) return launch_select<4>(Q, KbarT, mask_bits, row_cnt, col_idx, g, s);
        if (g.r == 2) return launch_select<2>(Q, KbarT, mask_bits, row_cnt, col_idx, g, s);
        return launch_select<1>(Q, KbarT, mask_bits, row_cnt, col_idx, g, s);
    }
    const float *Q = (const float *)Qp;
    if (g.r >= 3) return launch_select<4>(Q, KbarT, mask_bits, row_cnt, col_idx, g, s);
    if (g.r == 2) return launch_select<2>(Q, KbarT, mask_bits, row_cnt, col_idx, g, s);
    return launch_select<1>(Q, KbarT, mask_bits, row_cnt, col_idx, g, s);
}
