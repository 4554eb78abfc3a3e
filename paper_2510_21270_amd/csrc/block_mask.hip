// pbs_block_mask: Algorithm 2 (MeanPooling block selection) on the permuted (Q', K') plus the forced blocks.
//
// Everything that decides the discrete result runs in IEEE fp64 with the plain operation order (no fused
// multiply-add in the logits), so the mask does not depend on how a machine rounds lower precision:
//   1. pool_kernel     block means of Q' and K' (HBM-bound; sums of bf16 values are exact in fp64).
//                      Kbar is stored d-major ([head][e][T]) so that the next kernel reads it coalesced.
//   2. select_kernel   one workgroup per (query head, query block i): logits against the allowed columns,
//                      softmax, stable descending bitonic sort in LDS, inclusive scan, first k with
//                      cumulative mass >= tau, forced blocks, then bit-mask words by wave ballot and the
//                      ascending column list by prefix popcount.
#include "pbs_host.h"

namespace pbs {

// ---------------------------------------------------------------------------------------------
// grid = (T, heads); E = input element type.  TRANSPOSED: write out[head][e][T] instead of out[head][i][e].
// 256 threads: thread (cg = tid % cpr, rg = tid / cpr) sums its 16-byte column group over rows rg, rg+RG, ...
// ---------------------------------------------------------------------------------------------
template <typename E, bool TRANSPOSED>
__global__ __launch_bounds__(256) void pool_kernel(const E *__restrict__ X, double *__restrict__ out, int n, int d,
                                                   int block, int T)
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
    double acc[VEC];
#pragma unroll
    for (int u = 0; u < VEC; ++u) acc[u] = 0.0;
    for (int row = lo + rg; row < hi; row += RG) {
        const vec_t v = *reinterpret_cast<const vec_t *>(X + (head * n + row) * (size_t)d + cg * VEC);
#pragma unroll
        for (int u = 0; u < VEC; ++u) acc[u] += (double)ElemTraits<E>::to_float(v[u]);
    }
#pragma unroll
    for (int u = 0; u < VEC; ++u) red[threadIdx.x * VEC + u] = acc[u];
    __syncthreads();
    if (threadIdx.x < d) {
        const int e = threadIdx.x, c = e / VEC, u = e % VEC;
        double s = 0.0;
        for (int q = 0; q < RG; ++q) s += red[(q * cpr + c) * VEC + u];
        const double mean = s / (double)(hi - lo);
        if (TRANSPOSED) out[(head * d + e) * (size_t)T + i] = mean;
        else out[(head * T + i) * (size_t)d + e] = mean;
    }
}

// ---------------------------------------------------------------------------------------------
// Selection.  LDS holds, for the p2 >= n_i padded columns: the probabilities (sort keys) and their
// column indices.  Comparator: larger probability first, equal probabilities by smaller column.
// ---------------------------------------------------------------------------------------------
__device__ inline bool before(double pa, int ia, double pb, int ib)
{
    return pa > pb || (pa == pb && ia < ib);
}

template <int THREADS>
__device__ inline double block_reduce_max(double v, double *red)
{
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = red[0];
    for (int w = 1; w < THREADS / 64; ++w) r = fmax(r, red[w]);
    return r;
}

template <int THREADS>
__device__ inline double block_reduce_sum(double v, double *red)
{
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    double r = red[0];
    for (int w = 1; w < THREADS / 64; ++w) r += red[w];
    return r;
}

constexpr int kSelThreads = 256;

__global__ __launch_bounds__(kSelThreads) void select_kernel(const double *__restrict__ Qbar,   // [bhq][T][d]
                                                             const double *__restrict__ KbarT,  // [bhkv][d][T]
                                                             uint64_t *__restrict__ mask_bits,
                                                             int32_t *__restrict__ row_cnt,
                                                             int32_t *__restrict__ col_idx, Geo g, int p2max)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    double *prob = reinterpret_cast<double *>(smem_raw);             // [p2max]
    double *csum = prob + p2max;                                     // [p2max] inclusive scan of sorted probs
    int *order = reinterpret_cast<int *>(csum + p2max);              // [p2max]
    unsigned char *sel = reinterpret_cast<unsigned char *>(order + p2max);   // [p2max]
    __shared__ double q[128];
    __shared__ double red[kSelThreads / 64];
    __shared__ double wave_tot[kSelThreads / 64];
    __shared__ int kmin;
    __shared__ int word_cnt[kMaxT / 64];
    __shared__ uint64_t words[kMaxT / 64];

    const int i = blockIdx.x;
    const int bhq = blockIdx.y;
    const int b = bhq / g.h_q, hq = bhq % g.h_q;
    const int bhk = b * g.h_kv + hq / g.r;
    const int ni = allowed_cols(i, g);
    int p2 = 1;
    while (p2 < ni) p2 <<= 1;
    const int tid = threadIdx.x;

    for (int e = tid; e < g.d; e += kSelThreads) q[e] = Qbar[((size_t)bhq * g.T + i) * g.d + e];
    if (tid == 0) kmin = ni;
    __syncthreads();

    // logits, plain multiply-then-add in the order e = 0..d-1
    const double *kt = KbarT + (size_t)bhk * g.d * g.T;
    double lmax = -INFINITY;
    for (int j = tid; j < ni; j += kSelThreads) {
        double acc = 0.0;
        for (int e = 0; e < g.d; ++e) acc = __dadd_rn(acc, __dmul_rn(q[e], kt[(size_t)e * g.T + j]));
        const double v = __dmul_rn(acc, (double)g.scale);
        prob[j] = v;
        lmax = fmax(lmax, v);
    }
    lmax = block_reduce_max<kSelThreads>(lmax, red);
    double lsum = 0.0;
    for (int j = tid; j < ni; j += kSelThreads) {
        const double ev = exp(prob[j] - lmax);
        prob[j] = ev;
        lsum += ev;
    }
    lsum = block_reduce_sum<kSelThreads>(lsum, red);
    for (int j = tid; j < p2; j += kSelThreads) {
        prob[j] = j < ni ? prob[j] / lsum : -1.0;          // padding sorts last
        order[j] = j;
    }
    __syncthreads();

    // bitonic sort, "before" order
    for (int k = 2; k <= p2; k <<= 1) {
        for (int jj = k >> 1; jj > 0; jj >>= 1) {
            for (int t = tid; t < (p2 >> 1); t += kSelThreads) {
                const int lo = t & (jj - 1);
                const int a = ((t - lo) << 1) | lo;
                const int bb = a | jj;
                const bool asc = (a & k) == 0;
                const double pa = prob[a], pb = prob[bb];
                const int ia = order[a], ib = order[bb];
                const bool a_first = before(pa, ia, pb, ib);
                if (a_first != asc) { prob[a] = pb; prob[bb] = pa; order[a] = ib; order[bb] = ia; }
            }
            __syncthreads();
        }
    }

    // inclusive scan of the sorted probabilities: each thread owns a contiguous run
    const int per = (ni + kSelThreads - 1) / kSelThreads;
    const int t0 = min(ni, tid * per), t1 = min(ni, t0 + per);
    double run = 0.0;
    for (int t = t0; t < t1; ++t) run += prob[t];
    // exclusive prefix of the per-thread sums: wave scan + wave totals
    double incl = run;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const double up = __shfl_up(incl, o, 64);
        if ((tid & 63) >= o) incl += up;
    }
    if ((tid & 63) == 63) wave_tot[tid >> 6] = incl;
    __syncthreads();
    double offset = incl - run;
    for (int w = 0; w < (tid >> 6); ++w) offset += wave_tot[w];
    double c = offset;
    int first = ni;                                          // first sorted position whose cumsum reaches tau
    for (int t = t0; t < t1; ++t) {
        c += prob[t];
        csum[t] = c;
        if (c >= g.tau && first == ni) first = t;
    }
    if (first < ni) atomicMin(&kmin, first + 1);
    for (int j = tid; j < p2; j += kSelThreads) sel[j] = 0;
    __syncthreads();
    const int k = kmin;
    for (int t = tid; t < k; t += kSelThreads) sel[order[t]] = 1;
    __syncthreads();

    // forced blocks and output
    const int seg = i / g.R;
    const int flo = seg < g.G ? seg * g.R : i;
    const int W = (g.T + 63) >> 6;
    uint64_t *mrow = mask_bits + ((size_t)bhq * g.T + i) * W;
    const int lane = tid & 63;
    for (int w0 = 0; w0 < W; w0 += kSelThreads / 64) {
        const int w = w0 + (tid >> 6);
        const int j = w * 64 + lane;
        bool on = false;
        if (w < W && j < ni) on = sel[j] || j >= flo || (j == 0 && (g.flags & PBS_FLAG_FORCE_FIRST_BLOCK));
        const uint64_t word = __ballot(on);
        if (w < W && lane == 0) { mrow[w] = word; words[w] = word; word_cnt[w] = __popcll(word); }
    }
    __syncthreads();
    int32_t *crow = col_idx + ((size_t)bhq * g.T + i) * g.T;
    for (int w0 = 0; w0 < W; w0 += kSelThreads / 64) {
        const int w = w0 + (tid >> 6);
        if (w >= W) continue;
        int basec = 0;
        for (int x = 0; x < w; ++x) basec += word_cnt[x];
        const uint64_t word = words[w];
        if ((word >> lane) & 1ull) crow[basec + __popcll(word & ((1ull << lane) - 1ull))] = w * 64 + lane;
    }
    if (tid == 0) {
        int total = 0;
        for (int x = 0; x < W; ++x) total += word_cnt[x];
        row_cnt[(size_t)bhq * g.T + i] = total;
    }
}

size_t ws_block_mask(const pbs_problem *p)
{
    const Geo g = make_geo(p);
    return align_up((size_t)g.batch * g.h_q * g.T * g.d * sizeof(double), kWsAlign) +
           align_up((size_t)g.batch * g.h_kv * g.T * g.d * sizeof(double), kWsAlign);
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
    double *Qbar = reinterpret_cast<double *>(ws);
    double *KbarT = reinterpret_cast<double *>(reinterpret_cast<char *>(ws) +
                                               align_up((size_t)g.batch * g.h_q * g.T * g.d * sizeof(double), kWsAlign));
    const int nq = g.batch * g.h_q, nk = g.batch * g.h_kv;
    if (p->dtype == PBS_BF16) {
        hipLaunchKernelGGL((pool_kernel<bf16_t, false>), dim3(g.T, nq), dim3(256), 0, s, (const bf16_t *)Qp, Qbar, g.n,
                           g.d, g.block, g.T);
        hipLaunchKernelGGL((pool_kernel<bf16_t, true>), dim3(g.T, nk), dim3(256), 0, s, (const bf16_t *)Kp, KbarT, g.n,
                           g.d, g.block, g.T);
    } else {
        hipLaunchKernelGGL((pool_kernel<float, false>), dim3(g.T, nq), dim3(256), 0, s, (const float *)Qp, Qbar, g.n,
                           g.d, g.block, g.T);
        hipLaunchKernelGGL((pool_kernel<float, true>), dim3(g.T, nk), dim3(256), 0, s, (const float *)Kp, KbarT, g.n,
                           g.d, g.block, g.T);
    }
    if ((st = launch_status()) != PBS_OK) return st;
    int p2max = 1;
    while (p2max < g.T) p2max <<= 1;
    const size_t lds = (size_t)p2max * (8 + 8 + 4 + 1);
    if (lds > 48 * 1024) {
        static bool attr_set = false;
        if (!attr_set) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(&select_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kMaxT * 21) != hipSuccess)
                return PBS_ERR_HIP;
            attr_set = true;
        }
    }
    hipLaunchKernelGGL(select_kernel, dim3(g.T, nq), dim3(kSelThreads), lds, s, Qbar, KbarT, mask_bits, row_cnt,
                       col_idx, g, p2max);
    return launch_status();
}
