// pbs_key_scores: Eq. 4 with group-averaged queries (appendix "GQA Handling").
//
//   scores[j] = (1/B') * sum_r softmax_j( Qhat[r] . K[j] * scale ),   r over the last B' = min(block, n) rows
//
// The row softmax needs the global maximum and normaliser of each of the B' rows over all n keys, so K is
// swept twice: sweep 1 produces per-row (max, sum-exp) partials, a tiny kernel merges them into one
// constant c[r] = -max_r - log2(B' * sumexp_r) (log2 domain), and sweep 2 evaluates
// scores[j] = sum_r exp2(logit2[r][j] + c[r]).  Sweep 2 walks the key tiles in reverse so that it starts
// on what sweep 1 left in the last-level cache.
//
// bf16, d = 128: both sweeps form the 128 x keys logit tile on the matrix cores (32x32x16 bf16 MFMA, fp32
// accumulator).  Qhat is an fp32 mean, not a bf16 value, so it is pre-multiplied by scale*log2(e) and split
// into two bf16 terms hi + lo; each tile takes two MFMAs per fragment.  K fragments come straight from
// global memory: the contraction index may be permuted freely, so lane half h contracts d in [64h, 64h+64)
// and every lane reads one contiguous 128-byte half row.
// Everything else (fp32 inputs, d = 64): fp64 vector arithmetic, one thread per key.
#include "pbs_host.h"

namespace pbs {

constexpr int kQRows = 128;            // logit tile rows (>= B')
constexpr int kMaxKeysPerWg = 1024;    // keys per workgroup in the MFMA sweeps when there are enough keys
constexpr int kMinKeysPerWg = 128;     // one 32-key tile per wave
constexpr int kSweepWgs = 512;         // the sweeps shorten their key ranges until this many workgroups exist
                                       // (every workgroup first copies the 64 KiB split Qhat: more of them costs again)
constexpr float kLog2e = 1.4426950408889634f;

// ------------------------------------------------------------------ MFMA path: prep
// qsplit[bh][term][row][dswz]: row-major 128 x 128 bf16, 16-byte chunks XOR-swizzled by (row & 15) so that a
// flat copy into LDS is bank-conflict free for the fragment reads.  Rows >= bl are zero.
__global__ __launch_bounds__(256) void qhat_split_kernel(const bf16_t *__restrict__ Q, bf16_t *__restrict__ qsplit,
                                                         Geo g, int bl)
{
    // grid = (kQRows / 8, batch * h_kv): each workgroup converts 8 rows x 128 columns, 4 elements per thread
    const int bh = blockIdx.y;
    const int b = bh / g.h_kv, h = bh % g.h_kv;
    bf16_t *hi = qsplit + (size_t)bh * 2 * kQRows * 128;
    bf16_t *lo = hi + kQRows * 128;
    const float mul = g.scale * kLog2e / (float)g.r;
    const int row = blockIdx.x * 8 + (threadIdx.x >> 5);
    const int e0 = (threadIdx.x & 31) * 4;
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (row < bl)
        for (int t = 0; t < g.r; ++t) {
            const bf16x4 v = *reinterpret_cast<const bf16x4 *>(
                Q + (((size_t)b * g.h_q + h * g.r + t) * g.n + (g.n - bl + row)) * 128 + e0);
#pragma unroll
            for (int x = 0; x < 4; ++x) acc[x] += (float)v[x];
        }
    bf16x4 vh, vl;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const float v = acc[x] * mul;
        vh[x] = (bf16_t)v;
        vl[x] = (bf16_t)(v - (float)vh[x]);
    }
    const int chunk = (e0 >> 3) ^ (row & 15);
    const int dst = row * 128 + chunk * 8 + (e0 & 7);
    *reinterpret_cast<bf16x4 *>(hi + dst) = vh;
    *reinterpret_cast<bf16x4 *>(lo + dst) = vl;
}

// Fragment of the split Qhat held in LDS: rows 32*tile + (lane & 31), contraction chunk for k-step ks.
__device__ inline bf16x8 qfrag(const bf16_t *lds, int tile, int ks, int lane)
{
    const int row = tile * 32 + (lane & 31);
    const int chunk = ((lane >> 5) * 8 + ks) ^ (row & 15);   // d = 64*h + 8*ks .. +8  -> chunk 8*h + ks
    return *reinterpret_cast<const bf16x8 *>(lds + row * 128 + chunk * 8);
}

// K fragments of 32 keys starting at key0: lane (key = lane & 31, h = lane >> 5) reads d in [64h, 64h+64).
__device__ inline void load_kfrags(bf16x8 (&kf)[8], const bf16_t *Kh, int key0, int n, int lane)
{
    int key = key0 + (lane & 31);
    if (key >= n) key = n - 1;                                // clamped; masked by the caller
    const bf16x8 *src = reinterpret_cast<const bf16x8 *>(Kh + (size_t)key * 128 + (lane >> 5) * 64);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kf[ks] = src[ks];
}

// ------------------------------------------------------------------ MFMA path: sweep 1
// partial[bh][wg][row] = (max2, sumexp2) over the keys of workgroup wg, log2 domain.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void scores_sweep1_kernel(
    const bf16_t *__restrict__ K,
                                                            const bf16_t *__restrict__ qsplit,
                                                            float2 *__restrict__ partial, Geo g, int kpw)
{
    __shared__ __align__(16) bf16_t qs[2 * kQRows * 128];   // 64 KiB
    __shared__ float2 red[4][kQRows];
    const int bh = blockIdx.y, wg = blockIdx.x, nwg = gridDim.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    {
        const uintx4 *src = reinterpret_cast<const uintx4 *>(qsplit + (size_t)bh * 2 * kQRows * 128);
        uintx4 *dst = reinterpret_cast<uintx4 *>(qs);
        for (int c = threadIdx.x; c < 2 * kQRows * 128 / 8; c += blockDim.x) dst[c] = src[c];
    }
    __syncthreads();
    const bf16_t *Kh = K + (size_t)bh * g.n * 128;
    float m[4], l[4];
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) { m[nt] = -INFINITY; l[nt] = 0.0f; }
    const int key_end = min(g.n, (wg + 1) * kpw);
    bf16x8 kf[8], kn[8];                                     // current fragments and the prefetched next tile
    load_kfrags(kf, Kh, min(wg * kpw + wave * 32, g.n - 1), g.n, lane);
    for (int key0 = wg * kpw + wave * 32; key0 < key_end; key0 += 4 * 32) {
        load_kfrags(kn, Kh, key0 + 4 * 32 < key_end ? key0 + 4 * 32 : key0, g.n, lane);   // last tile: a cached re-read
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            asm volatile("" ::: "memory");                   // keeps the Qhat fragment reads inside the loop
            floatx16 acc = {0};
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qfrag(qs, nt, ks, lane), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qfrag(qs + kQRows * 128, nt, ks, lane), acc, 0,
                                                              0, 0);
            }
            // acc[i]: key = key0 + 8*(i/4) + 4*(lane>>5) + (i%4), query row = 32*nt + (lane & 31)
            float tmax = -INFINITY;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int key = key0 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
                if (key >= g.n) acc[i] = -INFINITY;
                tmax = fmaxf(tmax, acc[i]);
            }
            const float mn = fmaxf(m[nt], tmax);
            if (mn != -INFINITY) {
                float sum = 0.0f;
#pragma unroll
                for (int i = 0; i < 16; ++i) sum += exp2f(acc[i] - mn);
                l[nt] = l[nt] * exp2f(m[nt] - mn) + sum;     // exp2f(-inf) = 0 on the first tile
                m[nt] = mn;
            }
        }
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) kf[ks] = kn[ks];
    }
    // merge the two lane halves, then the four waves
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
        const float mo = __shfl_xor(m[nt], 32, 64), lo = __shfl_xor(l[nt], 32, 64);
        const float mn = fmaxf(m[nt], mo);
        float ln = 0.0f;
        if (mn != -INFINITY) ln = l[nt] * exp2f(m[nt] - mn) + lo * exp2f(mo - mn);
        if (lane < 32) red[wave][nt * 32 + lane] = make_float2(mn, ln);
    }
    __syncthreads();
    if (threadIdx.x < kQRows) {
        float mn = -INFINITY;
        for (int w = 0; w < 4; ++w) mn = fmaxf(mn, red[w][threadIdx.x].x);
        float ln = 0.0f;
        if (mn != -INFINITY)
            for (int w = 0; w < 4; ++w) ln += red[w][threadIdx.x].y * exp2f(red[w][threadIdx.x].x - mn);
        partial[((size_t)bh * nwg + wg) * kQRows + threadIdx.x] = make_float2(mn, ln);
    }
}

// c[bh][row] = -max - log2(bl * sumexp) for row < bl, -inf for the padding rows.
// 1024 threads: thread (grp, row) folds the partials grp, grp+8, ... of its row, then the 8 groups meet in LDS.
__global__ __launch_bounds__(1024) void scores_merge_kernel(const float2 *__restrict__ partial,
                                                            float *__restrict__ cvec, int nwg, int bl)
{
    __shared__ float2 red[8][kQRows];
    const int bh = blockIdx.x, row = threadIdx.x & (kQRows - 1), grp = threadIdx.x >> 7;
    float mn = -INFINITY, ln = 0.0f;
    for (int w = grp; w < nwg; w += 8) {
        const float2 pr = partial[((size_t)bh * nwg + w) * kQRows + row];
        if (pr.x != -INFINITY) {
            const float m2 = fmaxf(mn, pr.x);
            ln = ln * exp2f(mn - m2) + pr.y * exp2f(pr.x - m2);
            mn = m2;
        }
    }
    red[grp][row] = make_float2(mn, ln);
    __syncthreads();
    if (grp == 0) {
        float m2 = -INFINITY;
        for (int q = 0; q < 8; ++q) m2 = fmaxf(m2, red[q][row].x);
        float l2 = 0.0f;
        for (int q = 0; q < 8; ++q)
            if (red[q][row].x != -INFINITY) l2 += red[q][row].y * exp2f(red[q][row].x - m2);
        cvec[(size_t)bh * kQRows + row] = row < bl ? -m2 - log2f((float)bl * l2) : -INFINITY;
    }
}

// ------------------------------------------------------------------ MFMA path: sweep 2
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void scores_sweep2_kernel(
    const bf16_t *__restrict__ K,
                                                            const bf16_t *__restrict__ qsplit,
                                                            const float *__restrict__ cvec,
                                                            float *__restrict__ scores, Geo g, int kpw)
{
    __shared__ __align__(16) bf16_t qs[2 * kQRows * 128];
    const int bh = blockIdx.y;
    const int wg = gridDim.x - 1 - blockIdx.x;               // reverse order: reuse what sweep 1 left in cache
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    {
        const uintx4 *src = reinterpret_cast<const uintx4 *>(qsplit + (size_t)bh * 2 * kQRows * 128);
        uintx4 *dst = reinterpret_cast<uintx4 *>(qs);
        for (int c = threadIdx.x; c < 2 * kQRows * 128 / 8; c += blockDim.x) dst[c] = src[c];
    }
    // the accumulator starts at c[row]; row = 32*mt + 8*(i/4) + 4*(lane>>5) + (i%4)
    floatx16 cinit[4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i)
            cinit[mt][i] = cvec[(size_t)bh * kQRows + 32 * mt + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3)];
    __syncthreads();
    const bf16_t *Kh = K + (size_t)bh * g.n * 128;
    const int key_end = min(g.n, (wg + 1) * kpw);
    bf16x8 kf[8], kn[8];
    load_kfrags(kf, Kh, min(wg * kpw + wave * 32, g.n - 1), g.n, lane);
    for (int key0 = wg * kpw + wave * 32; key0 < key_end; key0 += 4 * 32) {
        load_kfrags(kn, Kh, key0 + 4 * 32 < key_end ? key0 + 4 * 32 : key0, g.n, lane);   // last tile: a cached re-read
        float sum = 0.0f;
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
            asm volatile("" ::: "memory");                   // keeps the Qhat fragment reads inside the loop
            floatx16 acc = cinit[mt];
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qfrag(qs, mt, ks, lane), kf[ks], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qfrag(qs + kQRows * 128, mt, ks, lane), kf[ks], acc, 0,
                                                              0, 0);
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) sum += exp2f(acc[i]);
        }
        sum += __shfl_xor(sum, 32, 64);
        const int key = key0 + (lane & 31);
        if (lane < 32 && key < g.n) scores[(size_t)bh * g.n + key] = sum;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) kf[ks] = kn[ks];
    }
}

// ------------------------------------------------------------------ generic path (fp64 accumulation)
template <typename E>
__global__ __launch_bounds__(256) void qhat_f64_kernel(const E *__restrict__ Q, double *__restrict__ qhat, Geo g,
                                                       int bl)
{
    const int bh = blockIdx.x;
    const int b = bh / g.h_kv, h = bh % g.h_kv;
    for (int idx = threadIdx.x; idx < bl * g.d; idx += blockDim.x) {
        const int row = idx / g.d, e = idx % g.d;
        double acc = 0.0;
        for (int t = 0; t < g.r; ++t)
            acc += (double)ElemTraits<E>::to_float(
                Q[(((size_t)b * g.h_q + h * g.r + t) * g.n + (g.n - bl + row)) * g.d + e]);
        qhat[(size_t)bh * bl * g.d + idx] = acc / (double)g.r;
    }
}

template <typename E>
__device__ inline double dot_f64(const double *__restrict__ q, const E *__restrict__ k, int d)
{
    double acc = 0.0;
    for (int e = 0; e < d; ++e) acc += q[e] * (double)ElemTraits<E>::to_float(k[e]);
    return acc;
}

// grid = (chunks, bl, nbh): partial (max, sumexp) of one logit row over one chunk of keys.
template <typename E>
__global__ __launch_bounds__(256) void scores_stats_f64_kernel(const E *__restrict__ K,
                                                               const double *__restrict__ qhat,
                                                               double2 *__restrict__ partial, Geo g, int bl,
                                                               int keys_per_chunk)
{
    __shared__ double q[128];
    __shared__ double redm[4], redl[4];
    const int chunk = blockIdx.x, row = blockIdx.y, bh = blockIdx.z;
    for (int e = threadIdx.x; e < g.d; e += blockDim.x) q[e] = qhat[((size_t)bh * bl + row) * g.d + e];
    __syncthreads();
    const E *Kh = K + (size_t)bh * g.n * g.d;
    const int j1 = min(g.n, (chunk + 1) * keys_per_chunk);
    double m = -INFINITY, l = 0.0;
    for (int j = chunk * keys_per_chunk + threadIdx.x; j < j1; j += blockDim.x) {
        const double v = dot_f64(q, Kh + (size_t)j * g.d, g.d) * (double)g.scale;
        const double mn = fmax(m, v);
        l = l * exp(m - mn) + exp(v - mn);
        m = mn;
    }
    const double wm = wave_max(m);
    const double wl = wave_sum(wm == -INFINITY ? 0.0 : l * exp(m - wm));
    if ((threadIdx.x & 63) == 0) { redm[threadIdx.x >> 6] = wm; redl[threadIdx.x >> 6] = wl; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double mn = fmax(fmax(redm[0], redm[1]), fmax(redm[2], redm[3]));
        double ln = 0.0;
        for (int w = 0; w < 4; ++w)
            if (redm[w] != -INFINITY) ln += redl[w] * exp(redm[w] - mn);
        partial[((size_t)bh * bl + row) * gridDim.x + chunk] = make_double2(mn, ln);
    }
}

__global__ __launch_bounds__(128) void scores_merge_f64_kernel(const double2 *__restrict__ partial,
                                                               double2 *__restrict__ stats, int bl, int chunks)
{
    const int row = threadIdx.x, bh = blockIdx.x;
    if (row >= bl) return;
    const double2 *pr = partial + ((size_t)bh * bl + row) * chunks;
    double mn = -INFINITY;
    for (int c = 0; c < chunks; ++c) mn = fmax(mn, pr[c].x);
    double ln = 0.0;
    for (int c = 0; c < chunks; ++c)
        if (pr[c].x != -INFINITY) ln += pr[c].y * exp(pr[c].x - mn);
    stats[(size_t)bh * bl + row] = make_double2(mn, ln);
}

// one thread per key: scores[j] = (1/bl) * sum_row exp(logit - max_row) / sumexp_row
template <typename E>
__global__ __launch_bounds__(256) void scores_final_f64_kernel(const E *__restrict__ K,
                                                               const double *__restrict__ qhat,
                                                               const double2 *__restrict__ stats,
                                                               float *__restrict__ scores, Geo g, int bl)
{
    constexpr int kRowsPerPass = 8;
    __shared__ double q[kRowsPerPass][128];
    __shared__ double2 st[kRowsPerPass];
    const int bh = blockIdx.y;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    const E *krow = K + ((size_t)bh * g.n + (j < g.n ? j : g.n - 1)) * g.d;
    double acc = 0.0;
    for (int r0 = 0; r0 < bl; r0 += kRowsPerPass) {
        const int nr = min(kRowsPerPass, bl - r0);
        __syncthreads();
        for (int idx = threadIdx.x; idx < nr * g.d; idx += blockDim.x)
            q[idx / g.d][idx % g.d] = qhat[((size_t)bh * bl + r0 + idx / g.d) * g.d + idx % g.d];
        if (threadIdx.x < nr) st[threadIdx.x] = stats[(size_t)bh * bl + r0 + threadIdx.x];
        __syncthreads();
        for (int rr = 0; rr < nr; ++rr) {
            const double v = dot_f64(q[rr], krow, g.d) * (double)g.scale;
            acc += exp(v - st[rr].x) / st[rr].y;
        }
    }
    if (j < g.n) scores[(size_t)bh * g.n + j] = (float)(acc / (double)bl);
}

static bool use_mfma(const pbs_problem *p) { return p->dtype == PBS_BF16 && p->d == 128; }

constexpr int kGenericKeysPerChunk = 4096;

// Keys per workgroup of the MFMA sweeps: 1024 for long inputs; halved (down to one tile per wave) while the
// grid would hold fewer than kSweepWgs workgroups, so that short inputs still spread over all compute units.
static int sweep_keys_per_wg(const Geo &g)
{
    int kpw = kMaxKeysPerWg;
    while (kpw > kMinKeysPerWg && (long long)ceil_div(g.n, kpw) * g.batch * g.h_kv < kSweepWgs) kpw >>= 1;
    return kpw;
}

size_t ws_key_scores(const pbs_problem *p)
{
    const Geo g = make_geo(p);
    const size_t nbh = (size_t)g.batch * g.h_kv;
    const int bl = g.block < g.n ? g.block : g.n;
    if (use_mfma(p)) {
        const size_t nwg = ceil_div(g.n, sweep_keys_per_wg(g));
        return align_up(nbh * 2 * kQRows * 128 * sizeof(bf16_t), kWsAlign) +
               align_up(nbh * nwg * kQRows * sizeof(float2), kWsAlign) + align_up(nbh * kQRows * sizeof(float), kWsAlign);
    }
    const size_t chunks = ceil_div(g.n, kGenericKeysPerChunk);
    return align_up(nbh * bl * g.d * sizeof(double), kWsAlign) + align_up(nbh * bl * chunks * sizeof(double2), kWsAlign) +
           align_up(nbh * bl * sizeof(double2), kWsAlign);
}

template <typename E>
static pbs_status run_generic(const pbs_problem *p, const Geo &g, const void *Q, const void *K, float *scores,
                              char *ws, hipStream_t s)
{
    const int nbh = g.batch * g.h_kv;
    const int bl = g.block < g.n ? g.block : g.n;
    const int chunks = ceil_div(g.n, kGenericKeysPerChunk);
    double *qhat = reinterpret_cast<double *>(ws);
    ws += align_up((size_t)nbh * bl * g.d * sizeof(double), kWsAlign);
    double2 *partial = reinterpret_cast<double2 *>(ws);
    ws += align_up((size_t)nbh * bl * chunks * sizeof(double2), kWsAlign);
    double2 *stats = reinterpret_cast<double2 *>(ws);
    pbs_status st;
    hipLaunchKernelGGL(qhat_f64_kernel<E>, dim3(nbh), dim3(256), 0, s, (const E *)Q, qhat, g, bl);
    if ((st = launch_status()) != PBS_OK) return st;
    hipLaunchKernelGGL(scores_stats_f64_kernel<E>, dim3(chunks, bl, nbh), dim3(256), 0, s, (const E *)K, qhat, partial,
                       g, bl, kGenericKeysPerChunk);
    if ((st = launch_status()) != PBS_OK) return st;
    hipLaunchKernelGGL(scores_merge_f64_kernel, dim3(nbh), dim3(128), 0, s, partial, stats, bl, chunks);
    if ((st = launch_status()) != PBS_OK) return st;
    hipLaunchKernelGGL(scores_final_f64_kernel<E>, dim3(ceil_div(g.n, 256), nbh), dim3(256), 0, s, (const E *)K, qhat,
                       stats, scores, g, bl);
    (void)p;
    return launch_status();
}

}  // namespace pbs

using namespace pbs;

extern "C" pbs_status pbs_key_scores(const pbs_problem *p, const void *Q, const void *K, float *scores, void *ws,
                                     size_t ws_bytes, void *stream)
{
    pbs_status st = validate(p);
    if (st != PBS_OK) return st;
    if (!Q || !K || !scores) return PBS_ERR_NULL;
    if (!aligned16(Q) || !aligned16(K)) return PBS_ERR_SHAPE;
    if ((st = check_ws(p, PBS_STAGE_KEY_SCORES, ws, ws_bytes)) != PBS_OK) return st;
    const Geo g = make_geo(p);
    hipStream_t s = (hipStream_t)stream;
    char *w = reinterpret_cast<char *>(ws);
    if (!use_mfma(p)) {
        if (p->dtype == PBS_BF16) return run_generic<bf16_t>(p, g, Q, K, scores, w, s);
        return run_generic<float>(p, g, Q, K, scores, w, s);
    }
    const int nbh = g.batch * g.h_kv;
    const int bl = g.block < g.n ? g.block : g.n;
    const int kpw = sweep_keys_per_wg(g);
    const int nwg = ceil_div(g.n, kpw);
    bf16_t *qsplit = reinterpret_cast<bf16_t *>(w);
    w += align_up((size_t)nbh * 2 * kQRows * 128 * sizeof(bf16_t), kWsAlign);
    float2 *partial = reinterpret_cast<float2 *>(w);
    w += align_up((size_t)nbh * nwg * kQRows * sizeof(float2), kWsAlign);
    float *cvec = reinterpret_cast<float *>(w);
    hipLaunchKernelGGL(qhat_split_kernel, dim3(kQRows / 8, nbh), dim3(256), 0, s, (const bf16_t *)Q, qsplit, g, bl);
    if ((st = launch_status()) != PBS_OK) return st;
    hipLaunchKernelGGL(scores_sweep1_kernel, dim3(nwg, nbh), dim3(256), 0, s, (const bf16_t *)K, qsplit, partial, g, kpw);
    if ((st = launch_status()) != PBS_OK) return st;
    hipLaunchKernelGGL(scores_merge_kernel, dim3(nbh), dim3(1024), 0, s, partial, cvec, nwg, bl);
    if ((st = launch_status()) != PBS_OK) return st;
    hipLaunchKernelGGL(scores_sweep2_kernel, dim3(nwg, nbh), dim3(256), 0, s, (const bf16_t *)K, qsplit, cvec, scores,
                       g, kpw);
    return launch_status();
}
