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
// into two bf16 terms hi + lo; each tile takes two MFMAs per fragment.  A wave keeps the fragments of its 32 rows
// of Qhat in registers and the K tiles go through LDS, shared by the four waves of a workgroup.
// Everything else (fp32 inputs, d = 64): fp64 vector arithmetic, one thread per key.
#include "pbs_host.h"

namespace pbs {

constexpr int kQRows = 128;            // logit tile rows (>= B')
constexpr int kMaxKeysPerWg = 1024;    // keys per workgroup in the MFMA sweeps when there are enough keys
constexpr int kMinKeysPerWg = 256;     // shorter ranges do not pay for a workgroup's start (Qhat fragments, first tiles)
constexpr int kSweepWgs = 512;         // the sweeps shorten their key ranges until this many workgroups exist
                                       // (every workgroup first copies the 64 KiB split Qhat: more of them costs again)
constexpr float kLog2e = 1.4426950408889634f;

// ------------------------------------------------------------------ MFMA path: prep
// qsplit[bh][term][row][dswz]: row-major 128 x 128 bf16, 16-byte chunks XOR-permuted by (row & 15) (the lanes of a
// fragment load then spread over the 16 chunk positions of their rows).  Rows >= bl are zero.
// qrows: positions of the bl query rows (device memory), or NULL for the last bl rows of the sequence (Eq. 4);
// positions outside [0, n) are clamped.  qavg != NULL instead: one query row, the fp64 mean over all positions.
__device__ inline int query_row_position(const int32_t *qrows, int row, int bl, int n)
{
    if (!qrows) return n - bl + row;
    const int pos = qrows[row];
    return pos < 0 ? 0 : (pos >= n ? n - 1 : pos);
}

__global__ __launch_bounds__(256) void qhat_split_kernel(const bf16_t *__restrict__ Q, bf16_t *__restrict__ qsplit,
                                                         Geo g, int bl, const int32_t *__restrict__ qrows,
                                                         const double *__restrict__ qavg)
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
    float mul_row = mul;
    if (row < bl) {
        if (qavg) {                                           // already the mean over heads and positions
#pragma unroll
            for (int x = 0; x < 4; ++x) acc[x] = (float)qavg[(size_t)bh * 128 + e0 + x];
            mul_row = g.scale * kLog2e;
        } else {
            const int pos = query_row_position(qrows, row, bl, g.n);
            for (int t = 0; t < g.r; ++t) {
                const bf16x4 v = *reinterpret_cast<const bf16x4 *>(
                    Q + (((size_t)b * g.h_q + h * g.r + t) * g.n + pos) * 128 + e0);
#pragma unroll
                for (int x = 0; x < 4; ++x) acc[x] += (float)v[x];
            }
        }
    }
    bf16x4 vh, vl;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const float v = acc[x] * mul_row;
        vh[x] = (bf16_t)v;
        vl[x] = (bf16_t)(v - (float)vh[x]);
    }
    const int chunk = (e0 >> 3) ^ (row & 15);
    const int dst = row * 128 + chunk * 8 + (e0 & 7);
    *reinterpret_cast<bf16x4 *>(hi + dst) = vh;
    *reinterpret_cast<bf16x4 *>(lo + dst) = vl;
}

// ------------------------------------------------------------------ MFMA path: tiles and fragments
// Wave w of a workgroup owns the logit rows 32 w .. 32 w + 31 and keeps their split Qhat fragments in registers
// (8 k-steps x 2 terms x 4 registers); the K tiles of 32 keys go through LDS, where all four waves read them, so a
// fragment read feeds two MFMAs and the tile is fetched from memory once.  A tile travels global -> registers ->
// LDS; kTilesAhead tiles per workgroup are in flight in registers, and two LDS copies alternate so that one
// barrier per tile suffices.
constexpr int kTileKeys = 32;
constexpr int kTilesAhead = 2;

// 32 keys x 256 bytes; the 16-byte piece c of row r sits at r * 256 + ((c ^ (r & 15)) << 4): conflict-free for the
// stores (16 lanes = the 16 pieces of a row) and for the fragment reads (16 lanes = 16 rows, one piece each).
struct KTile {
    unsigned char b[kTileKeys * 256];
};

// Thread tid moves pieces tid and tid + 256 of the 512 pieces of a tile (row = piece / 16, c = piece % 16).
__device__ inline void ktile_fetch(uintx4 (&v)[2], const bf16_t *Kh, int key0, int n, int tid)
{
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int piece = tid + 256 * u;
        int key = key0 + (piece >> 4);
        if (key >= n) key = n - 1;                            // clamped; masked by the caller
        v[u] = *reinterpret_cast<const uintx4 *>(Kh + (size_t)key * 128 + (piece & 15) * 8);
    }
}

__device__ inline void ktile_store(KTile &t, const uintx4 (&v)[2], int tid)
{
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int piece = tid + 256 * u;
        const int row = piece >> 4, c = piece & 15;
        *reinterpret_cast<uintx4 *>(t.b + row * 256 + ((c ^ (row & 15)) << 4)) = v[u];
    }
}

// MFMA operand of k-step ks: lane (key = lane & 31, h = lane >> 5) holds d = 16 ks + 8 h .. + 8 of its key.
__device__ inline bf16x8 kfrag(const KTile &t, int ks, int lane)
{
    const int row = lane & 31, c = 2 * ks + (lane >> 5);
    return *reinterpret_cast<const bf16x8 *>(t.b + row * 256 + ((c ^ (row & 15)) << 4));
}

// The wave's 32 rows of one term of the split Qhat, straight from qsplit (same d range per lane as kfrag).
__device__ inline void load_qfrags(bf16x8 (&qf)[8], const bf16_t *term, int wave, int lane)
{
    const int row = wave * 32 + (lane & 31);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const int c = 2 * ks + (lane >> 5);
        qf[ks] = *reinterpret_cast<const bf16x8 *>(term + row * 128 + ((c ^ (row & 15)) << 3));
    }
}

// Runs body(t, tile) for the tiles t = 0 .. ntiles - 1 of the keys from key_begin on, the tile being complete in
// LDS.  The loops over the tiles in flight are fully unrolled, so their register copies have compile-time indices.
template <typename Body>
__device__ __forceinline__ void sweep_tiles(KTile (&kt)[2], const bf16_t *Kh, int key_begin, int ntiles, int n, int tid,
                                            Body body)
{
    uintx4 pre[kTilesAhead][2];
#pragma unroll
    for (int a = 0; a < kTilesAhead; ++a) ktile_fetch(pre[a], Kh, min(key_begin + a * kTileKeys, n - 1), n, tid);
    ktile_store(kt[0], pre[0], tid);
    ktile_fetch(pre[0], Kh, min(key_begin + kTilesAhead * kTileKeys, n - 1), n, tid);
    __syncthreads();
    for (int t0 = 0; t0 < ntiles; t0 += kTilesAhead) {
#pragma unroll
        for (int a = 0; a < kTilesAhead; ++a) {
            const int t = t0 + a;
            if (t < ntiles) {                                  // uniform
                // tile t + 1 leaves its registers for the LDS copy that tile t - 1 used, and its registers take
                // tile t + 1 + kTilesAhead (reads past the range are clamped to the last key and never used)
                ktile_store(kt[(a + 1) & 1], pre[(a + 1) % kTilesAhead], tid);
                ktile_fetch(pre[(a + 1) % kTilesAhead], Kh, min(key_begin + (t + 1 + kTilesAhead) * kTileKeys, n - 1),
                            n, tid);
                body(t, kt[a & 1]);
                __syncthreads();                               // tile t consumed, tile t + 1 visible
            }
        }
    }
}

// ------------------------------------------------------------------ MFMA path: sweep 1
// partial[bh][wg][row] = (max2, sumexp2) over the keys of workgroup wg, log2 domain.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void scores_sweep1_kernel(
    const bf16_t *__restrict__ K, const bf16_t *__restrict__ qsplit, float2 *__restrict__ partial, Geo g, int kpw)
{
    __shared__ __align__(16) KTile kt[2];
    const int bh = blockIdx.y, wg = blockIdx.x, nwg = gridDim.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    bf16x8 qh[8], ql[8];
    load_qfrags(qh, qsplit + (size_t)bh * 2 * kQRows * 128, wave, lane);
    load_qfrags(ql, qsplit + (size_t)bh * 2 * kQRows * 128 + kQRows * 128, wave, lane);
    const bf16_t *Kh = K + (size_t)bh * g.n * 128;
    const int key_begin = wg * kpw, key_end = min(g.n, key_begin + kpw);
    const int ntiles = ceil_div(key_end - key_begin, kTileKeys);
    float m = -INFINITY, l = 0.0f;                           // row 32 wave + (lane & 31), this lane's half of the keys
    sweep_tiles(kt, Kh, key_begin, ntiles, g.n, tid, [&](int t, const KTile &tile) {
        floatx16 acc = {0};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 kf = kfrag(tile, ks, lane);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qh[ks], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, ql[ks], acc, 0, 0, 0);
        }
        // acc[i]: key = key0 + 8 (i / 4) + 4 (lane >> 5) + (i % 4), query row = 32 wave + (lane & 31)
        const int key0 = key_begin + t * kTileKeys;
        if (key0 + kTileKeys > g.n) {                          // the ragged last tile of the sequence
#pragma unroll
            for (int i = 0; i < 16; ++i)
                if (key0 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3) >= g.n) acc[i] = -INFINITY;
        }
        float tmax = acc[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, acc[i]);
        const float mn = fmaxf(m, tmax);
        if (mn != -INFINITY) {
            // arguments are <= 0: the bare instruction (no denormal rescue) loses nothing that a sum near 1 would see
            float sum = 0.0f;
#pragma unroll
            for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(acc[i] - mn);
            l = l * __builtin_amdgcn_exp2f(m - mn) + sum;    // exp2(-inf) = 0 on the first tile
            m = mn;
        }
    });
    // merge the two lane halves; the rows of a wave are its own
    const float mo = __shfl_xor(m, 32, 64), lo = __shfl_xor(l, 32, 64);
    const float mn = fmaxf(m, mo);
    float ln = 0.0f;
    if (mn != -INFINITY) ln = l * exp2f(m - mn) + lo * exp2f(mo - mn);
    if (lane < 32) partial[((size_t)bh * nwg + wg) * kQRows + wave * 32 + lane] = make_float2(mn, ln);
}

// c[bh][row] = -max - log2(bl * sumexp) for row < bl, -inf for the padding rows.
// 1024 threads: thread (grp, row) folds the partials grp, grp+8, ... of its row, then the 8 groups meet in LDS.
__global__ __launch_bounds__(1024) void scores_merge_kernel(const float2 *__restrict__ partial,
                                                            float *__restrict__ cvec, int nwg, int bl)
{
    __shared__ float2 red[8][kQRows];
    const int bh = blockIdx.x, row = threadIdx.x & (kQRows - 1), grp = threadIdx.x >> 7;
    float mn = -INFINITY, ln = 0.0f;
    for (int w0 = grp; w0 < nwg; w0 += 32) {                 // four independent loads per round trip
        float2 pr[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int w = w0 + 8 * q;
            pr[q] = w < nwg ? partial[((size_t)bh * nwg + w) * kQRows + row] : make_float2(-INFINITY, 0.0f);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (pr[q].x != -INFINITY) {
                const float m2 = fmaxf(mn, pr[q].x);
                ln = ln * exp2f(mn - m2) + pr[q].y * exp2f(pr[q].x - m2);
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
// scores[key] = sum over the 128 rows of exp2(logit2 + c[row]): each wave sums its 32 rows per key into LDS, the
// four partial sums of a key meet once at the end of the workgroup's range.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void scores_sweep2_kernel(
    const bf16_t *__restrict__ K, const bf16_t *__restrict__ qsplit, const float *__restrict__ cvec,
    float *__restrict__ scores, Geo g, int kpw)
{
    __shared__ __align__(16) KTile kt[2];
    __shared__ float psum[4][kMaxKeysPerWg];
    const int bh = blockIdx.y;
    const int wg = gridDim.x - 1 - blockIdx.x;               // reverse order: reuse what sweep 1 left in cache
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    bf16x8 qh[8], ql[8];
    load_qfrags(qh, qsplit + (size_t)bh * 2 * kQRows * 128, wave, lane);
    load_qfrags(ql, qsplit + (size_t)bh * 2 * kQRows * 128 + kQRows * 128, wave, lane);
    // the accumulator starts at c[row]; row = 32 wave + 8 (i / 4) + 4 (lane >> 5) + (i % 4)
    floatx16 cinit;
#pragma unroll
    for (int i = 0; i < 16; ++i)
        cinit[i] = cvec[(size_t)bh * kQRows + 32 * wave + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3)];
    const bf16_t *Kh = K + (size_t)bh * g.n * 128;
    const int key_begin = wg * kpw, key_end = min(g.n, key_begin + kpw);
    const int ntiles = ceil_div(key_end - key_begin, kTileKeys);
    sweep_tiles(kt, Kh, key_begin, ntiles, g.n, tid, [&](int t, const KTile &tile) {
        floatx16 acc = cinit;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 kf = kfrag(tile, ks, lane);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qh[ks], kf, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ql[ks], kf, acc, 0, 0, 0);
        }
        float sum = 0.0f;
#pragma unroll
        for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(acc[i]);
        sum += __shfl_xor(sum, 32, 64);
        if (lane < 32) psum[wave][t * kTileKeys + lane] = sum;      // key = key_begin + 32 t + lane
    });
    // the loop's last barrier has made every partial sum visible
    for (int k = tid; k < key_end - key_begin; k += 256)
        scores[(size_t)bh * g.n + key_begin + k] = (psum[0][k] + psum[1][k]) + (psum[2][k] + psum[3][k]);
}

// ------------------------------------------------------------------ generic path (fp64 accumulation)
template <typename E>
__global__ __launch_bounds__(256) void qhat_f64_kernel(const E *__restrict__ Q, double *__restrict__ qhat, Geo g,
                                                       int bl, const int32_t *__restrict__ qrows,
                                                       const double *__restrict__ qavg)
{
    const int bh = blockIdx.x;
    const int b = bh / g.h_kv, h = bh % g.h_kv;
    for (int idx = threadIdx.x; idx < bl * g.d; idx += blockDim.x) {
        const int row = idx / g.d, e = idx % g.d;
        if (qavg) {
            qhat[(size_t)bh * bl * g.d + idx] = qavg[(size_t)bh * 128 + e];
            continue;
        }
        const int pos = query_row_position(qrows, row, bl, g.n);
        double acc = 0.0;
        for (int t = 0; t < g.r; ++t)
            acc += (double)ElemTraits<E>::to_float(Q[(((size_t)b * g.h_q + h * g.r + t) * g.n + pos) * g.d + e]);
        qhat[(size_t)bh * bl * g.d + idx] = acc / (double)g.r;
    }
}

// ------------------------------------------------------------------ the average query (one proxy of the ablations)
// partial[bh][chunk][e] = fp64 sum over the chunk's positions and the group's r heads of Q[.., pos, e];
// grid = (kAvgChunks, nbh), 256 threads: thread (e = tid % d, slot = tid / d) walks the positions slot, slot + 256/d, ..
constexpr int kAvgChunks = 128;

template <typename E>
__global__ __launch_bounds__(256) void qavg_partial_kernel(const E *__restrict__ Q, double *__restrict__ partial, Geo g)
{
    __shared__ double red[256];
    const int bh = blockIdx.y, chunk = blockIdx.x;
    const int b = bh / g.h_kv, h = bh % g.h_kv;
    const int per = ceil_div(g.n, kAvgChunks);
    const int lo = chunk * per, hi = min(g.n, lo + per);
    const int e = threadIdx.x % g.d, slot = threadIdx.x / g.d, slots = 256 / g.d;
    double acc = 0.0;
    for (int t = 0; t < g.r; ++t) {
        const E *Qh = Q + ((size_t)b * g.h_q + h * g.r + t) * (size_t)g.n * g.d;
        for (int pos = lo + slot; pos < hi; pos += slots) acc += (double)ElemTraits<E>::to_float(Qh[(size_t)pos * g.d + e]);
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    if ((int)threadIdx.x < g.d) {
        double s = 0.0;
        for (int q = 0; q < slots; ++q) s += red[q * g.d + threadIdx.x];
        partial[((size_t)bh * kAvgChunks + chunk) * 128 + threadIdx.x] = s;
    }
}

// qavg[bh][e] = (sum of the partials) / (r * n)
__global__ __launch_bounds__(128) void qavg_final_kernel(const double *__restrict__ partial, double *__restrict__ qavg,
                                                         Geo g)
{
    const int bh = blockIdx.x, e = threadIdx.x;
    if (e >= g.d) return;
    double s = 0.0;
    for (int c = 0; c < kAvgChunks; ++c) s += partial[((size_t)bh * kAvgChunks + c) * 128 + e];
    qavg[(size_t)bh * 128 + e] = s / ((double)g.r * (double)g.n);
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
        const double v = dot_f64(q, Kh + (size_t)j * g.d, g.d) * g.scale64;
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
        if ((int)threadIdx.x < nr) st[threadIdx.x] = stats[(size_t)bh * bl + r0 + threadIdx.x];
        __syncthreads();
        for (int rr = 0; rr < nr; ++rr) {
            const double v = dot_f64(q[rr], krow, g.d) * g.scale64;
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

// bytes of the average-query region at the end of the workspace: the partial sums and the mean itself
static size_t ws_avg_query(size_t nbh) { return align_up(nbh * (kAvgChunks + 1) * 128 * sizeof(double), kWsAlign); }

// The generic path sizes its workspace for up to kQRows query rows (the block size may be smaller).
size_t ws_key_scores(const pbs_problem *p)
{
    const Geo g = make_geo(p);
    const size_t nbh = (size_t)g.batch * g.h_kv;
    if (use_mfma(p)) {
        const size_t nwg = ceil_div(g.n, sweep_keys_per_wg(g));
        return align_up(nbh * 2 * kQRows * 128 * sizeof(bf16_t), kWsAlign) +
               align_up(nbh * nwg * kQRows * sizeof(float2), kWsAlign) + align_up(nbh * kQRows * sizeof(float), kWsAlign) +
               ws_avg_query(nbh);
    }
    const size_t chunks = ceil_div(g.n, kGenericKeysPerChunk);
    const size_t rows = kQRows;
    return align_up(nbh * rows * g.d * sizeof(double), kWsAlign) + align_up(nbh * rows * chunks * sizeof(double2), kWsAlign) +
           align_up(nbh * rows * sizeof(double2), kWsAlign) + ws_avg_query(nbh);
}

// The average query of every kv head into qavg (fp64, 128 doubles per head), through `partial`.
template <typename E>
static pbs_status run_qavg(const Geo &g, const void *Q, double *partial, double *qavg, hipStream_t s)
{
    const int nbh = g.batch * g.h_kv;
    pbs_status st;
    if ((st = launch(qavg_partial_kernel<E>, dim3(kAvgChunks, nbh), dim3(256), 0, s, (const E *)Q, partial, g)) != PBS_OK)
        return st;
    return launch(qavg_final_kernel, dim3(nbh), dim3(128), 0, s, (const double *)partial, qavg, g);
}

// bl query rows: the last bl of the sequence (qrows == NULL), the listed ones, or (avg) the one average query.
template <typename E>
static pbs_status run_generic(const pbs_problem *p, const Geo &g, const void *Q, const void *K, float *scores,
                              char *ws, int bl, const int32_t *qrows, bool avg, hipStream_t s)
{
    const int nbh = g.batch * g.h_kv;
    const int chunks = ceil_div(g.n, kGenericKeysPerChunk);
    double *qhat = reinterpret_cast<double *>(ws);
    ws += align_up((size_t)nbh * kQRows * g.d * sizeof(double), kWsAlign);
    double2 *partial = reinterpret_cast<double2 *>(ws);
    ws += align_up((size_t)nbh * kQRows * chunks * sizeof(double2), kWsAlign);
    double2 *stats = reinterpret_cast<double2 *>(ws);
    ws += align_up((size_t)nbh * kQRows * sizeof(double2), kWsAlign);
    double *avg_partial = reinterpret_cast<double *>(ws), *qavg = avg_partial + (size_t)nbh * kAvgChunks * 128;
    pbs_status st;
    if (avg && (st = run_qavg<E>(g, Q, avg_partial, qavg, s)) != PBS_OK) return st;
    if ((st = launch(qhat_f64_kernel<E>, dim3(nbh), dim3(256), 0, s, (const E *)Q, qhat, g, bl, qrows,
                     (const double *)(avg ? qavg : nullptr))) != PBS_OK) return st;
    if ((st = launch(scores_stats_f64_kernel<E>, dim3(chunks, bl, nbh), dim3(256), 0, s, (const E *)K, qhat, partial,
                       g, bl, kGenericKeysPerChunk)) != PBS_OK) return st;
    if ((st = launch(scores_merge_f64_kernel, dim3(nbh), dim3(128), 0, s, partial, stats, bl, chunks)) != PBS_OK) return st;
    st = launch(scores_final_f64_kernel<E>, dim3(ceil_div(g.n, 256), nbh), dim3(256), 0, s, (const E *)K, qhat,
                       stats, scores, g, bl);
    (void)p;
    return st;
}

}  // namespace pbs

using namespace pbs;

// Everything after the argument checks: the launches of one scoring call with its scratch memory at `ws`.
// proxy: which query rows stand for all queries (pbs_proxy); qrows / m only for PBS_PROXY_QUERY_ROWS.
static pbs_status enqueue_key_scores(const pbs_problem *p, int proxy, const int32_t *qrows, int m, const void *Q,
                                     const void *K, float *scores, void *ws, hipStream_t s)
{
    pbs_status st;
    const Geo g = make_geo(p);
    char *w = reinterpret_cast<char *>(ws);
    const bool avg = proxy == PBS_PROXY_AVG_QUERY;
    const int bl = avg ? 1 : (proxy == PBS_PROXY_QUERY_ROWS ? m : (g.block < g.n ? g.block : g.n));
    if (proxy != PBS_PROXY_QUERY_ROWS) qrows = nullptr;
    if (!use_mfma(p)) {
        if (p->dtype == PBS_BF16) return run_generic<bf16_t>(p, g, Q, K, scores, w, bl, qrows, avg, s);
        return run_generic<float>(p, g, Q, K, scores, w, bl, qrows, avg, s);
    }
    const int nbh = g.batch * g.h_kv;
    const int kpw = sweep_keys_per_wg(g);
    const int nwg = ceil_div(g.n, kpw);
    bf16_t *qsplit = reinterpret_cast<bf16_t *>(w);
    w += align_up((size_t)nbh * 2 * kQRows * 128 * sizeof(bf16_t), kWsAlign);
    float2 *partial = reinterpret_cast<float2 *>(w);
    w += align_up((size_t)nbh * nwg * kQRows * sizeof(float2), kWsAlign);
    float *cvec = reinterpret_cast<float *>(w);
    w += align_up((size_t)nbh * kQRows * sizeof(float), kWsAlign);
    double *avg_partial = reinterpret_cast<double *>(w), *qavg = avg_partial + (size_t)nbh * kAvgChunks * 128;
    if (avg && (st = run_qavg<bf16_t>(g, Q, avg_partial, qavg, s)) != PBS_OK) return st;
    if ((st = launch(qhat_split_kernel, dim3(kQRows / 8, nbh), dim3(256), 0, s, (const bf16_t *)Q, qsplit, g, bl, qrows,
                     (const double *)(avg ? qavg : nullptr))) != PBS_OK) return st;
    if ((st = launch(scores_sweep1_kernel, dim3(nwg, nbh), dim3(256), 0, s, (const bf16_t *)K, qsplit, partial, g, kpw)) != PBS_OK) return st;
    if ((st = launch(scores_merge_kernel, dim3(nbh), dim3(1024), 0, s, partial, cvec, nwg, bl)) != PBS_OK) return st;
    return launch(scores_sweep2_kernel, dim3(nwg, nbh), dim3(256), 0, s, (const bf16_t *)K, qsplit, cvec, scores,
                       g, kpw);
}

extern "C" pbs_status pbs_key_scores(const pbs_problem *p, const void *Q, const void *K, float *scores, void *ws,
                                     size_t ws_bytes, void *stream)
{
    pbs_status st = validate(p);
    if (st != PBS_OK) return st;
    if (!Q || !K || !scores) return PBS_ERR_NULL;
    if (!aligned16(Q) || !aligned16(K)) return PBS_ERR_SHAPE;
    if ((st = check_ws(p, PBS_STAGE_KEY_SCORES, ws, ws_bytes)) != PBS_OK) return st;
    return enqueue_key_scores(p, PBS_PROXY_LAST_BLOCK, nullptr, 0, Q, K, scores, ws, (hipStream_t)stream);
}

extern "C" pbs_status pbs_key_scores_proxy(const pbs_problem *p, int proxy, const int32_t *qrows, int32_t m,
                                           const void *Q, const void *K, float *scores, void *ws, size_t ws_bytes,
                                           void *stream)
{
    pbs_status st = validate(p);
    if (st != PBS_OK) return st;
    if (!Q || !K || !scores) return PBS_ERR_NULL;
    if (proxy != PBS_PROXY_LAST_BLOCK && proxy != PBS_PROXY_QUERY_ROWS && proxy != PBS_PROXY_AVG_QUERY)
        return PBS_ERR_UNSUPPORTED;
    if (proxy == PBS_PROXY_QUERY_ROWS && !qrows) return PBS_ERR_NULL;
    if (proxy == PBS_PROXY_QUERY_ROWS && (m < 1 || m > kQRows)) return PBS_ERR_SHAPE;
    if (!aligned16(Q) || !aligned16(K)) return PBS_ERR_SHAPE;
    if ((st = check_ws(p, PBS_STAGE_KEY_SCORES, ws, ws_bytes)) != PBS_OK) return st;
    return enqueue_key_scores(p, proxy, qrows, m, Q, K, scores, ws, (hipStream_t)stream);
}

// ------------------------------------------------------------------ the entry point that allocates nothing
// pbs_key_scores with its scratch memory (split Qhat, per-workgroup row statistics, merged constants) in a
// file-scope device array instead of a caller-supplied workspace.  Every GPU holds its own copy of the array at its
// own address; the address is looked up once per device, with that device current, and host code only ever uses
// that address, never the array's name.
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static void *static_scratch_of_current_device()
{
    constexpr int kMaxDevices = 64;
    static std::atomic<void *> ptr_of[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void *ptr = ptr_of[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
        ptr_of[dev].store(ptr, std::memory_order_release);   // racing first calls look up the same address
    }
    return ptr;
}

extern "C" size_t pbs_key_scores_static_scratch_bytes(void) { return kStaticScratchBytes; }

extern "C" pbs_status pbs_key_scores_static(const pbs_problem *p, const void *Q, const void *K, float *scores,
                                            void *stream)
{
    pbs_status st = validate(p);
    if (st != PBS_OK) return st;
    if (!Q || !K || !scores) return PBS_ERR_NULL;
    if (!aligned16(Q) || !aligned16(K)) return PBS_ERR_SHAPE;
    if (pbs_workspace_bytes(p, PBS_STAGE_KEY_SCORES) > kStaticScratchBytes) return PBS_ERR_WORKSPACE;
    void *ws = static_scratch_of_current_device();
    if (!ws) return PBS_ERR_HIP;
    return enqueue_key_scores(p, PBS_PROXY_LAST_BLOCK, nullptr, 0, Q, K, scores, ws, (hipStream_t)stream);
}
