// Segmented permutation (Eq. 5 + Algorithm 1's first and last steps): per-segment stable descending
// argsort of the key scores, row gathers for K' and Q', the block-transposed gather for V', and the
// inverse row scatter for the output.  Pure integer/compare and copy work: bound by HBM.
#include "pbs_host.h"

namespace pbs {

// ---------------------------------------------------------------------------------------------
// One workgroup sorts one segment in LDS.  Key = (~orderable(score)) << 32 | position-in-segment, so an
// ascending 64-bit bitonic sort yields descending score with ties in ascending position.  -0.0 is
// folded onto +0.0 first so that the bit order agrees with the arithmetic order.
// One thread per compare-exchange pair (two pairs when the padded segment has 4096 keys).  The 64 pairs of a
// wave at strides up to 64 lie inside 128 consecutive keys that no other wave touches, so those stages (49 of
// the 55 at 1024 keys) are ordered by the wave's own in-order LDS accesses and only the wider strides meet at
// a workgroup barrier.
// grid = (G + 1, batch*h_kv); workgroup G writes the identity for the unpermuted tail.
// ---------------------------------------------------------------------------------------------
// identity != NULL: the positions 0 .. n-1 are written there as well (the kidx of a token-order copy).
// INT_KEYS: `scores` holds int32 keys instead, sorted ascending (equal keys in ascending position).
template <bool INT_KEYS>
__global__ __launch_bounds__(1024) void segment_argsort_kernel(const float *__restrict__ scores,
                                                               int32_t *__restrict__ kidx,
                                                               int32_t *__restrict__ identity, int n, int segment,
                                                               int G, int p2)
{
    extern __shared__ uint64_t keys[];
    const int g = blockIdx.x;
    const size_t base = (size_t)blockIdx.y * n;
    if (identity) {
        const int lo = g * segment, hi = g >= G ? n : lo + segment;
        for (int p = lo + threadIdx.x; p < hi; p += blockDim.x) identity[base + p] = p;
    }
    if (g >= G) {
        for (int p = G * segment + threadIdx.x; p < n; p += blockDim.x) kidx[base + p] = p;
        return;
    }
    const float *s = scores + base + (size_t)g * segment;
    for (int t = threadIdx.x; t < p2; t += blockDim.x) {
        uint64_t key = ~0ull;
        if (t < segment) {
            if (INT_KEYS) {
                const uint32_t u = (uint32_t)reinterpret_cast<const int32_t *>(s)[t] ^ 0x80000000u;   // signed order
                key = ((uint64_t)u << 32) | (uint32_t)t;
            } else {
                float f = s[t] + 0.0f;
                uint32_t u = __float_as_uint(f);
                u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);   // ascending in u == ascending in f
                key = ((uint64_t)(~u) << 32) | (uint32_t)t;
            }
        }
        keys[t] = key;
    }
    __syncthreads();
    for (int k = 2; k <= p2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < (p2 >> 1); t += blockDim.x) {
                // t-th compare-exchange pair of this stage: insert a zero bit at position log2(j)
                const int lo = t & (j - 1);
                const int a = ((t - lo) << 1) | lo;
                const int b = a | j;
                const bool asc = (a & k) == 0;
                const uint64_t ka = keys[a], kb = keys[b];
                if ((ka > kb) == asc) { keys[a] = kb; keys[b] = ka; }
            }
            // strides up to 64 wrote only the wave's own keys, which are all that its next stage reads
            if (j > 64) {
                __syncthreads();
            } else {
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
        }
        if (k > 64) __syncthreads();                         // the next k starts at stride k, across waves
    }
    for (int t = threadIdx.x; t < segment; t += blockDim.x)
        kidx[base + (size_t)g * segment + t] = g * segment + (int32_t)(keys[t] & 0xffffffffu);
}

__global__ __launch_bounds__(256) void iota_kernel(int32_t *__restrict__ idx, int32_t *__restrict__ idx2, int n,
                                                   size_t total)
{
    for (size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x; p < total; p += (size_t)gridDim.x * blockDim.x) {
        idx[p] = (int32_t)(p % (size_t)n);
        if (idx2) idx2[p] = (int32_t)(p % (size_t)n);
    }
}

// A 16-byte load of a source row.  Rows that are read once are read past the caches' retention (non-temporal); with
// the token-order copy every row is read twice, by neighbouring workgroups, and the second read should find it.
template <bool TWICE, typename T>
__device__ inline T load_once_or_twice(const T *ptr)
{
    if constexpr (TWICE) return *ptr;
    else return __builtin_nontemporal_load(ptr);
}

// ---------------------------------------------------------------------------------------------
// Row gather / scatter in 16-byte chunks; cpr = chunks per row (a power of two).
// SCATTER = false: dst[row] = src[head(row), idx[row]]     (X' = P X)
// SCATTER = true : dst[head(row), idx[row]] = src[row]     (O = P^T O')
// idx == NULL is the identity.  An index outside [0, n) gives a zero row (gather) or is dropped (scatter).
// ---------------------------------------------------------------------------------------------
// copy_stride > 0 (gather only): the grid is twice as wide; odd workgroups write a plain copy of the same range of
// rows copy_stride chunks behind dst (the token-order copy), right next in time to the even workgroup that gathers
// rows of the same segments, so that most of what they read is still in the last-level caches.
template <bool SCATTER, bool TWICE = false>
__global__ __launch_bounds__(256) void move_rows_kernel(const uintx4 *__restrict__ src,
                                                        const int32_t *__restrict__ idx,
                                                        uintx4 *__restrict__ dst, int n, int cpr_log2,
                                                        size_t copy_stride)
{
    // grid = (x, nbh): blockIdx.y is the head; workgroup x owns a contiguous range of that head's n * cpr chunks and
    // moves it in batches of U x 256 chunks: all index loads of a batch, then all data loads, then all stores, so
    // that every thread keeps U independent 16-byte loads in flight.
    constexpr int U = 4;
    const size_t head = (size_t)blockIdx.y * n;
    const uint32_t chunks = (uint32_t)n << cpr_log2;
    const uint32_t cmask = (1u << cpr_log2) - 1u;
    const bool plain = copy_stride != 0 && (blockIdx.x & 1);
    const uint32_t wg = copy_stride ? blockIdx.x >> 1 : blockIdx.x, nwg = copy_stride ? gridDim.x >> 1 : gridDim.x;
    const uintx4 *hsrc = src + (head << cpr_log2);
    uintx4 *hdst = dst + (head << cpr_log2) + (plain ? copy_stride : 0);
    const int32_t *hidx = (idx && !plain) ? idx + head : nullptr;
    const uint32_t batch = U * 256;
    const uint32_t per = ((chunks + nwg - 1) / nwg + batch - 1) / batch * batch;
    const uint32_t begin = min(wg * per, chunks), end = min(begin + per, chunks);
    for (uint32_t c0 = begin + threadIdx.x; c0 < end; c0 += batch) {
        int32_t other[U];
        uintx4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t c = c0 + u * 256;
            other[u] = c < end ? (hidx ? hidx[c >> cpr_log2] : (int32_t)(c >> cpr_log2)) : -1;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t c = c0 + u * 256;
            const bool ok = other[u] >= 0 && other[u] < n;
            v[u] = uintx4{0u, 0u, 0u, 0u};
            if (SCATTER ? c < end : ok)
                v[u] = load_once_or_twice<TWICE>(hsrc + (SCATTER ? c : ((uint32_t)other[u] << cpr_log2) + (c & cmask)));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t c = c0 + u * 256;
            const bool ok = other[u] >= 0 && other[u] < n;
            if (SCATTER ? ok : c < end)
                __builtin_nontemporal_store(v[u], hdst + (SCATTER ? ((uint32_t)other[u] << cpr_log2) + (c & cmask) : c));
        }
    }
}

// ---------------------------------------------------------------------------------------------
// The row gather of K' for 2-byte storage (move_rows_kernel<false> with the same grid, ranges and token-order copy)
// that also leaves the block means of K' behind, as Algorithm 2 needs them next: kbarT[head][feature][Ts] fp64.
// A workgroup owns whole key blocks (its range is a multiple of block * cpr chunks, and a block is a whole number of
// 1024-chunk batches), a thread always meets the same 16-byte column group, so it adds up its rows' eight features in
// fp64 registers while the rows pass through (sums of bf16 values are exact in fp64 in any order), and at the end of
// every block the 256 / cpr row slots of a column meet in LDS.  dst == NULL: only the block means are produced (index
// remapping: the attention kernel gathers the rows itself and no K' is written).
// ---------------------------------------------------------------------------------------------
template <bool TWICE>
__global__ __launch_bounds__(256) void gather_pool_kernel(const uintx4 *__restrict__ src,
                                                          const int32_t *__restrict__ idx, uintx4 *__restrict__ dst,
                                                          int n, int cpr_log2, size_t copy_stride,
                                                          double *__restrict__ kbarT, int block, int Ts)
{
    constexpr int U = 4;
    __shared__ double red[256 * 8];
    const size_t head = (size_t)blockIdx.y * n;
    const uint32_t chunks = (uint32_t)n << cpr_log2;
    const uint32_t cpr = 1u << cpr_log2, cmask = cpr - 1u;
    const bool plain = copy_stride != 0 && (blockIdx.x & 1);
    const uint32_t wg = copy_stride ? blockIdx.x >> 1 : blockIdx.x, nwg = copy_stride ? gridDim.x >> 1 : gridDim.x;
    const uintx4 *hsrc = src + (head << cpr_log2);
    uintx4 *hdst = dst + (head << cpr_log2) + (plain ? copy_stride : 0);
    const int32_t *hidx = (idx && !plain) ? idx + head : nullptr;
    const uint32_t batch = U * 256;
    const uint32_t cpb = (uint32_t)block << cpr_log2;        // chunks per key block, a multiple of batch
    const uint32_t per = ((chunks + nwg - 1) / nwg + cpb - 1) / cpb * cpb;
    const uint32_t begin = min(wg * per, chunks), end = min(begin + per, chunks);
    const int d = 8 << cpr_log2;
    double acc[8];
#pragma unroll
    for (int x = 0; x < 8; ++x) acc[x] = 0.0;
    for (uint32_t base = begin; base < end; base += batch) {
        int32_t other[U];
        uintx4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t c = base + threadIdx.x + u * 256;
            other[u] = c < end ? (hidx ? hidx[c >> cpr_log2] : (int32_t)(c >> cpr_log2)) : -1;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t c = base + threadIdx.x + u * 256;
            v[u] = uintx4{0u, 0u, 0u, 0u};
            if (other[u] >= 0 && other[u] < n)
                v[u] = load_once_or_twice<TWICE>(hsrc + ((uint32_t)other[u] << cpr_log2) + (c & cmask));
        }
        if (dst) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t c = base + threadIdx.x + u * 256;
                if (c < end) __builtin_nontemporal_store(v[u], hdst + c);
            }
        }
        if (plain) continue;                                  // uniform: the token-order copy is not pooled
#pragma unroll
        for (int u = 0; u < U; ++u)                           // rows past the end were loaded as zeros
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                acc[2 * x] += (double)__uint_as_float(v[u][x] << 16);
                acc[2 * x + 1] += (double)__uint_as_float(v[u][x] & 0xffff0000u);
            }
        const uint32_t done = base + batch - begin;
        if (done % cpb == 0 || base + batch >= end) {         // uniform: a key block is complete
            const int blk = (int)((base >> cpr_log2) / (uint32_t)block);
            const int rows = min(block, n - blk * block);
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                red[threadIdx.x * 8 + x] = acc[x];
                acc[x] = 0.0;
            }
            __syncthreads();
            if ((int)threadIdx.x < d) {
                const int e = threadIdx.x;
                double s = 0.0;
                for (uint32_t q = 0; q < 256 / cpr; ++q) s += red[(q * cpr + (e >> 3)) * 8 + (e & 7)];
                kbarT[((size_t)blockIdx.y * d + e) * Ts + blk] = s / (double)rows;
            }
            __syncthreads();
        }
    }
}

// ---------------------------------------------------------------------------------------------
// V' in the block-transposed layout Vt[bh][j][e][c] = V[bh][kidx[j*block + c]][e] (zero for slots >= n).
// One workgroup per (key block j, bh): gathered rows go to LDS with coalesced 16-byte reads, the tile is
// read back column-wise in 4-byte words and leaves as 16-byte pieces of Vt rows (VEC keys of one feature),
// neighbouring lanes writing neighbouring pieces of a key group, then the next feature.  LDS row r starts at word
// r * (row words) + (r / VEC) * (64 / gpp) with gpp pieces per Vt row: the lanes of a wave read gpp pieces x
// 64 / gpp word columns, which then fall into 64 different banks.
// E = storage type (2 or 4 bytes); VEC = elements per 16-byte chunk.
// ---------------------------------------------------------------------------------------------
// copy_stride > 0: the grid is twice as wide; odd workgroups transpose the same key block without the permutation
// into the copy copy_stride elements behind Vt (see move_rows_kernel).
template <typename E, bool TWICE>
__global__ __launch_bounds__(256) void gather_vt_kernel(const E *__restrict__ V, const int32_t *__restrict__ kidx,
                                                        E *__restrict__ Vt, int n, int d, int block, int T,
                                                        size_t copy_stride)
{
    constexpr int VEC = 16 / sizeof(E);
    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint32_t *tile = reinterpret_cast<uint32_t *>(smem_raw);
    const int roww = d * (int)sizeof(E) / 4;               // 4-byte words per row
    const bool plain = copy_stride != 0 && (blockIdx.x & 1);
    const int j = copy_stride ? blockIdx.x >> 1 : blockIdx.x;
    const size_t bh = blockIdx.y;
    if (plain) kidx = nullptr;
    const int cpr = d / VEC;
    const int G = vt_group(block);                         // keys per transposed group
    const int gpp = G / VEC;                               // 16-byte pieces per Vt row
    const int skew = 64 / gpp;                             // words; gpp is 2, 4 or 8
    typedef E vec_t __attribute__((ext_vector_type(VEC)));
    // batches of U chunks per thread: index loads, then row loads, then the LDS stores
    constexpr int U = 4;
    const int total = block * cpr;
    for (int c0 = threadIdx.x; c0 < total; c0 += U * 256) {
        int32_t from[U];
        vec_t v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + u * 256;
            const int slot = j * block + c / cpr;
            from[u] = (c < total && slot < n) ? (kidx ? kidx[bh * n + slot] : slot) : -1;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + u * 256;
            v[u] = vec_t{};
            if (from[u] >= 0 && from[u] < n)
                v[u] = load_once_or_twice<TWICE>(reinterpret_cast<const vec_t *>(V + (bh * n + from[u]) * (size_t)d + (c % cpr) * VEC));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + u * 256;
            const int row = c / cpr;
            if (c < total) *reinterpret_cast<vec_t *>(tile + row * roww + (row / VEC) * skew + (c % cpr) * 4) = v[u];
        }
    }
    __syncthreads();
    E *out = Vt + (bh * T + j) * (size_t)d * block + (plain ? copy_stride : 0);
    for (int c = threadIdx.x; c < roww * (block / VEC); c += blockDim.x) {
        const int kgi = c % gpp, w = (c / gpp) % roww, gi = c / (gpp * roww);
        const int kg = gi * gpp + kgi;                     // word column w of the rows kg*VEC .. kg*VEC+VEC-1
        uint32_t x[VEC];
#pragma unroll
        for (int u = 0; u < VEC; ++u) x[u] = tile[(kg * VEC + u) * roww + kg * skew + w];
        E *og = out + (size_t)gi * d * G + kgi * VEC;      // feature e of this piece: og + e * G
        if (sizeof(E) == 4) {
            uintx4 v;
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = x[u];
            __builtin_nontemporal_store(v, reinterpret_cast<uintx4 *>(og + (size_t)w * G));
        } else {                                           // word w holds elements 2w (low half) and 2w + 1
            uintx4 lo, hi;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                lo[u] = __builtin_amdgcn_perm(x[(2 * u + 1) % VEC], x[(2 * u) % VEC], 0x05040100u);
                hi[u] = __builtin_amdgcn_perm(x[(2 * u + 1) % VEC], x[(2 * u) % VEC], 0x07060302u);
            }
            __builtin_nontemporal_store(lo, reinterpret_cast<uintx4 *>(og + (size_t)(2 * w) * G));
            __builtin_nontemporal_store(hi, reinterpret_cast<uintx4 *>(og + (size_t)(2 * w + 1) * G));
        }
    }
}

static int ilog2(int v) { int l = 0; while ((1 << l) < v) ++l; return l; }

static int grid_for(size_t items, int per_block)
{
    size_t b = (items + per_block - 1) / per_block;
    const size_t cap = 256 * 32;                          // 32 workgroups per CU is plenty for a copy
    if (b > cap) b = cap;
    if (b < 1) b = 1;
    return (int)b;
}

// grid for move_rows_kernel and gather_pool_kernel: one batch of 4 x 256 chunks (16 KiB) per workgroup -- or `unit`
// chunks where a workgroup has to own whole key blocks --, so that the workgroups in flight at any time sweep one
// narrow window of addresses (measured on a plain 1 GiB copy: 5.3 TB/s read + write with 1024 long ranges, 6.3 with
// 65536 short ones and non-temporal accesses)
static dim3 move_grid(int n, int cpr, int nbh, size_t unit = 256 * 4)
{
    const size_t chunks = (size_t)n * cpr;
    size_t bx = (chunks + unit - 1) / unit;
    if (bx < 1) bx = 1;
    return dim3((unsigned)bx, (unsigned)nbh);
}

// idx[head][g*S + t] = position of the query with the t-th smallest (key, position) of segment g; the tail keeps its place.
pbs_status launch_segment_sort_by_int_key(const Geo &g, int heads, const int32_t *keys, int32_t *idx, hipStream_t s)
{
    int p2 = 1;
    while (p2 < g.segment) p2 <<= 1;
    const int threads = p2 / 2 < 64 ? 64 : (p2 / 2 > 1024 ? 1024 : p2 / 2);
    return launch(segment_argsort_kernel<true>, dim3(g.G + 1, heads), dim3(threads), (size_t)p2 * sizeof(uint64_t), s,
                  reinterpret_cast<const float *>(keys), idx, (int32_t *)nullptr, g.n, g.segment, g.G, p2);
}

size_t ws_block_mask(const pbs_problem *p);
pbs_status launch_pool_keys(const pbs_problem *p, const Geo &g, const void *Kp, double *KbarT, hipStream_t s);

}  // namespace pbs

using namespace pbs;

extern "C" pbs_status pbs_segment_permute(const pbs_problem *p, const float *scores, const void *K, const void *V,
                                          int32_t *kidx, void *Kp, void *Vt, void *ws, size_t ws_bytes,
                                          void *stream)
{
    pbs_status st = validate(p);
    if (st != PBS_OK) return st;
    if (!kidx) return PBS_ERR_NULL;
    const bool remap = (p->flags & PBS_FLAG_INDEX_REMAP) != 0;    // no K' is written: Kp is ignored and may be NULL
    if (remap) {
        if (p->flags & PBS_FLAG_TOKEN_ORDER_COPY) return PBS_ERR_UNSUPPORTED;
        if (Vt && !Kp) Kp = Vt;                                   // "both or none" below is about Vt alone then
        if (!Vt) Kp = nullptr;
    }
    if ((Kp == nullptr) != (Vt == nullptr)) return PBS_ERR_NULL;
    if (ws && Kp && ((reinterpret_cast<uintptr_t>(ws) & (kWsAlign - 1)) != 0 || ws_bytes < ws_block_mask(p)))
        return PBS_ERR_WORKSPACE;
    if (Kp && (!K || !V)) return PBS_ERR_NULL;
    if (Kp && (!aligned16(K) || !aligned16(V) || !aligned16(Kp) || !aligned16(Vt))) return PBS_ERR_SHAPE;
    void *kdst = remap ? nullptr : Kp;
    const Geo g = make_geo(p);
    hipStream_t s = (hipStream_t)stream;
    const int nbh = g.batch * g.h_kv;
    const bool token_copy = (p->flags & PBS_FLAG_TOKEN_ORDER_COPY) != 0;
    const size_t tok_rows = (size_t)nbh * g.T * g.block;   // the token-order copies start this many rows in
    int32_t *kidx_tok = token_copy ? kidx + tok_rows : nullptr;
    if (scores) {
        int p2 = 1;
        while (p2 < g.segment) p2 <<= 1;
        const int threads = p2 / 2 < 64 ? 64 : (p2 / 2 > 1024 ? 1024 : p2 / 2);
        st = launch(segment_argsort_kernel<false>, dim3(g.G + 1, nbh), dim3(threads), (size_t)p2 * sizeof(uint64_t), s,
                           scores, kidx, kidx_tok, g.n, g.segment, g.G, p2);
    } else {
        const size_t total = (size_t)nbh * g.n;
        st = launch(iota_kernel, dim3(grid_for(total, 256)), dim3(256), 0, s, kidx, kidx_tok, g.n, total);
    }
    if (st != PBS_OK) return st;
    if (!Kp) return PBS_OK;
    const size_t es = elem_size(p->dtype);
    const int cpr = (int)(g.d * es / 16);
    const size_t vt_half = (size_t)nbh * g.T * g.d * g.block;           // elements

    // with a workspace, the block means of K' are left there for pbs_block_mask: by the gather itself where a key
    // block is a whole number of its 1024-chunk batches (2-byte storage), by the pooling kernel otherwise
    double *kbarT = reinterpret_cast<double *>(ws);
    const bool pool_on_the_way = kbarT && p->dtype == PBS_BF16 && (g.block * cpr) % 1024 == 0;
    dim3 mg = pool_on_the_way ? move_grid(g.n, cpr, nbh, (size_t)g.block * cpr) : move_grid(g.n, cpr, nbh);
    if (token_copy) mg.x *= 2;
    if (remap && kbarT && !pool_on_the_way) return PBS_ERR_UNSUPPORTED;   // means without K' only from the gather kernel
    const size_t kcopy = token_copy ? tok_rows * cpr : (size_t)0;
    const int Tsk = kbar_stride(g.T), cl = ilog2(cpr);
    if (pool_on_the_way)
        st = token_copy ? launch(gather_pool_kernel<true>, mg, dim3(256), 0, s, (const uintx4 *)K, (const int32_t *)kidx,
                                 (uintx4 *)kdst, g.n, cl, kcopy, kbarT, g.block, Tsk)
                        : launch(gather_pool_kernel<false>, mg, dim3(256), 0, s, (const uintx4 *)K, (const int32_t *)kidx,
                                 (uintx4 *)kdst, g.n, cl, kcopy, kbarT, g.block, Tsk);
    else if (kdst)
        st = token_copy ? launch((move_rows_kernel<false, true>), mg, dim3(256), 0, s, (const uintx4 *)K,
                                 (const int32_t *)kidx, (uintx4 *)kdst, g.n, cl, kcopy)
                        : launch((move_rows_kernel<false, false>), mg, dim3(256), 0, s, (const uintx4 *)K,
                                 (const int32_t *)kidx, (uintx4 *)kdst, g.n, cl, kcopy);
    if (st != PBS_OK) return st;
    if (kbarT && !pool_on_the_way && (st = launch_pool_keys(p, g, Kp, kbarT, s)) != PBS_OK) return st;
    const dim3 vg(token_copy ? 2 * g.T : g.T, nbh);
    const size_t vcopy = token_copy ? vt_half : (size_t)0;
    if (p->dtype == PBS_BF16) {
        const size_t lds = (size_t)g.block * g.d * 2 + (size_t)(g.block / 8) * (64 / (vt_group(g.block) / 8)) * 4;   // tile + skew
        st = token_copy ? launch((gather_vt_kernel<uint16_t, true>), vg, dim3(256), lds, s, (const uint16_t *)V,
                                 (const int32_t *)kidx, (uint16_t *)Vt, g.n, g.d, g.block, g.T, vcopy)
                        : launch((gather_vt_kernel<uint16_t, false>), vg, dim3(256), lds, s, (const uint16_t *)V,
                                 (const int32_t *)kidx, (uint16_t *)Vt, g.n, g.d, g.block, g.T, vcopy);
    } else {
        const size_t lds = (size_t)g.block * g.d * 4 + (size_t)(g.block / 4) * (64 / (vt_group(g.block) / 4)) * 4;
        st = token_copy ? launch((gather_vt_kernel<uint32_t, true>), vg, dim3(256), lds, s, (const uint32_t *)V,
                                 (const int32_t *)kidx, (uint32_t *)Vt, g.n, g.d, g.block, g.T, vcopy)
                        : launch((gather_vt_kernel<uint32_t, false>), vg, dim3(256), lds, s, (const uint32_t *)V,
                                 (const int32_t *)kidx, (uint32_t *)Vt, g.n, g.d, g.block, g.T, vcopy);
    }
    return st;
}

extern "C" pbs_status pbs_permute_rows(const pbs_problem *p, int32_t heads, const void *X, const int32_t *idx,
                                       void *Xp, void *stream)
{
    pbs_status st = validate(p);
    if (st != PBS_OK) return st;
    if (!X || !idx || !Xp) return PBS_ERR_NULL;
    if (heads < 1) return PBS_ERR_SHAPE;
    if ((long long)p->batch * heads > 65535) return PBS_ERR_UNSUPPORTED;   // heads ride on gridDim.y
    if (!aligned16(X) || !aligned16(Xp) || X == Xp) return PBS_ERR_SHAPE;
    const int cpr = (int)(p->d * elem_size(p->dtype) / 16);
    return launch(move_rows_kernel<false>, move_grid(p->n, cpr, p->batch * heads), dim3(256), 0,
                       (hipStream_t)stream, (const uintx4 *)X, idx, (uintx4 *)Xp, p->n, ilog2(cpr), (size_t)0);
}

extern "C" pbs_status pbs_unpermute(const pbs_problem *p, const void *Op, const int32_t *qidx, void *O, void *stream)
{
    pbs_status st = validate(p);
    if (st != PBS_OK) return st;
    if (!Op || !O) return PBS_ERR_NULL;
    if (!aligned16(Op) || !aligned16(O)) return PBS_ERR_SHAPE;
    if (Op == O) return qidx ? PBS_ERR_SHAPE : PBS_OK;     // in place only for the identity
    const int cpr = (int)(p->d * elem_size(p->dtype) / 16);
    return launch(move_rows_kernel<true>, move_grid(p->n, cpr, p->batch * p->h_q), dim3(256), 0,
                       (hipStream_t)stream, (const uintx4 *)Op, qidx, (uintx4 *)O, p->n, ilog2(cpr), (size_t)0);
}
