// pbs_attn_fwd: Algorithm 1's main loop -- online-softmax attention over the listed key blocks only.
//
// Matrix-core kernel (bf16, d = 128, block 64 or 128).  Everything is kept TRANSPOSED so that one lane owns
// one query for the whole row of work:
//     S^T = K'_j Q'_i^T      A = K' tile rows (from LDS), B = Q' fragments (registers, loaded once)
//     O^T += V'_j^T P^T      A = V'^T tile rows (from LDS; V' is stored block-transposed in HBM), B = P^T
// With v_mfma_f32_32x32x16_bf16 the accumulator of S^T gives lane (n, h) the scores of query n against 16 keys
// of every 32-key tile, which after exp2 and a bf16 pack IS the B operand of the second product -- no
// cross-lane traffic for P, and the running max / sum / rescale of a query are lane-local (one xor-32
// exchange).  The K' tile is stored in LDS with bits 2 and 3 of the row index swapped so that the 8 values a
// lane contributes to one 16-key contraction step are 8 CONSECUTIVE keys, which lets V'^T be read from LDS
// with plain 16-byte loads.  LDS tiles are XOR-swizzled in 16-byte chunks against bank conflicts.
// A block that is not listed costs nothing: the loop runs over the list.
//
// Vector kernel (fp32 arithmetic): every other supported dtype / d / block.
#include <limits.h>

#include "pbs_host.h"

namespace pbs {

constexpr float kLog2eF = 1.4426950408889634f;
constexpr float kLn2F = 0.6931471805599453f;

__device__ inline int swap23(int m) { return (m & ~12) | ((m & 4) << 1) | ((m & 8) >> 1); }

// ---------------------------------------------------------------------------------------------
// MFMA kernel.  BLOCK = block size; WAVES = waves per workgroup; each wave owns BLOCK / WAVES query rows.
// grid = (T, batch*h_q); blockIdx.x = T-1-i so that the long rows are dispatched first.
// ---------------------------------------------------------------------------------------------
template <int BLOCK, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void attn_mfma_kernel(
    const bf16_t *__restrict__ Qp, const bf16_t *__restrict__ Kp, const bf16_t *__restrict__ Vt,
    const int32_t *__restrict__ qidx, const int32_t *__restrict__ kidx, const int32_t *__restrict__ row_cnt,
    const int32_t *__restrict__ col_idx, bf16_t *__restrict__ Op, float *__restrict__ lse, Geo g)
{
    constexpr int D = 128;
    constexpr int THREADS = WAVES * 64;
    constexpr int NT = BLOCK / WAVES / 32;         // 32-query tiles per wave
    constexpr int MT = BLOCK / 32;                 // 32-key tiles per block
    constexpr int KS2 = BLOCK / 16;                // 16-key contraction steps of the second product
    constexpr int VCH = BLOCK / 8;                 // 16-byte chunks per V'^T row
    static_assert(NT >= 1, "each wave needs at least one 32-query tile");

    __shared__ __align__(16) bf16_t ks[BLOCK * D];   // K' tile, row = swap23(key), chunk ^= row & 15
    __shared__ __align__(16) bf16_t vs[D * BLOCK];   // V'^T tile, row = d index, swizzled chunks
    __shared__ int kpos[BLOCK];                      // original positions of the tile's keys

    const int i = g.T - 1 - (int)blockIdx.x;
    const int bhq = blockIdx.y;
    const int b = bhq / g.h_q, hq = bhq % g.h_q;
    const size_t bhk = (size_t)b * g.h_kv + hq / g.r;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ln = lane & 31, lh = lane >> 5;
    const int q0 = i * BLOCK + wave * (BLOCK / WAVES);

    // Q' fragments: lane (n, h) holds Q'[q0 + 32 nt + n][16 ks + 8 h .. +8]
    bf16x8 qf[NT][8];
    int qpos[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int qs = q0 + 32 * nt + ln;
        const int qc = qs < g.n ? qs : g.n - 1;
        const bf16_t *src = Qp + ((size_t)bhq * g.n + qc) * D + 8 * lh;
#pragma unroll
        for (int k = 0; k < 8; ++k) qf[nt][k] = *reinterpret_cast<const bf16x8 *>(src + 16 * k);
        qpos[nt] = qs < g.n ? (qidx ? qidx[(size_t)bhq * g.n + qs] : qs) : -1;
    }

    floatx16 acc_o[4][NT];
    float m2[NT], l[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        m2[nt] = -INFINITY;
        l[nt] = 0.0f;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int x = 0; x < 16; ++x) acc_o[dt][nt][x] = 0.0f;
    }

    const float c2 = g.scale * kLog2eF;
    const int ni = allowed_cols(i, g);
    const int jmask = first_masked_col(i, g);
    const int cnt = min(row_cnt[(size_t)bhq * g.T + i], g.T);
    const int32_t *cols = col_idx + ((size_t)bhq * g.T + i) * g.T;
    const bf16_t *Kh = Kp + bhk * (size_t)g.n * D;
    const bf16_t *Vh = Vt + bhk * (size_t)g.T * D * BLOCK;
    const int32_t *kih = kidx + bhk * (size_t)g.n;

    for (int t = 0; t < cnt; ++t) {
        const int j = cols[t];
        if (j < 0 || j >= ni) continue;                       // uniform across the workgroup
        const bool masked = j >= jmask;
        __syncthreads();                                      // previous tile fully consumed
        // ---- stage K' tile (BLOCK rows x 16 chunks) and V'^T tile (128 rows x VCH chunks)
        for (int c = threadIdx.x; c < BLOCK * 16; c += THREADS) {
            const int row = c >> 4, ch = c & 15;
            int slot = j * BLOCK + row;
            if (slot >= g.n) slot = g.n - 1;                  // clamped; such keys are masked below
            const uintx4 v = *reinterpret_cast<const uintx4 *>(Kh + (size_t)slot * D + ch * 8);
            const int lrow = (row & ~31) | swap23(row & 31);
            *reinterpret_cast<uintx4 *>(ks + lrow * D + ((ch ^ (lrow & 15)) << 3)) = v;
        }
        for (int c = threadIdx.x; c < D * VCH; c += THREADS) {
            const int row = c / VCH, ch = c % VCH;
            const uintx4 v = *reinterpret_cast<const uintx4 *>(Vh + ((size_t)j * D + row) * BLOCK + ch * 8);
            const int sw = BLOCK == 128 ? (row & 15) : ((row >> 1) & 7);
            *reinterpret_cast<uintx4 *>(vs + row * BLOCK + ((ch ^ sw) << 3)) = v;
        }
        if (masked)
            for (int c = threadIdx.x; c < BLOCK; c += THREADS) {
                const int slot = j * BLOCK + c;
                kpos[c] = slot < g.n ? kih[slot] : INT_MAX;
            }
        __syncthreads();

        // ---- S^T = K' Q'^T
        floatx16 acc_s[MT][NT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int x = 0; x < 16; ++x) acc_s[mt][nt][x] = 0.0f;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int lrow = 32 * mt + ln;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const bf16x8 a =
                    *reinterpret_cast<const bf16x8 *>(ks + lrow * D + (((2 * k + lh) ^ (lrow & 15)) << 3));
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc_s[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[nt][k], acc_s[mt][nt], 0, 0, 0);
            }
        }
        // acc_s[mt][nt][x]: key (within the block) = 32 mt + 16 (x / 8) + 8 h + (x % 8), query = q0 + 32 nt + n

        // ---- token-level causality inside the query block's own segment / the unpermuted tail
        if (masked) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int x = 0; x < 16; ++x) {
                    const int kp = kpos[32 * mt + 16 * (x >> 3) + 8 * lh + (x & 7)];
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        if (kp > qpos[nt]) acc_s[mt][nt][x] = -INFINITY;
                }
        }

        // ---- online softmax (log2 domain), P packed to bf16 in place of the second product's B operand
        bf16x8 pf[NT][KS2];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            float rmax = -INFINITY;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int x = 0; x < 16; ++x) rmax = fmaxf(rmax, acc_s[mt][nt][x]);
            rmax = fmaxf(rmax, __shfl_xor(rmax, 32, 64));
            const float mnew = fmaxf(m2[nt], rmax * c2);
            const float muse = mnew == -INFINITY ? 0.0f : mnew;
            const float alpha = __builtin_amdgcn_exp2f(m2[nt] - muse);
            float rsum = 0.0f;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    floatx2 pr[4];
#pragma unroll
                    for (int x = 0; x < 8; ++x) {
                        const float p = __builtin_amdgcn_exp2f(acc_s[mt][nt][8 * u + x] * c2 - muse);
                        rsum += p;
                        pr[x >> 1][x & 1] = p;
                    }
                    bf16x8 pk;
#pragma unroll
                    for (int y = 0; y < 4; ++y) {
                        const bf16x2 t2 = __builtin_convertvector(pr[y], bf16x2);
                        pk[2 * y] = t2[0];
                        pk[2 * y + 1] = t2[1];
                    }
                    pf[nt][2 * mt + u] = pk;
                }
            l[nt] = l[nt] * alpha + rsum;
            m2[nt] = mnew;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int x = 0; x < 16; ++x) acc_o[dt][nt][x] *= alpha;
        }

        // ---- O^T += V'^T P^T
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            const int row = 32 * dt + ln;
            const int sw = BLOCK == 128 ? (row & 15) : ((row >> 1) & 7);
#pragma unroll
            for (int k2 = 0; k2 < KS2; ++k2) {
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(vs + row * BLOCK + (((2 * k2 + lh) ^ sw) << 3));
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc_o[dt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[nt][k2], acc_o[dt][nt], 0, 0, 0);
            }
        }
    }

    // ---- O' = diag(l)^-1 O; acc_o[dt][nt][x]: d = 32 dt + 8 (x / 4) + 4 h + (x % 4), query = q0 + 32 nt + n
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const float lt = l[nt] + __shfl_xor(l[nt], 32, 64);
        const float inv = lt > 0.0f ? 1.0f / lt : 0.0f;
        const int qs = q0 + 32 * nt + ln;
        if (qs < g.n) {
            bf16_t *dst = Op + ((size_t)bhq * g.n + qs) * D;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    floatx2 a = {acc_o[dt][nt][4 * gq] * inv, acc_o[dt][nt][4 * gq + 1] * inv};
                    floatx2 bb = {acc_o[dt][nt][4 * gq + 2] * inv, acc_o[dt][nt][4 * gq + 3] * inv};
                    const bf16x2 pa = __builtin_convertvector(a, bf16x2), pb = __builtin_convertvector(bb, bf16x2);
                    bf16x4 o4 = {pa[0], pa[1], pb[0], pb[1]};
                    *reinterpret_cast<bf16x4 *>(dst + 32 * dt + 8 * gq + 4 * lh) = o4;
                }
            if (lse && lh == 0)
                lse[(size_t)bhq * g.n + qs] = lt > 0.0f ? (m2[nt] + log2f(lt)) * kLn2F : -INFINITY;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Vector kernel: two threads per query row, each owning half of d.  K' and V'^T tiles are staged in LDS as
// fp32; every key updates the running (m, l, O) directly.  grid = (T, batch*h_q), 2*block threads.
// ---------------------------------------------------------------------------------------------
template <typename E, int D>
__global__ __launch_bounds__(256) void attn_vector_kernel(
    const E *__restrict__ Qp, const E *__restrict__ Kp, const E *__restrict__ Vt, const int32_t *__restrict__ qidx,
    const int32_t *__restrict__ kidx, const int32_t *__restrict__ row_cnt, const int32_t *__restrict__ col_idx,
    E *__restrict__ Op, float *__restrict__ lse, Geo g)
{
    constexpr int HALF = D / 2;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    float *kt = reinterpret_cast<float *>(smem_raw);             // [block][D]
    float *vt = kt + g.block * D;                                // [D][block]
    int *kpos = reinterpret_cast<int *>(vt + D * g.block);       // [block]

    const int i = g.T - 1 - (int)blockIdx.x;
    const int bhq = blockIdx.y;
    const int b = bhq / g.h_q, hq = bhq % g.h_q;
    const size_t bhk = (size_t)b * g.h_kv + hq / g.r;
    const int row = threadIdx.x >> 1, half = threadIdx.x & 1;
    const int qs = i * g.block + row;
    const bool live = qs < g.n;
    const int qpos = live ? (qidx ? qidx[(size_t)bhq * g.n + qs] : qs) : -1;

    float q[HALF], o[HALF];
    {
        const E *src = Qp + ((size_t)bhq * g.n + (live ? qs : g.n - 1)) * D + half * HALF;
#pragma unroll
        for (int e = 0; e < HALF; ++e) { q[e] = ElemTraits<E>::to_float(src[e]); o[e] = 0.0f; }
    }
    float m = -INFINITY, l = 0.0f;
    const int ni = allowed_cols(i, g);
    const int cnt = min(row_cnt[(size_t)bhq * g.T + i], g.T);
    const int32_t *cols = col_idx + ((size_t)bhq * g.T + i) * g.T;
    const E *Kh = Kp + bhk * (size_t)g.n * D;
    const E *Vh = Vt + bhk * (size_t)g.T * D * g.block;
    const int32_t *kih = kidx + bhk * (size_t)g.n;

    for (int t = 0; t < cnt; ++t) {
        const int j = cols[t];
        if (j < 0 || j >= ni) continue;
        __syncthreads();
        for (int c = threadIdx.x; c < g.block * D; c += blockDim.x) {
            const int kr = c / D, e = c % D;
            const int slot = j * g.block + kr;
            kt[c] = slot < g.n ? ElemTraits<E>::to_float(Kh[(size_t)slot * D + e]) : 0.0f;
            vt[c] = ElemTraits<E>::to_float(Vh[(size_t)j * D * g.block + c]);
        }
        for (int c = threadIdx.x; c < g.block; c += blockDim.x) {
            const int slot = j * g.block + c;
            kpos[c] = slot < g.n ? kih[slot] : INT_MAX;
        }
        __syncthreads();
        for (int c = 0; c < g.block; ++c) {
            float part = 0.0f;
            const float *kr = kt + c * D + half * HALF;
#pragma unroll
            for (int e = 0; e < HALF; ++e) part += q[e] * kr[e];
            const float s = (part + __shfl_xor(part, 1, 64)) * g.scale;
            if (kpos[c] > qpos) continue;
            if (s > m) {
                const float alpha = __expf(m - s);               // exp(-inf) = 0 on the first visible key
                l *= alpha;
#pragma unroll
                for (int e = 0; e < HALF; ++e) o[e] *= alpha;
                m = s;
            }
            const float p = __expf(s - m);
            l += p;
            const float *vr = vt + (half * HALF) * g.block + c;
#pragma unroll
            for (int e = 0; e < HALF; ++e) o[e] += p * vr[e * g.block];
        }
    }
    if (live) {
        const float inv = l > 0.0f ? 1.0f / l : 0.0f;
        E *dst = Op + ((size_t)bhq * g.n + qs) * D + half * HALF;
#pragma unroll
        for (int e = 0; e < HALF; ++e) dst[e] = ElemTraits<E>::from_float(o[e] * inv);
        if (lse && half == 0) lse[(size_t)bhq * g.n + qs] = l > 0.0f ? m + logf(l) : -INFINITY;
    }
}

size_t ws_attn_fwd(const pbs_problem *) { return 0; }

template <typename E, int D>
static pbs_status launch_vector(const Geo &g, const void *Qp, const void *Kp, const void *Vt, const int32_t *qidx,
                                const int32_t *kidx, const int32_t *row_cnt, const int32_t *col_idx, void *Op,
                                float *lse, hipStream_t s)
{
    const size_t lds = (size_t)2 * g.block * D * sizeof(float) + (size_t)g.block * sizeof(int);
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_vector_kernel<E, D>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 2048) != hipSuccess)
            return PBS_ERR_HIP;
        attr_set = true;
    }
    hipLaunchKernelGGL((attn_vector_kernel<E, D>), dim3(g.T, g.batch * g.h_q), dim3(2 * g.block), lds, s,
                       (const E *)Qp, (const E *)Kp, (const E *)Vt, qidx, kidx, row_cnt, col_idx, (E *)Op, lse, g);
    return launch_status();
}

}  // namespace pbs

using namespace pbs;

extern "C" pbs_status pbs_attn_fwd(const pbs_problem *p, const void *Qp, const void *Kp, const void *Vt,
                                   const int32_t *qidx, const int32_t *kidx, const int32_t *row_cnt,
                                   const int32_t *col_idx, void *Op, float *lse, void *ws, size_t ws_bytes,
                                   void *stream)
{
    (void)ws; (void)ws_bytes;
    pbs_status st = validate(p);
    if (st != PBS_OK) return st;
    if (!Qp || !Kp || !Vt || !kidx || !row_cnt || !col_idx || !Op) return PBS_ERR_NULL;
    if (!aligned16(Qp) || !aligned16(Kp) || !aligned16(Vt) || !aligned16(Op)) return PBS_ERR_SHAPE;
    const Geo g = make_geo(p);
    hipStream_t s = (hipStream_t)stream;
    const dim3 grid(g.T, g.batch * g.h_q);
    if (p->dtype == PBS_BF16 && p->d == 128 && (p->block == 128 || p->block == 64)) {
        if (p->block == 128)
            hipLaunchKernelGGL((attn_mfma_kernel<128, 2>), grid, dim3(128), 0, s, (const bf16_t *)Qp,
                               (const bf16_t *)Kp, (const bf16_t *)Vt, qidx, kidx, row_cnt, col_idx, (bf16_t *)Op, lse,
                               g);
        else
            hipLaunchKernelGGL((attn_mfma_kernel<64, 2>), grid, dim3(128), 0, s, (const bf16_t *)Qp,
                               (const bf16_t *)Kp, (const bf16_t *)Vt, qidx, kidx, row_cnt, col_idx, (bf16_t *)Op, lse,
                               g);
        return launch_status();
    }
    if (p->dtype == PBS_BF16)
        return p->d == 128 ? launch_vector<bf16_t, 128>(g, Qp, Kp, Vt, qidx, kidx, row_cnt, col_idx, Op, lse, s)
                           : launch_vector<bf16_t, 64>(g, Qp, Kp, Vt, qidx, kidx, row_cnt, col_idx, Op, lse, s);
    return p->d == 128 ? launch_vector<float, 128>(g, Qp, Kp, Vt, qidx, kidx, row_cnt, col_idx, Op, lse, s)
                       : launch_vector<float, 64>(g, Qp, Kp, Vt, qidx, kidx, row_cnt, col_idx, Op, lse, s);
}
