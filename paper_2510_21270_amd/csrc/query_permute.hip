// pbs_query_permutation: the key-aware query permutation of Section "Design Choice: Why Permute Keys but not
// Queries?" -- an ablation of the paper (its main setting keeps the queries in place).
//
//   centroids   Kbar_j = block means of the given keys (pool_kernel, fp64, row-major)
//   rinv_j      = 1 / sqrt(sum_e Kbar_j[e]^2), 0 for a zero centroid                       (centroid_rnorm_kernel)
//   c*(t)       = argmax over the centroids j a query's segment may attend to, j < (g+1) R capped at T, of
//                 u_j = (q_t . Kbar_j) * rinv_j, i.e. of the cosine similarity (|q_t| does not depend on j),
//                 ties to the lowest j                                                      (assign_kernel)
//   sigma       inside every full segment the queries in ascending order of c*, equal c* in original order; the
//                 tail keeps its place                                                      (segment sort, permute.hip)
//
// The decision is an argmax of fp64 values, so every sum runs over the features in ascending order with separate
// multiplications and additions (no contraction into fused multiply-adds anywhere in this file): the plain
// definition evaluated the plain way, which a CPU reproduces bit for bit.
#include "pbs_host.h"

#pragma clang fp contract(off)

namespace pbs {

pbs_status launch_pool_keys_rowmajor(const pbs_problem *p, const Geo &g, const void *K, double *Kbar, hipStream_t s);
pbs_status launch_segment_sort_by_int_key(const Geo &g, int heads, const int32_t *keys, int32_t *idx, hipStream_t s);

// one thread per centroid
__global__ __launch_bounds__(256) void centroid_rnorm_kernel(const double *__restrict__ Kbar, double *__restrict__ rinv,
                                                             int total, int d)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= total) return;
    const double *kb = Kbar + (size_t)c * d;
    double nsq = 0.0;
    for (int e = 0; e < d; ++e) nsq = nsq + kb[e] * kb[e];
    rinv[c] = nsq > 0.0 ? 1.0 / sqrt(nsq) : 0.0;
}

// One thread per query of the full segments.  The query's D features stay in registers in their storage type (exact
// in fp64 for both); the centroid rows are read at wave-uniform addresses, so they arrive in scalar registers and cost
// no vector instruction.  What costs is the f32 -> f64 conversion of a query value, a quarter-rate instruction beside
// the full-rate multiplication and addition of a term, so a value is converted once per 32 features x 16 centroids:
// sixteen dot products advance together, each over the features in ascending order, one term (one multiplication,
// one addition) at a time as the definition has it.  grid = (ceil(G * S / 256), batch * h_q).
template <typename E, int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 2))) void assign_kernel(const E *__restrict__ Q, const double *__restrict__ Kbar,
                                                     const double *__restrict__ rinv, int32_t *__restrict__ cstar, Geo g)
{
    constexpr int C = 16;                                    // centroids per tile
    constexpr int FB = sizeof(E) == 2 ? 32 : 16;             // features per conversion (fp32 rows take twice the registers)
    constexpr int VEC = 16 / sizeof(E);
    typedef E vec_t __attribute__((ext_vector_type(VEC)));
    const int bhq = blockIdx.y;
    const int b = bhq / g.h_q, hk = (bhq % g.h_q) / g.r;
    const int pos0 = blockIdx.x * 256;
    const int full = g.G * g.segment;
    const int pos = pos0 + threadIdx.x;
    const bool live = pos < full;
    const int pc = live ? pos : full - 1;
    vec_t q[D / VEC];
    const vec_t *qr = reinterpret_cast<const vec_t *>(Q + ((size_t)bhq * g.n + pc) * D);
#pragma unroll
    for (int e = 0; e < D / VEC; ++e) q[e] = qr[e];
    auto ncand_of = [&](int p) { const int v = (p / g.segment + 1) * g.R; return v < g.T ? v : g.T; };
    const int mine = ncand_of(pc);
    const int most = ncand_of(min(pos0 + 255, full - 1));    // uniform: the workgroup's last query sees the most
    const double *kb = Kbar + (size_t)(b * g.h_kv + hk) * g.T * D;
    const double *ri = rinv + (size_t)(b * g.h_kv + hk) * g.T;
    int best = 0;
    double ubest = 0.0;
#pragma unroll 1
    for (int j0 = 0; j0 < most; j0 += C) {
        double dot[C];
#pragma unroll
        for (int c = 0; c < C; ++c) dot[c] = 0.0;
        // (opaque to the compiler: otherwise all D conversions are done once ahead of this loop and the query takes
        // 2 * D registers as doubles)
#pragma unroll
        for (int e = 0; e < D / VEC; ++e) asm volatile("" : "+v"(q[e]));
        // The tile as a flat sequence of steps s = (feature block, centroid, half of the block): 16 terms of one dot
        // product each.  The 16 centroid values of step s + 1 are requested (two scalar loads) before the terms of
        // step s are computed and waited for after them.
        constexpr int HB = FB / 2, STEPS = (D / FB) * C * 2;
        auto fetch = [&](double (&k)[HB], int s_, int j0_) {
            const int e0 = (s_ / (2 * C)) * FB, c = (s_ % (2 * C)) / 2, h = s_ % 2;
            // (rows past the last candidate are the last centroid's again; their results are never looked at)
            const double *src = kb + (size_t)min(j0_ + c, g.T - 1) * D + e0 + h * HB;
#pragma unroll
            for (int e = 0; e < HB; ++e) k[e] = src[e];
        };
        double qd[FB];
        auto terms = [&](const double (&k)[HB], int s_) {
            const int c = (s_ % (2 * C)) / 2, h = s_ % 2;
#pragma unroll
            for (int e = 0; e < HB; ++e) dot[c] = dot[c] + qd[h * HB + e] * k[e];
        };
        // a use of the values: the wait for them is placed here, before the other buffer's loads are issued
        // (after them it would wait for those as well)
        auto arrived = [&](const double (&k)[HB]) {
            asm volatile("" ::"s"(k[0]), "s"(k[HB - 1]));
            __builtin_amdgcn_sched_barrier(0);
        };
        double ka[HB], kc[HB];
        fetch(ka, 0, j0);
#pragma unroll
        for (int s_ = 0; s_ < STEPS; s_ += 2) {
            if (s_ % (2 * C) == 0) {
                const int e0 = (s_ / (2 * C)) * FB;
#pragma unroll
                for (int e = 0; e < FB; ++e) qd[e] = (double)ElemTraits<E>::to_float(q[(e0 + e) / VEC][(e0 + e) % VEC]);
            }
            arrived(ka);
            fetch(kc, s_ + 1, j0);
            __builtin_amdgcn_sched_barrier(0);
            terms(ka, s_);
            __builtin_amdgcn_sched_barrier(0);
            arrived(kc);
            if (s_ + 2 < STEPS) fetch(ka, s_ + 2, j0);
            __builtin_amdgcn_sched_barrier(0);
            terms(kc, s_ + 1);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const int j = j0 + c;
            const double u = dot[c] * ri[min(j, g.T - 1)];
            if (j < mine && (j == 0 || u > ubest)) { ubest = u; best = j; }
        }
    }
    if (live) cstar[(size_t)bhq * g.n + pos] = best;
}

size_t ws_query_permute(const pbs_problem *p)
{
    const Geo g = make_geo(p);
    const size_t nbk = (size_t)g.batch * g.h_kv;
    return align_up(nbk * g.T * g.d * sizeof(double), kWsAlign) + align_up(nbk * g.T * sizeof(double), kWsAlign) +
           align_up((size_t)g.batch * g.h_q * g.n * sizeof(int32_t), kWsAlign);
}

}  // namespace pbs

using namespace pbs;

extern "C" pbs_status pbs_query_permutation(const pbs_problem *p, const void *Q, const void *Kc, int32_t *qidx, void *ws,
                                            size_t ws_bytes, void *stream)
{
    pbs_status st = validate(p);
    if (st != PBS_OK) return st;
    if (!Q || !Kc || !qidx) return PBS_ERR_NULL;
    if (!aligned16(Q) || !aligned16(Kc)) return PBS_ERR_SHAPE;
    if ((st = check_ws(p, PBS_STAGE_QUERY_PERMUTE, ws, ws_bytes)) != PBS_OK) return st;
    const Geo g = make_geo(p);
    hipStream_t s = (hipStream_t)stream;
    const size_t nbk = (size_t)g.batch * g.h_kv;
    char *w = reinterpret_cast<char *>(ws);
    double *Kbar = reinterpret_cast<double *>(w);
    w += align_up(nbk * g.T * g.d * sizeof(double), kWsAlign);
    double *rinv = reinterpret_cast<double *>(w);
    w += align_up(nbk * g.T * sizeof(double), kWsAlign);
    int32_t *cstar = reinterpret_cast<int32_t *>(w);
    const int heads = g.batch * g.h_q;
    if (g.G > 0) {
        if ((st = launch_pool_keys_rowmajor(p, g, Kc, Kbar, s)) != PBS_OK) return st;
        const int total = (int)(nbk * g.T);
        if ((st = launch(centroid_rnorm_kernel, dim3((total + 255) / 256), dim3(256), 0, s, (const double *)Kbar, rinv, total,
                         g.d)) != PBS_OK) return st;
        const dim3 grid((g.G * g.segment + 255) / 256, heads);
        if (p->dtype == PBS_BF16) {
            st = g.d == 128 ? launch((assign_kernel<bf16_t, 128>), grid, dim3(256), 0, s, (const bf16_t *)Q,
                                     (const double *)Kbar, (const double *)rinv, cstar, g)
                            : launch((assign_kernel<bf16_t, 64>), grid, dim3(256), 0, s, (const bf16_t *)Q,
                                     (const double *)Kbar, (const double *)rinv, cstar, g);
        } else {
            st = g.d == 128 ? launch((assign_kernel<float, 128>), grid, dim3(256), 0, s, (const float *)Q,
                                     (const double *)Kbar, (const double *)rinv, cstar, g)
                            : launch((assign_kernel<float, 64>), grid, dim3(256), 0, s, (const float *)Q,
                                     (const double *)Kbar, (const double *)rinv, cstar, g);
        }
        if (st != PBS_OK) return st;
    }
    // ascending by assigned centroid inside every full segment (stable), identity in the tail
    return launch_segment_sort_by_int_key(g, heads, cstar, qidx, s);
}
