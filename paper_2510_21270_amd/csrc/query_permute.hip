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

// One thread per query of the full segments: the query's D features stay in registers as fp32 (exact for both storage
// types), the centroid rows are read at wave-uniform addresses.  grid = (ceil(G * S / 256), batch * h_q).
template <typename E, int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 2))) void assign_kernel(const E *__restrict__ Q, const double *__restrict__ Kbar,
                                                     const double *__restrict__ rinv, int32_t *__restrict__ cstar, Geo g)
{
    const int bhq = blockIdx.y;
    const int b = bhq / g.h_q, hk = (bhq % g.h_q) / g.r;
    const int pos0 = blockIdx.x * 256;
    const int full = g.G * g.segment;
    const int pos = pos0 + threadIdx.x;
    const bool live = pos < full;
    const int pc = live ? pos : full - 1;
    float q[D];
    const E *qr = Q + ((size_t)bhq * g.n + pc) * D;
#pragma unroll
    for (int e = 0; e < D; ++e) q[e] = ElemTraits<E>::to_float(qr[e]);
    auto ncand_of = [&](int p) { const int v = (p / g.segment + 1) * g.R; return v < g.T ? v : g.T; };
    const int mine = ncand_of(pc);
    const int most = ncand_of(min(pos0 + 255, full - 1));    // uniform: the workgroup's last query sees the most
    const double *kb = Kbar + (size_t)(b * g.h_kv + hk) * g.T * D;
    const double *ri = rinv + (size_t)(b * g.h_kv + hk) * g.T;
    int best = 0;
    double ubest = 0.0;
    for (int j = 0; j < most; ++j) {
        const double *kj = kb + (size_t)j * D;
        double dot = 0.0;
#pragma unroll
        for (int e = 0; e < D; ++e) dot = dot + (double)q[e] * kj[e];
        const double u = dot * ri[j];
        if (j < mine && (j == 0 || u > ubest)) { ubest = u; best = j; }
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
