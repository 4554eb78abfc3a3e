// Coverage tooling for the block-selection objective of Section "The Problem of Information Fragmentation": the
// attention mass (softmax over every visible key) that falls into the blocks a list names.  Two small kernels; the
// log-sum-exp values they combine come from two pbs_attn_fwd calls.
#include "pbs_host.h"

namespace pbs {

// row_cnt[bh][i] = number of key blocks the extended causal mask admits for query block i, col_idx[bh][i][0..] = 0, 1, ...
// grid = (T, batch * h_q)
__global__ __launch_bounds__(256) void admitted_lists_kernel(int32_t *__restrict__ row_cnt, int32_t *__restrict__ col_idx,
                                                             Geo g)
{
    const int i = blockIdx.x;
    const size_t row = (size_t)blockIdx.y * g.T + i;
    const int ni = allowed_cols(i, g);
    if (threadIdx.x == 0) row_cnt[row] = ni;
    for (int j = threadIdx.x; j < ni; j += blockDim.x) col_idx[row * g.T + j] = j;
}

// covered = exp(lse_listed - lse_admitted); a query that sees nothing in the listed blocks (-inf) covers 0
__global__ __launch_bounds__(256) void mass_covered_kernel(const float *__restrict__ lse_listed,
                                                           const float *__restrict__ lse_admitted,
                                                           float *__restrict__ covered, size_t total)
{
    for (size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (size_t)gridDim.x * blockDim.x) {
        const float a = lse_listed[t], b = lse_admitted[t];
        covered[t] = (a == -INFINITY || !(b > -INFINITY)) ? 0.0f : expf(a - b);
    }
}

}  // namespace pbs

using namespace pbs;

extern "C" pbs_status pbs_admitted_lists(const pbs_problem *p, int32_t *row_cnt, int32_t *col_idx, void *stream)
{
    pbs_status st = validate(p);
    if (st != PBS_OK) return st;
    if (!row_cnt || !col_idx) return PBS_ERR_NULL;
    const Geo g = make_geo(p);
    return launch(admitted_lists_kernel, dim3(g.T, g.batch * g.h_q), dim3(256), 0, (hipStream_t)stream, row_cnt, col_idx, g);
}

extern "C" pbs_status pbs_mass_covered(const pbs_problem *p, const float *lse_listed, const float *lse_admitted,
                                       float *covered, void *stream)
{
    pbs_status st = validate(p);
    if (st != PBS_OK) return st;
    if (!lse_listed || !lse_admitted || !covered) return PBS_ERR_NULL;
    const size_t total = (size_t)p->batch * p->h_q * p->n;
    size_t blocks = (total + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    return launch(mass_covered_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, lse_listed, lse_admitted,
                  covered, total);
}
