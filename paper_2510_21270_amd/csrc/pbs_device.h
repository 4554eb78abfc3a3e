// Device-side helpers shared by the PBS-Attn kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/pbs.h"

namespace pbs {

typedef __bf16 bf16_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t uintx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uintx2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

// Geometry derived from a pbs_problem, computed once on the host and passed by value to kernels.
struct Geo {
    int batch, h_q, h_kv, r, n, d, block, segment;
    int T;      // ceil(n / block)
    int R;      // blocks per segment
    int G;      // full segments
    float scale;
    double scale64; // the scale in the fp64 arithmetic that decides masks and fp32-input scores: the caller's float, or
                    // 1/sqrt(d) formed in double when the caller leaves the default (the two differ in the 8th digit)
    double tau;
    unsigned flags;
};

__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// number of key blocks the extended causal mask lets query block i see
__host__ __device__ inline int allowed_cols(int i, const Geo &g)
{
    int s = i / g.R;
    if (s < g.G) {
        int v = (s + 1) * g.R;
        return v < g.T ? v : g.T;
    }
    return i + 1;
}

// first key block of query block i whose entries need the token-level position test
__host__ __device__ inline int first_masked_col(int i, const Geo &g)
{
    int s = i / g.R;
    return s < g.G ? s * g.R : i;
}

// Vt stores every key block as groups of vt_group(block) consecutive key slots, each group transposed:
// element (group gi, feature e, key k of the group) of a block sits at ((gi * d + e) * vt_group + k).
__host__ __device__ inline int vt_group(int block) { return block < 32 ? block : 32; }

// The pooled keys are kept feature-major, [kv head][feature][kbar_stride(T)] fp64: the columns of one feature padded
// to a multiple of four, so that four neighbouring columns are two aligned 16-byte pieces.
__host__ __device__ inline int kbar_stride(int T) { return (T + 3) & ~3; }

template <typename T> struct ElemTraits;
template <> struct ElemTraits<float> {
    __device__ static inline float to_float(float v) { return v; }
    __device__ static inline float from_float(float v) { return v; }
};
template <> struct ElemTraits<bf16_t> {
    __device__ static inline float to_float(bf16_t v) { return (float)v; }
    __device__ static inline bf16_t from_float(float v) { return (bf16_t)v; }
};

__device__ inline float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ inline double wave_max(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ inline double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Sum over the wave without LDS traffic: butterflies inside each row of 16 lanes by DPP, then the four row totals
// through scalar registers.  Every lane receives the same value, formed in the same order.
__device__ inline double wave_sum_dpp(double v)
{
#define PBS_DPP_STEP(ctrl)                                                                      \
    {                                                                                           \
        const long long bits = __double_as_longlong(v);                                         \
        const int lo = __builtin_amdgcn_update_dpp(0, (int)bits, ctrl, 0xf, 0xf, false);        \
        const int hi = __builtin_amdgcn_update_dpp(0, (int)(bits >> 32), ctrl, 0xf, 0xf, false); \
        v += __longlong_as_double(((long long)hi << 32) | (unsigned)lo);                        \
    }
    PBS_DPP_STEP(0xB1)    // quad_perm [1,0,3,2]
    PBS_DPP_STEP(0x4E)    // quad_perm [2,3,0,1]
    PBS_DPP_STEP(0x141)   // row_half_mirror
    PBS_DPP_STEP(0x140)   // row_mirror
#undef PBS_DPP_STEP
    double rows[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const long long bits = __double_as_longlong(v);
        const int lo = __builtin_amdgcn_readlane((int)bits, 16 * r);
        const int hi = __builtin_amdgcn_readlane((int)(bits >> 32), 16 * r);
        rows[r] = __longlong_as_double(((long long)hi << 32) | (unsigned)lo);
    }
    return (rows[0] + rows[1]) + (rows[2] + rows[3]);
}

}  // namespace pbs
