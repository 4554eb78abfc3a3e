// pbs_mfma_rate_probe: the matrix rate this GPU sustains on v_mfma_f32_32x32x16_bf16 alone -- one wave per SIMD,
// operands in registers, no memory traffic -- with all-zero or pseudo-random operands.  The chip lowers its clock under
// the power the matrix units draw, and that power depends on the operand bits, so the rate with random operands
// (not the published peak) is what a kernel with real data can approach.  A measurement aid for bench.py; the
// attention path does not use it.
#include "pbs_host.h"

namespace pbs {
namespace {

constexpr int kProbeGroups = 512, kProbeThreads = 128, kProbeMfmas = 32;

__global__ __launch_bounds__(kProbeThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void mfma_probe_kernel(
    float *__restrict__ sink, int iters, int random_operands)
{
    floatx16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int x = 0; x < 16; ++x) acc[i][x] = 0.0f;
    bf16x8 a[8], b[8];
    unsigned h = (blockIdx.x * kProbeThreads + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            h = h * 1664525u + 1013904223u;
            const float ra = ((h >> 8) & 0xffff) / 65536.0f - 0.5f;
            h = h * 1664525u + 1013904223u;
            const float rb = ((h >> 8) & 0xffff) / 65536.0f - 0.5f;
            a[s][x] = (bf16_t)(random_operands ? ra : 0.0f);
            b[s][x] = (bf16_t)(random_operands ? rb : 0.0f);
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < kProbeMfmas; ++m)
            acc[m & 7] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m & 7], b[(m >> 2) & 7], acc[m & 7], 0, 0, 0);
        // one operand changes sign every iteration, so the accumulators stay small
#pragma unroll
        for (int s = 0; s < 8; ++s)
#pragma unroll
            for (int x = 0; x < 8; ++x) a[s][x] = -a[s][x];
    }
    float t = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int x = 0; x < 16; ++x) t += acc[i][x];
    sink[blockIdx.x * kProbeThreads + threadIdx.x] = t;
}

}  // namespace
}  // namespace pbs

extern "C" pbs_status pbs_mfma_rate_probe(int random_operands, int iters, float *sink, size_t sink_floats, double *flop,
                                          void *stream)
{
    using namespace pbs;
    if (!sink || !flop) return PBS_ERR_NULL;
    if (iters < 1 || iters > (1 << 22) || sink_floats < (size_t)kProbeGroups * kProbeThreads) return PBS_ERR_SHAPE;
    const pbs_status st = launch(mfma_probe_kernel, dim3(kProbeGroups), dim3(kProbeThreads), 0, (hipStream_t)stream, sink, iters,
                       random_operands);
    *flop = (double)kProbeGroups * (kProbeThreads / kWave) * (double)iters * kProbeMfmas * (2.0 * 32 * 32 * 16);
    return st;
}
