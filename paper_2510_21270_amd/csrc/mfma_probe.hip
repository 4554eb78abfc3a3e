// Measurement aids for bench.py; the attention path does not use them.
//
// pbs_mfma_rate_probe: the matrix rate this GPU sustains on v_mfma_f32_32x32x16_bf16 alone -- four waves per SIMD,
// operands in registers, no memory traffic and no other instruction in the loop -- with all-zero or pseudo-random
// operands.  The instruction issues every 32 clocks either way (8 passes of 4); what changes is the clock the chip
// grants: about 2.4 GHz with zero operands, far less with operand bits that toggle, because the power the matrix units
// draw depends on them.  The rate with random operands, not the published peak, is therefore what a kernel that
// multiplies real data can approach.  sink[0..1] also receive the shader clock seen by one wave of the launch and its
// clocks per instruction (4 x 32 once all four waves of its SIMD are running).
//
// pbs_shader_clock_meter: one wave that watches the shader-clock counter against the constant 100 MHz counter for a
// given time; launched on a second stream beside a kernel under test it reports the clock that kernel runs at.
#include "pbs_host.h"

namespace pbs {
namespace {

constexpr int kProbeGroups = 1024, kProbeThreads = 256, kProbeMfmas = 32;

__global__ __launch_bounds__(kProbeThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void mfma_probe_kernel(
    float *__restrict__ sink, int iters, int random_operands)
{
    floatx16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
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
    const unsigned long long c0 = __builtin_readcyclecounter(), r0 = wall_clock64();
    // nothing but matrix instructions: a vector instruction that rewrites an operand costs several of the 32 clocks
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < kProbeMfmas; ++m)
            acc[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m & 7], b[(m >> 2) & 7], acc[m & 3], 0, 0, 0);
    }
    const unsigned long long c1 = __builtin_readcyclecounter(), r1 = wall_clock64();
    float t = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int x = 0; x < 16; ++x) t += acc[i][x];
    const unsigned id = blockIdx.x * kProbeThreads + threadIdx.x;
    const float mhz = (float)((double)(c1 - c0) / ((double)(r1 - r0) / 100.0));             // shader clock
    const float cpi = (float)((double)(c1 - c0) / ((double)iters * kProbeMfmas));   // clocks per instruction of this wave
    sink[id] = id == 0 ? mhz : (id == 1 ? cpi : t);          // the first wave reports what it saw in its own two slots
}

// out[0] = shader clock in MHz averaged over about `micros` microseconds, out[1] = microseconds actually watched
__global__ __launch_bounds__(64) void shader_clock_meter_kernel(float *__restrict__ out, int micros)
{
    const unsigned long long r0 = wall_clock64(), c0 = __builtin_readcyclecounter();
    unsigned long long r1 = r0, c1 = c0;
    const unsigned long long want = (unsigned long long)micros * 100ull;       // the constant counter runs at 100 MHz
    for (int spin = 0; spin < (1 << 26) && r1 - r0 < want; ++spin) {           // bounded: ends even if the counter stalls
        __builtin_amdgcn_s_sleep(32);
        r1 = wall_clock64();
        c1 = __builtin_readcyclecounter();
    }
    if (threadIdx.x == 0) {
        out[0] = r1 > r0 ? (float)((double)(c1 - c0) / ((double)(r1 - r0) / 100.0)) : 0.0f;
        out[1] = (float)((double)(r1 - r0) / 100.0);
    }
}

}  // namespace
}  // namespace pbs

extern "C" pbs_status pbs_mfma_rate_probe(int random_operands, int iters, float *sink, size_t sink_floats, double *flop,
                                          void *stream)
{
    using namespace pbs;
    if (!sink || !flop) return PBS_ERR_NULL;
    if (iters < 1 || iters > (1 << 22) || sink_floats < (size_t)kProbeGroups * kProbeThreads) return PBS_ERR_SHAPE;
    const pbs_status st = launch(mfma_probe_kernel, dim3(kProbeGroups), dim3(kProbeThreads), 0, (hipStream_t)stream, sink,
                                 iters, random_operands);
    *flop = (double)kProbeGroups * (kProbeThreads / kWave) * (double)iters * kProbeMfmas * (2.0 * 32 * 32 * 16);
    return st;
}

extern "C" pbs_status pbs_shader_clock_meter(float *out, int micros, void *stream)
{
    using namespace pbs;
    if (!out) return PBS_ERR_NULL;
    if (micros < 1 || micros > 2000000) return PBS_ERR_SHAPE;
    return launch(shader_clock_meter_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, out, micros);
}
