// Host-side validation and geometry shared by the C-ABI entry points.
#pragma once
#include <math.h>

#include <atomic>
#include <tuple>
#include <type_traits>

#include "pbs_device.h"

namespace pbs {

constexpr int kMaxSegment = 4096;
constexpr int kMaxT = 4096;
constexpr size_t kWsAlign = 256;

inline size_t elem_size(int dtype) { return dtype == PBS_BF16 ? 2 : 4; }

inline pbs_status validate(const pbs_problem *p)
{
    if (!p) return PBS_ERR_NULL;
    if (p->batch < 1 || p->h_q < 1 || p->h_kv < 1 || p->n < 1 || p->d < 1 || p->block < 1 || p->segment < 1)
        return PBS_ERR_SHAPE;
    if (p->h_q % p->h_kv != 0 || p->segment % p->block != 0) return PBS_ERR_SHAPE;
    if (!(p->tau == p->tau) || !(p->scale == p->scale) || p->scale < 0.0f || isinf(p->scale)) return PBS_ERR_SHAPE;
    if (p->dtype != PBS_F32 && p->dtype != PBS_BF16) return PBS_ERR_UNSUPPORTED;
    if (p->d != 64 && p->d != 128) return PBS_ERR_UNSUPPORTED;
    if (p->block != 16 && p->block != 32 && p->block != 64 && p->block != 128) return PBS_ERR_UNSUPPORTED;
    if (p->segment > kMaxSegment) return PBS_ERR_UNSUPPORTED;
    if ((p->n + p->block - 1) / p->block > kMaxT) return PBS_ERR_UNSUPPORTED;
    // every tensor is indexed with 64-bit offsets, but row counts must fit an int
    if ((long long)p->batch * p->h_q * (long long)p->n > 0x7fffffffLL) return PBS_ERR_UNSUPPORTED;
    if ((long long)p->batch * p->h_q > 65535) return PBS_ERR_UNSUPPORTED;   // heads ride on gridDim.y
    return PBS_OK;
}

inline Geo make_geo(const pbs_problem *p)
{
    Geo g;
    g.batch = p->batch; g.h_q = p->h_q; g.h_kv = p->h_kv; g.r = p->h_q / p->h_kv;
    g.n = p->n; g.d = p->d; g.block = p->block; g.segment = p->segment;
    g.T = (p->n + p->block - 1) / p->block;
    g.R = p->segment / p->block;
    g.G = p->n / p->segment;
    g.scale = p->scale > 0.0f ? p->scale : (float)(1.0 / sqrt((double)p->d));
    g.scale64 = p->scale > 0.0f ? (double)p->scale : 1.0 / sqrt((double)p->d);
    g.tau = (double)p->tau;
    g.flags = p->flags;
    return g;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline bool aligned16(const void *ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15u) == 0; }

inline pbs_status check_ws(const pbs_problem *p, int stage, const void *ws, size_t ws_bytes)
{
    size_t need = pbs_workspace_bytes(p, stage);
    if (need == 0) return PBS_OK;
    if (!ws) return PBS_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(ws) & (kWsAlign - 1)) != 0 || ws_bytes < need) return PBS_ERR_WORKSPACE;
    return PBS_OK;
}

// Enqueues `kernel` and returns the status of this very launch (the return value of hipLaunchKernel), so that an
// error left behind by some earlier, unrelated runtime call is neither reported as ours nor cleared.  The arguments
// are converted to the kernel's parameter types first.
template <typename... Params, typename... Args>
inline pbs_status launch(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds, hipStream_t s, Args &&...args)
{
    static_assert(sizeof...(Params) == sizeof...(Args), "one argument per kernel parameter");
    std::tuple<typename std::remove_cv<Params>::type...> vals{static_cast<Params>(args)...};
    return std::apply(
        [&](auto &...v) {
            void *ptrs[] = {static_cast<void *>(&v)...};
            return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, lds, s) == hipSuccess
                       ? PBS_OK : PBS_ERR_HIP;
        },
        vals);
}

// Raises a kernel's dynamic LDS limit once per device (the attribute belongs to the current device's copy of the
// kernel).  `done` is a bit per device ordinal, one such word per kernel; devices beyond 63 set it on every call.
inline pbs_status raise_lds_limit(const void *kernel, int bytes, std::atomic<unsigned long long> &done)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return PBS_ERR_HIP;
    const bool tracked = dev >= 0 && dev < 64;
    if (tracked && ((done.load(std::memory_order_acquire) >> dev) & 1ull)) return PBS_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return PBS_ERR_HIP;
    if (tracked) done.fetch_or(1ull << dev, std::memory_order_release);
    return PBS_OK;
}

}  // namespace pbs
